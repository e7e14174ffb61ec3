"""The GPU fill kernels and the torch generators produce the same bytes as the numpy ones."""
import numpy as np
import pytest
import torch

from paper_2510_00554_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("backend", [None, "torch"])
def test_uniform_bytes_on_gpu(backend):
    for start, n in ((0, 4096), (3, 77), (5, 8), (13, 100_003), ((1 << 33) + 1, 5000), (8, 1), (7, 0)):
        want = wl.uniform_bytes(7, start, n)
        got = wl.uniform_bytes(7, start, n, device="cuda", backend=backend).cpu().numpy()
        assert (got == want).all(), (backend, start, n)
    # into a slice whose address is not 8-byte aligned
    buf = torch.zeros(1000, dtype=torch.uint8, device="cuda")
    wl.uniform_bytes(9, 10, 900, device="cuda", out=buf[3:903], backend=backend)
    assert (buf[3:903].cpu().numpy() == wl.uniform_bytes(9, 10, 900)).all()
    assert not buf[:3].any() and not buf[903:].any()


@pytest.mark.parametrize("backend", [None, "torch"])
def test_normal_bf16_on_gpu(backend):
    for e0, n in ((0, 100_000), (12345, 7), ((1 << 32) + 5, 70_001)):
        want = wl.normal_bf16_bits(11, e0, n)
        got = wl.normal_bf16_bits(11, e0, n, device="cuda", backend=backend).cpu().numpy().view(np.uint16)
        assert (got == want).all(), (backend, e0, n)


def test_checkpoint_flat_on_gpu():
    lay = wl.layout_tiny()
    buf, offs = wl.checkpoint_flat_torch(lay, "cuda")
    flat = np.concatenate(wl.checkpoint_bytes_np(lay))
    assert (buf.cpu().numpy() == flat).all()


def test_uniform_bytes_past_4gib_unaligned():
    # more than 2^32 bytes from an odd stream offset: the byte-wise path must stride
    n = (1 << 32) + 12345
    buf = wl.uniform_bytes(21, 3, n, device="cuda")
    for pos in (0, (1 << 32) - 100, (1 << 32) + 100, n - 50):
        assert (buf[pos:pos + 50].cpu().numpy() == wl.uniform_bytes(21, 3 + pos, 50)).all(), pos

"""GPU parity: Merkle trees over BLAKE2b-512 and SHA3-256 against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import to_dev

pytestmark = pytest.mark.gpu

HASHES = [(sentry.HASH_BLAKE2B, 64), (sentry.HASH_SHA3_256, 32), (sentry.HASH_SHA256, 32)]


def gpu_root_h(hid, dl, buf, leaf):
    d = to_dev(buf) if buf.size else torch.empty(16, dtype=torch.uint8, device="cuda")
    out = torch.zeros(80, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_root_h(hid, d.data_ptr() if buf.size else 0, buf.size, leaf, out.data_ptr())
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert not o[dl:].any()
    if buf.size:
        assert (d.cpu().numpy() == buf).all()
    return bytes(o[:dl])


@pytest.mark.parametrize("hid,dl", HASHES)
@pytest.mark.parametrize("leaf", [64, 192, 4096])
def test_edge_lengths(hid, dl, leaf):
    for n in (0, 1, 7, 8, 63, 64, 65, 127, 128, 129, 135, 136, 137, 271, 272, 273, leaf - 1, leaf, leaf + 1,
              2 * leaf, 2 * leaf + 57, 3 * leaf, 5 * leaf - 8):
        buf = wl.uniform_bytes(4000 + leaf + hid, 0, n)
        assert gpu_root_h(hid, dl, buf, leaf) == oracle.merkle_root_h(hid, buf, leaf), (hid, leaf, n)


@pytest.mark.parametrize("hid,dl", HASHES[:2])
@pytest.mark.parametrize("n_leaves", [2, 3, 255, 256, 257, 511, 512, 513, 1025, 512 * 512 + 3])
def test_leaf_counts(hid, dl, n_leaves):
    for tail in (0, 17):
        size = 64 * n_leaves - (64 - tail if tail else 0)
        buf = wl.uniform_bytes(4100, 0, size)
        assert gpu_root_h(hid, dl, buf, 64) == oracle.merkle_root_h(hid, buf, 64), (hid, n_leaves, tail)


@pytest.mark.parametrize("hid,dl", HASHES[:2])
def test_config1_shape_and_paper_default_block(hid, dl):
    buf = wl.uniform_bytes(wl.SEED_C1, 0, 16 << 20)
    for leaf in (4096, 8192):
        assert gpu_root_h(hid, dl, buf, leaf) == oracle.merkle_root_h(hid, buf, leaf)


def test_unknown_hash_and_unaligned_output():
    buf = wl.uniform_bytes(4200, 0, 1000)
    d = to_dev(buf)
    out = torch.zeros(70, dtype=torch.uint8, device="cuda")
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_root_h(7, d.data_ptr(), 1000, 64, out.data_ptr())
    sentry.sentry_merkle_root_h(sentry.HASH_BLAKE2B, d.data_ptr(), 1000, 64, out.data_ptr() + 3)
    torch.cuda.synchronize()
    assert bytes(out[3:67].cpu().numpy()) == oracle.merkle_root_h(oracle.HASH_BLAKE2B, buf, 64)

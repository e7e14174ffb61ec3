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


def gpu_segments_h(hid, dl, segs, leaf, want_roots=True):
    devs = [to_dev(s) if s.size else None for s in segs]
    ptrs = [d.data_ptr() if d is not None else 0 for d in devs]
    lens = [int(s.size) for s in segs]
    n = len(segs)
    roots = torch.zeros(dl * n + 16, dtype=torch.uint8, device="cuda")
    top = torch.zeros(80, dtype=torch.uint8, device="cuda")
    flat = torch.zeros(80, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_segments_h(hid, ptrs, lens, leaf, roots.data_ptr() if want_roots else 0, top.data_ptr())
    sentry.sentry_merkle_inplace_h(hid, ptrs, lens, leaf, flat.data_ptr())
    torch.cuda.synchronize()
    r, t, f = roots.cpu().numpy(), top.cpu().numpy(), flat.cpu().numpy()
    assert not r[dl * n:].any() and not t[dl:].any() and not f[dl:].any()
    for d, s in zip(devs, segs):
        if d is not None:
            assert (d.cpu().numpy() == s).all()
    return [bytes(r[dl * i:dl * (i + 1)]) for i in range(n)], bytes(t[:dl]), bytes(f[:dl])


@pytest.mark.parametrize("hid,dl", HASHES)
def test_per_tensor_and_flat_trees_small_and_edge(hid, dl):
    L = 128
    rng = np.random.default_rng(4300 + hid)
    for k, sizes in enumerate(([1], [0], [L], [L + 1, 0, 3 * L, 5], [0, 0], [7 * L - 1, L, 2 * L + 9, 0, 64, 33 * L],
                               [int(x) for x in rng.integers(0, 6 * L, size=40)])):
        segs = [wl.uniform_bytes(4310 + 7 * k + i, 0, n) for i, n in enumerate(sizes)]
        roots, top, flat = gpu_segments_h(hid, dl, segs, L)
        want_roots, want_top = oracle.merkle_segments_h(hid, segs, L)
        assert roots == want_roots and top == want_top, (hid, sizes)
        assert flat == oracle.merkle_inplace_h(hid, segs, L), (hid, sizes)


@pytest.mark.parametrize("hid,dl", HASHES[:2])
def test_per_tensor_trees_with_several_reduce_levels(hid, dl):
    # 64-byte leaves: tensors of 1, 511..513 and 512*512+3 leaves need zero to three reduce levels
    # in one table-driven call; more than 512 tensors make the tree over the roots two levels deep
    L = 64
    sizes = [64 * (512 * 512 + 3) - 9, 64, 64 * 511, 64 * 512, 64 * 513 - 1, 0, 64 * 1025] + [64 * (1 + i % 5) for i in range(600)]
    segs = [wl.uniform_bytes(4400 + i, 0, n) for i, n in enumerate(sizes)]
    roots, top, flat = gpu_segments_h(hid, dl, segs, L)
    want_roots, want_top = oracle.merkle_segments_h(hid, segs, L)
    assert roots == want_roots
    assert top == want_top
    assert flat == oracle.merkle_inplace_h(hid, segs, L)
    _, top2, _ = gpu_segments_h(hid, dl, segs, L, want_roots=False)
    assert top2 == want_top


@pytest.mark.parametrize("hid,dl", HASHES[:2])
def test_tiny_checkpoint_layout_paper_default_block(hid, dl):
    tensors = wl.checkpoint_bytes_np(wl.layout_tiny())
    roots, top, flat = gpu_segments_h(hid, dl, tensors, 8192)
    want_roots, want_top = oracle.merkle_segments_h(hid, tensors, 8192)
    assert roots == want_roots and top == want_top
    assert flat == oracle.merkle_inplace_h(hid, tensors, 8192)
    # whole blocks only: the flat tree equals the tree over the concatenated tensors
    whole = [t[:t.size - t.size % 8192] for t in tensors if t.size >= 8192]
    _, _, flat_whole = gpu_segments_h(hid, dl, whole, 8192)
    assert flat_whole == oracle.merkle_root_h(hid, np.concatenate(whole), 8192)

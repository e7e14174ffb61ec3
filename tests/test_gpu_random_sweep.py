"""GPU parity on seeded random shapes: every entry point against the oracle on inputs whose
segment counts, lengths, leaf sizes, record mixes and source counts are drawn at random (fixed
seeds), to reach combinations the hand-picked cases do not list."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import to_dev

pytestmark = pytest.mark.gpu

HASHES = [(sentry.HASH_SHA256, 32), (sentry.HASH_BLAKE2B, 64), (sentry.HASH_SHA3_256, 32)]


def random_lengths(rng, n, leaf):
    kinds = rng.integers(0, 5, size=n)
    out = []
    for k in kinds:
        if k == 0:
            out.append(0)
        elif k == 1:
            out.append(int(rng.integers(1, leaf)))                       # shorter than a leaf
        elif k == 2:
            out.append(int(leaf * rng.integers(1, 70)))                  # whole leaves
        elif k == 3:
            out.append(int(leaf * rng.integers(1, 70) + rng.integers(1, leaf)))
        else:
            out.append(int(rng.integers(0, 300_000)))
    return out


@pytest.mark.parametrize("seed", range(12))
def test_trees_over_random_tensor_lists(seed):
    rng = np.random.default_rng(7000 + seed)
    leaf = int(rng.choice([64, 192, 1024, 4096, 8192]))
    n_seg = int(rng.integers(1, 40))
    sizes = random_lengths(rng, n_seg, leaf)
    segs = [wl.uniform_bytes(7100 + 50 * seed + i, 0, n) for i, n in enumerate(sizes)]
    devs = [to_dev(s) if s.size else None for s in segs]
    ptrs = [d.data_ptr() if d is not None else 0 for d in devs]
    lens = [int(s.size) for s in segs]
    whole = np.concatenate(segs) if sum(lens) else np.zeros(0, np.uint8)
    dwhole = to_dev(whole) if whole.size else None
    for hid, dl in HASHES:
        roots = torch.zeros(dl * n_seg, dtype=torch.uint8, device="cuda")
        top = torch.zeros(64, dtype=torch.uint8, device="cuda")
        flat = torch.zeros(64, dtype=torch.uint8, device="cuda")
        one = torch.zeros(64, dtype=torch.uint8, device="cuda")
        sentry.sentry_merkle_segments_h(hid, ptrs, lens, leaf, roots.data_ptr(), top.data_ptr())
        sentry.sentry_merkle_inplace_h(hid, ptrs, lens, leaf, flat.data_ptr())
        sentry.sentry_merkle_root_h(hid, dwhole.data_ptr() if dwhole is not None else 0, whole.size, leaf, one.data_ptr())
        torch.cuda.synchronize()
        want_roots, want_top = oracle.merkle_segments_h(hid, segs, leaf)
        r = roots.cpu().numpy()
        assert [bytes(r[dl * i:dl * (i + 1)]) for i in range(n_seg)] == want_roots, (seed, hid, leaf, sizes)
        assert bytes(top.cpu().numpy()[:dl]) == want_top, (seed, hid, leaf, sizes)
        assert bytes(flat.cpu().numpy()[:dl]) == oracle.merkle_inplace_h(hid, segs, leaf), (seed, hid, leaf, sizes)
        assert bytes(one.cpu().numpy()[:dl]) == oracle.merkle_root_h(hid, whole, leaf), (seed, hid, leaf)
    # the model lattice hash over the same tensors (block = leaf, a multiple of 16)
    layers = torch.zeros(32 * n_seg, dtype=torch.int16, device="cuda")
    total = torch.zeros(32, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_model(ptrs, lens, leaf, layers.data_ptr(), total.data_ptr())
    torch.cuda.synchronize()
    want_layers, want_total = oracle.lthash_model(segs, leaf)
    assert (layers.cpu().numpy().view(np.uint16).reshape(n_seg, 32) == want_layers).all(), (seed, leaf, sizes)
    assert (total.cpu().numpy().view(np.uint16) == want_total).all()


@pytest.mark.parametrize("seed", range(10))
def test_lattice_hash_over_random_record_mixes(seed):
    rng = np.random.default_rng(7500 + seed)
    n = int(rng.integers(1, 3000))
    style = seed % 4
    if style == 0:      # short records, many empty
        lens = rng.integers(0, 200, size=n) * (rng.random(n) > 0.3)
    elif style == 1:    # mean above the four-lane threshold
        n = int(rng.integers(1, 200))
        lens = rng.integers(0, 120_000, size=n)
    elif style == 2:    # one giant among dwarfs
        lens = rng.integers(0, 2000, size=n)
        lens[int(rng.integers(0, n))] = 700_000
    else:               # around the block size
        lens = 128 * rng.integers(0, 6, size=n) + rng.integers(-1, 2, size=n).clip(0)
    lens = lens.astype(np.uint64)
    off = np.zeros(n + 1, dtype=np.uint64)
    off[1:] = np.cumsum(lens)
    shift = int(rng.integers(0, 4))                                       # any byte alignment
    data = wl.uniform_bytes(7600 + seed, 0, int(off[-1]) + shift)
    dd, do = to_dev(data), to_dev(off + np.uint64(shift))
    lanes = torch.zeros(1024, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash(dd.data_ptr(), do.data_ptr(), n, lanes.data_ptr())
    torch.cuda.synchronize()
    want = oracle.lthash(data[shift:], off)
    assert (lanes.cpu().numpy().view(np.uint16) == want).all(), (seed, style, n)
    # the same records spread over sources, on top of a carried sum
    n_src = int(rng.integers(1, 40))
    src = rng.integers(0, n_src + 2, size=n).astype(np.uint32)            # a few ids out of range
    acc0 = rng.integers(0, 65536, size=(n_src, 1024)).astype(np.uint16)
    acc = to_dev(acc0.reshape(-1))
    sentry.sentry_lthash_sources(dd.data_ptr(), do.data_ptr(), to_dev(src.view(np.int32)).data_ptr(), n, n_src, acc.data_ptr())
    torch.cuda.synchronize()
    want_acc = oracle.lthash_sources(data[shift:], off, src, n_src, acc=acc0.copy())
    assert (acc.cpu().numpy().view(np.uint16).reshape(n_src, 1024) == want_acc).all(), (seed, style, n, n_src)
    # and from pinned host memory in batches
    host = torch.from_numpy(data).pin_memory()
    hoff = (off + np.uint64(shift)).copy()
    longest = int(lens.max()) if n else 1
    lanes.zero_()
    sentry.sentry_lthash_h2d(host.data_ptr(), hoff.ctypes.data, n, max(longest, int(off[-1]) // 5 + 1), lanes.data_ptr())
    torch.cuda.synchronize()
    assert (lanes.cpu().numpy().view(np.uint16) == want).all(), (seed, style, n)


@pytest.mark.parametrize("seed", range(8))
def test_coalesced_trees_over_random_tensor_lists(seed):
    # both ways of Algorithm 1, tensors at random alignments
    rng = np.random.default_rng(7300 + seed)
    hid, dl = HASHES[seed % 3]
    leaf = int(rng.choice([64, 192, 1024, 4096, 65_536]))
    n_seg = int(rng.integers(1, 30))
    sizes = random_lengths(rng, n_seg, leaf)
    shifts = [int(rng.integers(0, 16)) if rng.integers(0, 2) else 0 for _ in sizes]
    segs = [wl.uniform_bytes(7310 + 40 * seed + i, 0, n) for i, n in enumerate(sizes)]
    devs, ptrs = [], []
    for s, sh in zip(segs, shifts):
        d = torch.zeros(s.size + sh + 16, dtype=torch.uint8, device="cuda")
        if s.size:
            d[sh:sh + s.size] = to_dev(s)
        devs.append(d)
        ptrs.append(d.data_ptr() + sh if s.size else 0)
    total = sum(sizes)
    padded = -(-total // leaf) * leaf
    buf = torch.zeros(padded + 16, dtype=torch.uint8, device="cuda")
    a = torch.zeros(64, dtype=torch.uint8, device="cuda")
    b = torch.zeros(64, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_coalesced_h(hid, ptrs, sizes, leaf, buf.data_ptr(), padded, a.data_ptr())
    sentry.sentry_merkle_coalesced_h(hid, ptrs, sizes, leaf, 0, 0, b.data_ptr())
    torch.cuda.synchronize()
    want = oracle.merkle_coalesced_h(hid, segs, leaf)
    assert bytes(a.cpu().numpy()[:dl]) == want, (hid, leaf, sizes, shifts)
    assert bytes(b.cpu().numpy()[:dl]) == want, (hid, leaf, sizes, shifts)


@pytest.mark.parametrize("seed", range(10))
def test_32_partition_hash_over_random_record_mixes(seed):
    # plain, per source (counters in LDS and in memory) and for samples of one size
    rng = np.random.default_rng(7400 + seed)
    n = int(rng.choice([1, 7, 100, 3000, 40_000]))
    hi = int(rng.choice([40, 700, 5000])) if n <= 3000 else 60
    lens = rng.integers(0, hi, n).astype(np.uint64)
    if n <= 100:
        lens[int(rng.integers(0, n))] = int(rng.integers(5000, 200_000))      # one long record among short ones
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(7410 + seed, 0, max(int(off[-1]), 1))[:int(off[-1])]
    sh = int(rng.integers(0, 4))
    buf = torch.zeros(data.size + sh + 16, dtype=torch.uint8, device="cuda")
    if data.size:
        buf[sh:sh + data.size] = to_dev(data)
    d_off = to_dev(off)
    out = torch.zeros(32, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash32(buf.data_ptr() + sh, d_off.data_ptr(), n, out.data_ptr())
    n_src = int(rng.choice([1, 3, 16, 255, 256, 257, 1000, 4096]))
    src = rng.integers(0, n_src + 1, n).astype(np.uint32)                       # some ids outside the table
    acc0 = rng.integers(0, 65536, (n_src, 32)).astype(np.uint16)
    acc, d_src = to_dev(acc0.reshape(-1)), to_dev(src.view(np.int32))
    sentry.sentry_lthash32_sources(buf.data_ptr() + sh, d_off.data_ptr(), d_src.data_ptr(), n, n_src, acc.data_ptr())
    rb = int(rng.choice([0, 1, 100, 129, 3072]))
    m = min(n, data.size // rb) if rb else n
    fixed = torch.zeros(32, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash32_fixed(buf.data_ptr() + sh, rb, m, fixed.data_ptr())
    torch.cuda.synchronize()
    assert (out.cpu().numpy().view(np.uint16) == oracle.lthash32(data, off)).all(), (n, hi, sh)
    want = oracle.lthash32_sources(data, off, src, n_src, acc=acc0)
    assert (acc.cpu().numpy().view(np.uint16).reshape(n_src, 32) == want).all(), (n, n_src, sh)
    o2 = np.arange(m + 1, dtype=np.uint64) * np.uint64(rb)
    assert (fixed.cpu().numpy().view(np.uint16) == oracle.lthash32(data[:rb * m], o2)).all(), (rb, m, sh)


@pytest.mark.parametrize("seed", range(12))
def test_per_source_sums_over_random_batches(seed):
    # batch sizes on both sides of what the root-hash launch sorts by itself (8192 records, 256
    # sources), numbers of sources on both sides of one 64-entry stretch of the unit table, sources
    # without records, one source that owns everything, ids outside the table; twice into one sum
    rng = np.random.default_rng(7900 + seed)
    n = int(rng.choice([1, 64, 65, 2048, 2049, 8191, 8192, 8193, 12_000, int(rng.integers(1, 9000))]))
    n_src = int(rng.choice([1, 2, 16, 64, 65, 255, 256, 257, 1000, 4096]))
    lens = rng.integers(0, int(rng.choice([2, 40, 300])), size=n).astype(np.uint64)
    if seed % 3 == 0:
        lens[int(rng.integers(0, n))] = int(rng.integers(1000, 50_000))
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(7950 + seed, 0, int(off[-1]))
    mode = seed % 4
    if mode == 0:
        src = rng.integers(0, n_src, size=n)
    elif mode == 1:
        src = rng.integers(0, n_src + 1, size=n)
    elif mode == 2:
        src = np.full(n, int(rng.integers(0, n_src)))
    else:
        src = (rng.integers(0, n_src, size=n) // 7) * 7 % n_src
    src = src.astype(np.uint32)
    acc0 = rng.integers(0, 65536, size=(n_src, 1024)).astype(np.uint16)
    acc = to_dev(acc0.reshape(-1))
    dd, do, ds = to_dev(data), to_dev(off), to_dev(src.view(np.int32))
    want = acc0
    for _ in range(2):
        sentry.sentry_lthash_sources(dd.data_ptr(), do.data_ptr(), ds.data_ptr(), n, n_src, acc.data_ptr())
        torch.cuda.synchronize()
        want = oracle.lthash_sources(data, off, src, n_src, acc=want)
        assert (acc.cpu().numpy().view(np.uint16).reshape(n_src, 1024) == want).all(), (seed, n, n_src, mode)

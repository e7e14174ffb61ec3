"""The synthetic-input generators: numpy and torch versions are bit-identical, shapes
match the target configurations."""
import numpy as np
import torch

from paper_2510_00554_amd import workloads as wl


def test_uniform_bytes_numpy_equals_torch():
    for start, n in ((0, 100), (3, 77), (8, 8), (13, 4099), (1 << 33, 1000)):
        a = wl.uniform_bytes(7, start, n)
        b = wl.uniform_bytes(7, start, n, device="cpu", chunk=1001).numpy()
        assert a.dtype == np.uint8 and (a == b).all(), (start, n)
    # a sub-range is a slice of the stream
    full = wl.uniform_bytes(9, 0, 5000)
    assert (wl.uniform_bytes(9, 1234, 999) == full[1234:2233]).all()
    assert abs(full.mean() - 127.5) < 4 and len(np.unique(full)) == 256


def test_normal_bf16_numpy_equals_torch():
    a = wl.normal_bf16_bits(11, 5, 20000)
    b = wl.normal_bf16_bits(11, 5, 20000, device="cpu", chunk=777).numpy().view(np.uint16)
    assert (a == b).all()
    vals = torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    assert abs(vals.mean()) < 1e-3 and abs(vals.std() - 0.02) < 1e-3
    # the integer rounding to bf16 equals torch's own float32 -> bfloat16 conversion
    w = wl._words_np(11, 5, 20005)
    s = ((w & np.uint64(0xFFFF)) + ((w >> np.uint64(16)) & np.uint64(0xFFFF))
         + ((w >> np.uint64(32)) & np.uint64(0xFFFF)) + (w >> np.uint64(48))).astype(np.int64) - 131070
    x = torch.from_numpy(s.astype(np.float32) * np.float32(wl.SCALE32))
    assert (x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16) == a).all()


def test_layout_sizes():
    l7 = wl.layout_7b()
    assert len(l7) == 291 and sum(n for _, n in l7) == 6_738_415_616
    l70 = wl.layout_70b()
    assert len(l70) == 723 and 2 * sum(n for _, n in l70) == 137_953_296_384
    assert all((2 * n) % 16 == 0 for _, n in l7 + l70 + wl.layout_tiny())


def test_record_lengths_and_batches():
    ln = wl.lognormal_record_lengths(20000)
    assert ln.min() >= 8000 and ln.max() <= 1_000_000
    assert abs(np.median(ln.astype(np.float64)) - 110_000) < 3000
    off = wl.offsets_from_lengths(ln)
    cuts = wl.cut_batches(off, 50_000_000)
    assert cuts[0][0] == 0 and cuts[-1][1] == 20000
    for (a, b), (c, d) in zip(cuts, cuts[1:]):
        assert b == c
    for a, b in cuts:
        assert int(off[b] - off[a]) <= 50_000_000
        if b < 20000:
            assert int(off[b + 1] - off[a]) > 50_000_000


def test_checkpoint_flat_equals_per_tensor():
    lay = wl.layout_tiny()
    buf, offs = wl.checkpoint_flat_torch(lay, "cpu")
    per = wl.checkpoint_bytes_np(lay)
    assert offs[-1] == sum(p.size for p in per)
    for i, p in enumerate(per):
        assert (buf[offs[i]:offs[i + 1]].numpy() == p).all()


def test_checkpoint_stream_ranges():
    lay = wl.layout_tiny()
    flat = np.concatenate(wl.checkpoint_bytes_np(lay))
    for start, n in ((0, 1000), (511, 4097), (flat.size - 777, 777), (2 * lay[0][1] - 3, 10)):
        assert (wl.checkpoint_stream_np(lay, start, n) == flat[start:start + n]).all(), (start, n)


def test_dirichlet_source_ids():
    for n_src in (1, 16, 128):
        ids = wl.dirichlet_source_ids(50_000, n_src, 99)
        assert ids.dtype == np.uint32 and ids.shape == (50_000,) and int(ids.max()) < n_src
        assert (ids == wl.dirichlet_source_ids(50_000, n_src, 99)).all()          # a function of the seed
        counts = np.bincount(ids, minlength=n_src)
        assert counts.sum() == 50_000
        if n_src > 1:
            assert (ids != wl.dirichlet_source_ids(50_000, n_src, 100)).any()
            # shares of concentration 1 are far from even: the largest is a multiple of the mean
            assert counts.max() > 2 * 50_000 / n_src and counts.min() < 0.5 * 50_000 / n_src

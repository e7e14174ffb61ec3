"""GPU parity: the HIP lattice-hash path against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import to_dev

pytestmark = pytest.mark.gpu


def gpu_lthash(data_np, off_np, base_shift=0):
    """base_shift moves the record bytes inside the device buffer to vary their alignment."""
    n = len(off_np) - 1
    buf = torch.zeros(data_np.size + base_shift + 16, dtype=torch.uint8, device="cuda")
    if data_np.size:
        buf[base_shift:base_shift + data_np.size] = to_dev(data_np)
    off = to_dev(np.asarray(off_np, dtype=np.uint64))
    out = torch.full((1024,), 0x5555, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash(buf.data_ptr() + base_shift, off.data_ptr(), n, out.data_ptr())
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16)


def test_empty_set():
    out = torch.full((1024,), 0x5555, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash(0, 0, 0, out.data_ptr())
    torch.cuda.synchronize()
    assert not out.cpu().numpy().any()


@pytest.mark.parametrize("length", [0, 1, 2, 3, 4, 5, 63, 64, 127, 128, 129, 130, 131, 132, 255, 256, 257,
                                    383, 384, 385, 3072, 8000, 100_003])
def test_single_record_every_alignment(length):
    data = wl.uniform_bytes(1000 + length, 0, length)
    off = np.array([0, length], np.uint64)
    want = oracle.lthash(data, off)
    for shift in (0, 1, 2, 3):
        assert (gpu_lthash(data, off, shift) == want).all(), (length, shift)


def test_many_small_variable_records():
    rng = np.random.default_rng(31)
    lens = rng.integers(0, 700, 3000).astype(np.uint64)
    lens[:20] = [0, 1, 127, 128, 129, 255, 256, 257, 0, 0, 5, 640, 128, 128, 1, 2, 3, 4, 384, 512]
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(1100, 0, int(off[-1]))
    assert (gpu_lthash(data, off) == oracle.lthash(data, off)).all()
    # offsets need not start at zero: drop the first 7 records from the set, not from the buffer
    assert (gpu_lthash(data, off[7:]) == oracle.lthash(data, off[7:])).all()


def test_lognormal_records_sample():
    lens = wl.lognormal_record_lengths(300, seed=77)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(1200, 0, int(off[-1]))
    assert (gpu_lthash(data, off) == oracle.lthash(data, off)).all()


def test_config2_images_and_halves():
    n = 50_000
    data, off = wl.image_records(n)
    want = oracle.lthash(data, off)
    d = to_dev(data)
    o = to_dev(off)
    full = torch.zeros(1024, dtype=torch.int16, device="cuda")
    a = torch.zeros(1024, dtype=torch.int16, device="cuda")
    b = torch.zeros(1024, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash(d.data_ptr(), o.data_ptr(), n, full.data_ptr())
    sentry.sentry_lthash(d.data_ptr(), o.data_ptr(), n // 2, a.data_ptr())
    sentry.sentry_lthash(d.data_ptr(), o.data_ptr() + 8 * (n // 2), n - n // 2, b.data_ptr())
    torch.cuda.synchronize()
    assert (full.cpu().numpy().view(np.uint16) == want).all()
    assert (a.cpu().numpy().view(np.uint16) == oracle.lthash(data, off[:n // 2 + 1])).all()
    assert (b.cpu().numpy().view(np.uint16) == oracle.lthash(data, off[n // 2:])).all()
    sentry.sentry_lthash_combine(a.data_ptr(), b.data_ptr())
    torch.cuda.synchronize()
    assert (a.cpu() == full.cpu()).all()
    sentry.sentry_lthash_remove(a.data_ptr(), b.data_ptr())
    torch.cuda.synchronize()
    assert (a.cpu().numpy().view(np.uint16) == oracle.lthash(data, off[:n // 2 + 1])).all()
    assert (d.cpu().numpy() == data).all()


def test_order_invariance_and_duplicates():
    rng = np.random.default_rng(41)
    recs = [wl.uniform_bytes(1300 + i, 0, int(l)) for i, l in enumerate(rng.integers(1, 500, 200))]
    perm = rng.permutation(200)
    a = np.concatenate(recs)
    b = np.concatenate([recs[i] for i in perm])
    off_a = wl.offsets_from_lengths([r.size for r in recs])
    off_b = wl.offsets_from_lengths([recs[i].size for i in perm])
    ha, hb = gpu_lthash(a, off_a), gpu_lthash(b, off_b)
    assert (ha == hb).all() and (ha == oracle.lthash(a, off_a)).all()
    twice = np.concatenate([a, recs[3]])
    off_t = wl.offsets_from_lengths([r.size for r in recs] + [recs[3].size])
    assert (gpu_lthash(twice, off_t) == oracle.lthash(twice, off_t)).all()


def test_combine_remove_against_oracle_with_wraparound():
    rng = np.random.default_rng(51)
    x = rng.integers(0, 65536, 1024).astype(np.uint16)
    y = rng.integers(0, 65536, 1024).astype(np.uint16)
    x[:4] = [0xFFFF, 0xFFFF, 0, 0x8000]
    y[:4] = [1, 0xFFFF, 1, 0x8000]
    dx, dy = to_dev(x), to_dev(y)
    sentry.sentry_lthash_combine(dx.data_ptr(), dy.data_ptr())
    torch.cuda.synchronize()
    assert (dx.cpu().numpy().view(np.uint16) == oracle.lthash_combine(x, y)).all()
    sentry.sentry_lthash_remove(dx.data_ptr(), dy.data_ptr())
    sentry.sentry_lthash_remove(dx.data_ptr(), dy.data_ptr())
    torch.cuda.synchronize()
    assert (dx.cpu().numpy().view(np.uint16) == oracle.lthash_remove(x, y)).all()
    # acc == x doubles / clears
    dz = to_dev(y)
    sentry.sentry_lthash_combine(dz.data_ptr(), dz.data_ptr())
    torch.cuda.synchronize()
    assert (dz.cpu().numpy().view(np.uint16) == oracle.lthash_combine(y, y)).all()
    sentry.sentry_lthash_remove(dz.data_ptr(), dz.data_ptr())
    torch.cuda.synchronize()
    assert not dz.cpu().numpy().any()
    # odd (2-byte) alignment and pinned host lanes
    pin = torch.zeros(1025, dtype=torch.int16).pin_memory()
    pin[1:] = torch.from_numpy(x.view(np.int16))
    sentry.sentry_lthash_combine(pin.data_ptr() + 2, dy.data_ptr())
    torch.cuda.synchronize()
    assert (pin[1:].numpy().view(np.uint16) == oracle.lthash_combine(x, y)).all() and pin[0] == 0


def test_same_record_65536_times_is_zero():
    rec = wl.uniform_bytes(1400, 0, 40)
    data = np.tile(rec, 65536)
    off = np.arange(65537, dtype=np.uint64) * np.uint64(40)
    assert not gpu_lthash(data, off).any()


def test_four_lane_path_edge_lengths_and_alignments():
    # a mean record length of 16 KiB or more selects four lanes per record: short records of
    # every edge length ride along with one long record
    lens = [0, 1, 2, 3, 4, 5, 31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 130, 131, 132,
            159, 160, 161, 255, 256, 257, 383, 384, 385, 4095, 4096, 4097, 1_500_003]
    off = wl.offsets_from_lengths(np.array(lens, np.uint64))
    assert int(off[-1]) >= 16384 * len(lens)
    data = wl.uniform_bytes(1500, 0, int(off[-1]))
    want = oracle.lthash(data, off)
    for shift in (0, 1, 2, 3):
        assert (gpu_lthash(data, off, shift) == want).all(), shift
    # the long record first, and a record count that is not a multiple of 16
    lens2 = [1_000_001] + lens[:20]
    off2 = wl.offsets_from_lengths(np.array(lens2, np.uint64))
    data2 = wl.uniform_bytes(1501, 0, int(off2[-1]))
    assert (gpu_lthash(data2, off2, 1) == oracle.lthash(data2, off2)).all()


def test_four_lane_path_many_records_in_length_order():
    # tens of thousands of records with a mean above 16 KiB: the device orders them by length
    # (many records per lane of the ordering workgroup, every bin of the top range in use, ties,
    # records beyond the last bin) and hashes sixteen per wave in that order
    n = 40_001
    rng = np.random.default_rng(62)
    lens = rng.integers(6_000, 42_000, n).astype(np.uint64)
    lens[::97] = 0
    lens[5::1013] = 20_480                 # ties on a bin boundary
    lens[7] = 1_300_000                    # beyond the last bin
    off = wl.offsets_from_lengths(lens)
    assert int(off[-1]) >= 16384 * n
    data = wl.uniform_bytes(1550, 0, int(off[-1]))
    assert (gpu_lthash(data, off, 3) == oracle.lthash(data, off)).all()


def test_unequal_short_records_take_the_ordered_four_lane_path():
    # mean far below 16 KiB, but records of very different lengths: the device finds that out from
    # 256 records at fixed positions (index k n / 256) and orders the batch; ten workgroups share
    # the ordering here, the last with a short run
    n = 40_001
    rng = np.random.default_rng(63)
    lens = np.clip(np.round(2500 * np.exp(0.9 * rng.standard_normal(n))), 0, 150_000).astype(np.uint64)
    lens[::131] = 0
    lens[(np.arange(256) * n) >> 8] = 6000           # what the device samples: >= 4 KiB and >= 1.5 x the mean
    off = wl.offsets_from_lengths(lens)
    assert 1.5 * int(off[-1]) / n <= 6000 and int(off[-1]) < 16384 * n
    data = wl.uniform_bytes(1560, 0, int(off[-1]))
    assert (gpu_lthash(data, off, 1) == oracle.lthash(data, off)).all()
    # the same lengths without the long samples: one lane per record, unordered
    lens[(np.arange(256) * n) >> 8] = 100
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(1561, 0, int(off[-1]))
    assert (gpu_lthash(data, off, 2) == oracle.lthash(data, off)).all()


def test_few_records_take_four_lanes_unordered():
    # up to 32,768 records: four lanes per record whatever the lengths, in the given order when
    # the lengths are about equal; both sides of the limit
    for n in (32_768, 32_769):
        lens = np.full(n, 700, np.uint64)
        lens[5] = 0
        off = wl.offsets_from_lengths(lens)
        data = wl.uniform_bytes(1570 + n % 7, 0, int(off[-1]))
        assert (gpu_lthash(data, off) == oracle.lthash(data, off)).all(), n


@pytest.mark.parametrize("unequal", [False, True])
def test_more_short_records_than_lanes_on_the_chip(unequal):
    # short records, one lane each, several rounds of waves per SIMD; or, with a few long records
    # where the device samples the lengths, in length order with four lanes each (all 64
    # workgroups of the ordering at work)
    n = 262_144 + 37
    rng = np.random.default_rng(61)
    lens = rng.integers(0, 48, n).astype(np.uint64)
    if unequal:
        lens[(np.arange(256) * n) >> 8] = 5000
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(1600, 0, int(off[-1]))
    assert (gpu_lthash(data, off) == oracle.lthash(data, off)).all()


@pytest.mark.parametrize("n", [1, 2, 3, 15, 16, 17, 64, 1000, 4097, 40_000])
def test_digests_one_by_one_and_their_sum(n):
    # every record's 1024 lanes written out, then Eq. (1) over those rows: both against the
    # oracle, and the sum against the fused path
    rng = np.random.default_rng(1700 + n)
    lens = rng.integers(0, 700, n).astype(np.uint64)
    if n > 2:
        lens[1] = 0
        lens[2] = 40_000
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(1700 + n, 0, int(off[-1]) + 1)
    dd, do = to_dev(data), to_dev(off)
    rows = torch.full((n + 1, 1024), 0x5555, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_digests(dd.data_ptr(), do.data_ptr(), n, rows.data_ptr())
    torch.cuda.synchronize()
    got = rows.cpu().numpy().view(np.uint16)
    want = oracle.lthash_digests(data, off)
    assert (got[:n] == want).all()
    assert (got[n] == 0x5555).all()                       # nothing past the last row
    out = torch.full((1024,), 0x5555, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_sum(rows.data_ptr(), n, out.data_ptr())
    torch.cuda.synchronize()
    assert (out.cpu().numpy().view(np.uint16) == oracle.lthash_sum(want)).all()
    assert (out.cpu().numpy().view(np.uint16) == gpu_lthash(data, off)).all()


@pytest.mark.parametrize("n", [0, 1, 2, 15, 16, 17, 255, 4096, 32_768 + 3, 70_001])
def test_sum_of_given_digests(n):
    # rows of arbitrary lanes (not digests of anything): the plain column sum mod 2^16, across
    # the sizes where the grid, the eight-rows-in-flight loop and its tail change
    rng = np.random.default_rng(1800 + n)
    d = rng.integers(0, 65536, size=(n, 1024)).astype(np.uint16)
    if n > 3:
        d[:3] = 0xFFFF                                     # carries must stay inside their lane
    dev = to_dev(d.reshape(-1)) if n else None
    out = torch.full((1024,), 0x5555, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_sum(dev.data_ptr() if n else 0, n, out.data_ptr())
    torch.cuda.synchronize()
    assert (out.cpu().numpy().view(np.uint16) == oracle.lthash_sum(d)).all()
    if n:
        assert (dev.cpu().numpy().view(np.uint16).reshape(n, 1024) == d).all()   # input untouched


def test_a_million_unequal_records_by_properties_and_samples():
    # too many for the oracle in full: the halves add up to the whole, the digests written out add
    # up to it too, and sampled digests (the longest record among them) equal the oracle's
    n = 1_000_000
    rng = np.random.default_rng(64)
    lens = np.clip(np.round(900 * np.exp(0.9 * rng.standard_normal(n))), 0, 120_000).astype(np.uint64)
    lens[(np.arange(256) * n) >> 8] = 7000           # the sampled lengths say "unequal"
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(1580, 0, int(off[-1]), device="cuda")
    d_off = to_dev(off)
    whole, a, b, s = (torch.zeros(1024, dtype=torch.int16, device="cuda") for _ in range(4))
    half = n // 2 + 17
    sentry.sentry_lthash(data.data_ptr(), d_off.data_ptr(), n, whole.data_ptr())
    sentry.sentry_lthash(data.data_ptr(), d_off.data_ptr(), half, a.data_ptr())
    sentry.sentry_lthash(data.data_ptr(), d_off.data_ptr() + 8 * half, n - half, b.data_ptr())
    sentry.sentry_lthash_combine(a.data_ptr(), b.data_ptr())
    rows = torch.empty((n, 1024), dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_digests(data.data_ptr(), d_off.data_ptr(), n, rows.data_ptr())
    sentry.sentry_lthash_sum(rows.data_ptr(), n, s.data_ptr())
    torch.cuda.synchronize()
    assert whole.cpu().numpy().any()
    assert torch.equal(whole, a) and torch.equal(whole, s)
    picks = [0, 1, n - 1, int(np.argmax(lens)), int(np.argmin(lens))] + [int(x) for x in rng.integers(0, n, 40)]
    for i in picks:
        rec = data[int(off[i]):int(off[i + 1])].cpu().numpy()
        assert (rows[i].cpu().numpy().view(np.uint16) == oracle.lthash_one(rec)).all(), i


def gpu_sources(data_np, off_np, src_np, n_sources, acc=None):
    n = len(off_np) - 1
    buf = to_dev(data_np) if data_np.size else torch.zeros(16, dtype=torch.uint8, device="cuda")
    off = to_dev(np.asarray(off_np, dtype=np.uint64))
    src = torch.from_numpy(np.asarray(src_np, dtype=np.uint32).view(np.int32).copy()).cuda()
    if acc is None:
        acc = torch.zeros(n_sources * 1024, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_sources(buf.data_ptr(), off.data_ptr(), src.data_ptr(), n, n_sources, acc.data_ptr())
    torch.cuda.synchronize()
    return acc


def as_u16(acc, n_sources):
    return acc.cpu().numpy().view(np.uint16).reshape(n_sources, 1024)


@pytest.mark.parametrize("n,n_sources", [(1, 1), (60, 5), (1000, 16), (5000, 128), (333, 4096), (9000, 2), (9000, 9)])
def test_per_source_running_sums(n, n_sources):
    rng = np.random.default_rng(71 + n)
    lens = rng.integers(0, 600, n).astype(np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(1700 + n, 0, int(off[-1]))
    src = rng.integers(0, n_sources, n).astype(np.uint32)
    if n > 10:
        src[3] = n_sources          # ids outside the table are left out
        src[7] = 0xFFFFFFFF
    want = oracle.lthash_sources(data, off, src, n_sources)
    acc = gpu_sources(data, off, src, n_sources)
    assert (as_u16(acc, n_sources) == want).all()
    # a second batch lands on top of the running sums
    want2 = oracle.lthash_sources(data, off, src, n_sources, acc=want)
    acc = gpu_sources(data, off, src, n_sources, acc=acc)
    assert (as_u16(acc, n_sources) == want2).all()


@pytest.mark.parametrize("n,n_sources", [(2, 2), (63, 3), (64, 255), (65, 256), (128, 16), (129, 257), (2048, 200),
                                         (8191, 7), (8192, 256), (8193, 256), (8192, 257), (1500, 2)])
def test_per_source_small_batches_sorted_inside_the_root_hash_launch(n, n_sources):
    # up to 8192 records over up to 256 sources the sort by source is one more workgroup of the
    # root-hash launch; one step beyond either limit it is the two sort kernels: both sides of
    # both limits, sources without records, ids outside the table, and the same call twice over
    # (the second finds the tables as the first left them) and then the other path on top
    rng = np.random.default_rng(7100 + 31 * n + n_sources)
    lens = rng.integers(0, 300, n).astype(np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(7200 + n, 0, int(off[-1]))
    src = rng.integers(0, n_sources, n).astype(np.uint32)
    if n_sources > 4:
        src[src == 1] = 0                      # a source with no record
        src[src == n_sources - 2] = n_sources - 1
    if n > 10:
        src[5] = n_sources
        src[9] = 0xFFFFFFFF
    want = oracle.lthash_sources(data, off, src, n_sources)
    acc = gpu_sources(data, off, src, n_sources)
    assert (as_u16(acc, n_sources) == want).all()
    want = oracle.lthash_sources(data, off, src, n_sources, acc=want)
    acc = gpu_sources(data, off, src, n_sources, acc=acc)
    assert (as_u16(acc, n_sources) == want).all()
    # a larger batch (the two sort kernels) and the small one again, into the same sums
    big = 9000
    lens_b = rng.integers(0, 100, big).astype(np.uint64)
    off_b = wl.offsets_from_lengths(lens_b)
    data_b = wl.uniform_bytes(7300 + n, 0, int(off_b[-1]))
    src_b = rng.integers(0, n_sources, big).astype(np.uint32)
    want = oracle.lthash_sources(data_b, off_b, src_b, n_sources, acc=want)
    acc = gpu_sources(data_b, off_b, src_b, n_sources, acc=acc)
    assert (as_u16(acc, n_sources) == want).all()
    want = oracle.lthash_sources(data, off, src, n_sources, acc=want)
    acc = gpu_sources(data, off, src, n_sources, acc=acc)
    assert (as_u16(acc, n_sources) == want).all()


@pytest.mark.parametrize("n,n_sources", [(6000, 16), (20_000, 128)])
def test_per_source_with_shares_of_a_dirichlet_draw(n, n_sources):
    # the source mix of the paper's run over the number of sources (section 5.2): uneven shares
    lens = np.full(n, 96, dtype=np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(7400 + n, 0, int(off[-1]))
    src = wl.dirichlet_source_ids(n, n_sources, 7401)
    want = oracle.lthash_sources(data, off, src, n_sources)
    assert (as_u16(gpu_sources(data, off, src, n_sources), n_sources) == want).all()


@pytest.mark.parametrize("n,n_sources,long_record", [(32_769, 16, False), (33_000, 256, True), (40_000, 3, False),
                                                    (33_000, 257, True), (70_000, 200, True)])
def test_per_source_large_batches_sorted_inside_the_two_root_hash_launches(n, n_sources, long_record):
    # more than 32,768 records over up to 256 sources: the count by source rides in the one-lane
    # root-hash launch and the scatter in the four-lane launch; whichever of the two the device picks
    # to hash the batch (short equal records: one lane; one record far longer than the rest among
    # those the device samples: four lanes), both steps must have run.  257 sources: the two sort
    # launches.  Twice into one set of sums.
    rng = np.random.default_rng(7700 + n + n_sources)
    lens = rng.integers(0, 48, n).astype(np.uint64)
    if long_record:
        lens[(5 * n) >> 8] = 60_000
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(7800 + n, 0, int(off[-1]))
    src = wl.dirichlet_source_ids(n, n_sources, 7801 + n)
    src[11] = n_sources
    src[n - 1] = 0xFFFFFFFF
    want = oracle.lthash_sources(data, off, src, n_sources)
    acc = gpu_sources(data, off, src, n_sources)
    assert (as_u16(acc, n_sources) == want).all()
    want = oracle.lthash_sources(data, off, src, n_sources, acc=want)
    acc = gpu_sources(data, off, src, n_sources, acc=acc)
    assert (as_u16(acc, n_sources) == want).all()


def test_per_source_skewed_and_single_source_equals_plain_hash():
    n = 3000
    rng = np.random.default_rng(81)
    lens = rng.integers(1, 400, n).astype(np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(1800, 0, int(off[-1]))
    src = np.zeros(n, np.uint32)
    src[rng.choice(n, 40, replace=False)] = rng.integers(1, 8, 40)   # one source owns nearly everything
    assert (as_u16(gpu_sources(data, off, src, 8), 8) == oracle.lthash_sources(data, off, src, 8)).all()
    one = as_u16(gpu_sources(data, off, np.zeros(n, np.uint32), 1), 1)
    assert (one[0] == gpu_lthash(data, off)).all() and (one[0] == oracle.lthash(data, off)).all()


def test_per_source_many_records_larger_units():
    # more than 8192 units of 32 records: the unit size doubles
    n = 300_000
    rng = np.random.default_rng(91)
    lens = rng.integers(0, 24, n).astype(np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(1900, 0, int(off[-1]))
    src = rng.integers(0, 16, n).astype(np.uint32)
    assert (as_u16(gpu_sources(data, off, src, 16), 16) == oracle.lthash_sources(data, off, src, 16)).all()


def test_per_source_image_batches_like_the_paper():
    # 16 sources, batches of 512 image-shaped samples (section 5: batch sizes 32..512, 16 sources)
    n_sources, batch = 16, 512
    data, off = wl.image_records(4 * batch)
    rng = np.random.default_rng(95)
    src = rng.integers(0, n_sources, 4 * batch).astype(np.uint32)
    acc = torch.zeros(n_sources * 1024, dtype=torch.int16, device="cuda")
    for b in range(4):
        lo, hi = b * batch, (b + 1) * batch
        acc = gpu_sources(data, off[lo:hi + 1], src[lo:hi], n_sources, acc=acc)
    assert (as_u16(acc, n_sources) == oracle.lthash_sources(data, off, src, n_sources)).all()

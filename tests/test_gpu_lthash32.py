"""GPU parity: the 32-partition lattice hash (plain BLAKE2b-512 digests, section 4.2.2)
against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import to_dev

pytestmark = pytest.mark.gpu


def gpu_lthash32(data_np, off_np, base_shift=0):
    """base_shift moves the record bytes inside the device buffer to vary their alignment."""
    n = len(off_np) - 1
    buf = torch.zeros(data_np.size + base_shift + 16, dtype=torch.uint8, device="cuda")
    if data_np.size:
        buf[base_shift:base_shift + data_np.size] = to_dev(data_np)
    off = to_dev(np.asarray(off_np, dtype=np.uint64))
    out = torch.full((32,), 0x5555, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash32(buf.data_ptr() + base_shift, off.data_ptr(), n, out.data_ptr())
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16)


def test_empty_set():
    out = torch.full((32,), 0x5555, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash32(0, 0, 0, out.data_ptr())
    torch.cuda.synchronize()
    assert not out.cpu().numpy().any()


@pytest.mark.parametrize("length", [0, 1, 2, 3, 4, 5, 63, 64, 127, 128, 129, 130, 131, 132, 255, 256, 257,
                                    383, 384, 385, 3072, 8000, 100_003])
def test_single_record_every_alignment(length):
    data = wl.uniform_bytes(4000 + length, 0, length)
    off = np.array([0, length], np.uint64)
    want = oracle.lthash32(data, off)
    for shift in (0, 1, 2, 3):
        assert (gpu_lthash32(data, off, shift) == want).all(), (length, shift)


def test_many_small_variable_records_one_lane_each():
    rng = np.random.default_rng(131)
    lens = rng.integers(0, 700, 3000).astype(np.uint64)
    lens[:20] = [0, 1, 127, 128, 129, 255, 256, 257, 0, 0, 5, 640, 128, 128, 1, 2, 3, 4, 384, 512]
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(4100, 0, int(off[-1]))
    assert (gpu_lthash32(data, off) == oracle.lthash32(data, off)).all()
    # offsets need not start at zero
    assert (gpu_lthash32(data, off[7:]) == oracle.lthash32(data, off[7:])).all()


def test_equal_long_records_four_lanes_each():
    # equal lengths of 384 bytes and more go four lanes to a record, unordered
    for length, n, shift in ((3072, 300, 0), (385, 257, 1), (150_528, 9, 2)):
        off = wl.offsets_from_lengths(np.full(n, length, np.uint64))
        data = wl.uniform_bytes(4200 + n, 0, int(off[-1]))
        assert (gpu_lthash32(data, off, shift) == oracle.lthash32(data, off)).all(), (length, n)


def test_unequal_long_records_in_length_order():
    lens = wl.lognormal_record_lengths(400, seed=177)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(4300, 0, int(off[-1]))
    assert (gpu_lthash32(data, off, 3) == oracle.lthash32(data, off)).all()


def test_few_records():
    lens = np.array([5, 0, 1000, 129, 128], np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(4400, 0, int(off[-1]))
    assert (gpu_lthash32(data, off) == oracle.lthash32(data, off)).all()


@pytest.mark.parametrize("n", [1, 15, 16, 17, 255, 256, 257, 4095, 4097, 70_001, 300_000])
def test_row_sum_over_one_and_many_workgroups(n):
    """Short records, so that the count decides how the digest rows are cut among the
    workgroups of the sum: one workgroup, a ragged last trip, runs of unequal length."""
    rng = np.random.default_rng(n)
    lens = rng.integers(0, 24, n).astype(np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(4500 + n, 0, max(int(off[-1]), 1))[:int(off[-1])]
    assert (gpu_lthash32(data, off) == oracle.lthash32(data, off)).all()


def test_same_record_65536_times_is_zero_and_order_does_not_matter():
    rec = wl.uniform_bytes(4600, 0, 40)
    data = np.tile(rec, 65536)
    off = wl.offsets_from_lengths(np.full(65536, 40, np.uint64))
    assert not gpu_lthash32(data, off).any()
    lens = np.array([40, 3, 200, 7, 90], np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(4601, 0, int(off[-1]))
    parts = [data[int(off[i]):int(off[i + 1])] for i in range(5)]
    perm = [3, 0, 4, 2, 1]
    data2 = np.concatenate([parts[i] for i in perm])
    off2 = wl.offsets_from_lengths(lens[perm])
    assert (gpu_lthash32(data, off) == gpu_lthash32(data2, off2)).all()


def test_combine_and_remove_against_the_oracle_with_wraparound():
    lens = np.array([100, 400, 3, 0, 129, 77, 5000, 64], np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(4700, 0, int(off[-1]))
    a = oracle.lthash32(data, off[:4])          # records 0..2
    b = oracle.lthash32(data, off[3:])          # records 3..7
    whole = oracle.lthash32(data, off)
    da = to_dev(a.view(np.int16).copy())
    db = to_dev(b.view(np.int16).copy())
    sentry.sentry_lthash32_combine(da.data_ptr(), db.data_ptr())
    torch.cuda.synchronize()
    assert (da.cpu().numpy().view(np.uint16) == whole).all()
    sentry.sentry_lthash32_remove(da.data_ptr(), db.data_ptr())
    torch.cuda.synchronize()
    assert (da.cpu().numpy().view(np.uint16) == a).all()
    # lanes that wrap: 0xffff + 2 = 1, 1 - 2 = 0xffff
    x = to_dev(np.full(32, -1, np.int16))
    y = to_dev(np.full(32, 2, np.int16))
    sentry.sentry_lthash32_combine(x.data_ptr(), y.data_ptr())
    torch.cuda.synchronize()
    assert (x.cpu().numpy().view(np.uint16) == 1).all()
    sentry.sentry_lthash32_remove(x.data_ptr(), y.data_ptr())
    torch.cuda.synchronize()
    assert (x.cpu().numpy().view(np.uint16) == 0xffff).all()
    want = oracle.lanes_sub(whole.copy(), b)
    assert (want == a).all()
    # the 1024-lane calls and the 32-lane calls do not disturb each other on one stream
    big = torch.zeros(1024, dtype=torch.int16, device="cuda")
    d_data, d_off = to_dev(data), to_dev(off)
    sentry.sentry_lthash(d_data.data_ptr(), d_off.data_ptr(), len(lens), big.data_ptr())
    small = gpu_lthash32(data, off)
    torch.cuda.synchronize()
    assert (big.cpu().numpy().view(np.uint16) == oracle.lthash(data, off)).all()
    assert (small == whole).all()


@pytest.mark.parametrize("pinned", [True, False])
def test_running_sum_over_batches_fed_from_host_memory(pinned):
    # 13 batches of unequal sizes (one empty, one of a single empty record) fed back to back on a
    # stream of their own: every staging slot and hash stream is used several times, and a 1024-lane
    # running sum is fed in between on the same stream (they share staging buffers and scratch)
    lens = wl.lognormal_record_lengths(1300, seed=151, median=9_000, lo=0, hi=300_000)
    lens[700] = 0
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(4800, 0, int(off[-1]))
    want = oracle.lthash32(data, off)
    host = torch.from_numpy(data.copy())
    hoff = torch.from_numpy(off.view(np.int64).copy())
    if pinned:
        host, hoff = host.pin_memory(), hoff.pin_memory()
    cuts = [0, 10, 11, 11, 300, 350, 700, 701, 900, 901, 1000, 1100, 1250, 1300]
    s = torch.cuda.Stream()
    out = torch.full((48,), 0x2222, dtype=torch.int16, device="cuda")
    out_wide = torch.zeros(1024, dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()     # torch fills the outputs on its own stream, which s does not wait for
    st = sentry.sentry_lthash32_stream_begin()
    wide = sentry.sentry_lthash_stream_begin()
    for k, (a, b) in enumerate(zip(cuts[:-1], cuts[1:])):
        sentry.sentry_lthash_stream_update_h2d(st, host.data_ptr(), hoff.data_ptr() + 8 * a, b - a, s.cuda_stream)
        if k in (3, 4):
            sentry.sentry_lthash_stream_update_h2d(wide, host.data_ptr(), hoff.data_ptr() + 8 * a, b - a, s.cuda_stream)
    sentry.sentry_lthash_stream_final(st, out.data_ptr(), s.cuda_stream)
    sentry.sentry_lthash_stream_final(wide, out_wide.data_ptr(), s.cuda_stream)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    assert (got[:32] == want).all() and (got[32:] == 0x2222).all()
    assert (out_wide.cpu().numpy().view(np.uint16) == oracle.lthash(data[:int(off[350])], off[11:351])).all()
    # two batches; and nothing at all
    st = sentry.sentry_lthash32_stream_begin()
    sentry.sentry_lthash_stream_update_h2d(st, host.data_ptr(), hoff.data_ptr() + 8 * 300, 400, s.cuda_stream)
    sentry.sentry_lthash_stream_update_h2d(st, host.data_ptr(), hoff.data_ptr(), 300, s.cuda_stream)
    sentry.sentry_lthash_stream_final(st, out.data_ptr(), s.cuda_stream)
    torch.cuda.synchronize()
    assert (out.cpu().numpy().view(np.uint16)[:32] == oracle.lthash32(data[:int(off[700])], off[:701])).all()
    st = sentry.sentry_lthash32_stream_begin()
    sentry.sentry_lthash_stream_final(st, out.data_ptr(), s.cuda_stream)
    torch.cuda.synchronize()
    assert (out.cpu()[:32] == 0).all()
    st = sentry.sentry_lthash32_stream_begin()
    sentry.sentry_lthash_stream_abort(st)


def gpu_sources32(data_np, off_np, src_np, n_sources, acc=None):
    n = len(off_np) - 1
    buf = torch.zeros(max(data_np.size, 1) + 16, dtype=torch.uint8, device="cuda")
    if data_np.size:
        buf[:data_np.size] = to_dev(data_np)
    off = to_dev(np.asarray(off_np, dtype=np.uint64))
    src = to_dev(np.asarray(src_np, dtype=np.uint32).view(np.int32))
    if acc is None:
        acc = torch.zeros(n_sources * 32 + 8, dtype=torch.int16, device="cuda")
        acc[n_sources * 32:] = 0x1111
    sentry.sentry_lthash32_sources(buf.data_ptr(), off.data_ptr(), src.data_ptr(), n, n_sources, acc.data_ptr())
    torch.cuda.synchronize()
    return acc


def rows32(acc, n_sources):
    a = acc.cpu().numpy().view(np.uint16)
    assert (a[n_sources * 32:] == 0x1111).all()
    return a[:n_sources * 32].reshape(n_sources, 32)


@pytest.mark.parametrize("n,n_sources", [(1, 1), (60, 5), (1000, 16), (5000, 128), (9000, 256), (9000, 257), (333, 4096),
                                         (300_000, 16), (300_000, 1000)])
def test_per_source_running_sums(n, n_sources):
    # counters in LDS up to 256 sources and in memory beyond; one and many workgroups; ids outside the table
    rng = np.random.default_rng(171 + n + n_sources)
    lens = rng.integers(0, 600 if n < 100_000 else 24, n).astype(np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(4900 + n, 0, int(off[-1]))
    src = rng.integers(0, n_sources, n).astype(np.uint32)
    if n > 10:
        src[3] = n_sources
        src[7] = 0xFFFFFFFF
    want = oracle.lthash32_sources(data, off, src, n_sources)
    acc = gpu_sources32(data, off, src, n_sources)
    assert (rows32(acc, n_sources) == want).all()
    # a second batch lands on top of the running sums
    want2 = oracle.lthash32_sources(data, off, src, n_sources, acc=want)
    acc = gpu_sources32(data, off, src, n_sources, acc=acc)
    assert (rows32(acc, n_sources) == want2).all()


def test_per_source_one_owner_of_nearly_everything_and_one_source_is_the_plain_hash():
    n = 70_000                                        # more than 65,536 records meet in one counter
    rng = np.random.default_rng(181)
    lens = rng.integers(1, 40, n).astype(np.uint64)
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(4950, 0, int(off[-1]))
    src = np.zeros(n, np.uint32)
    src[rng.choice(n, 40, replace=False)] = rng.integers(1, 8, 40)
    assert (rows32(gpu_sources32(data, off, src, 8), 8) == oracle.lthash32_sources(data, off, src, 8)).all()
    one = rows32(gpu_sources32(data, off, np.zeros(n, np.uint32), 1), 1)
    assert (one[0] == gpu_lthash32(data, off)).all() and (one[0] == oracle.lthash32(data, off)).all()
    # no record at all: the running sums stay as they are
    acc = torch.full((8 * 32 + 8,), 0x1111, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash32_sources(0, 0, 0, 0, 8, acc.data_ptr())
    torch.cuda.synchronize()
    assert (acc.cpu() == 0x1111).all()

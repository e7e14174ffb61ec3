"""GPU parity: the lattice hash of samples of one size laid back to back (no offsets array), at
both widths, against the CPU oracle fed the same bytes with the offsets written out."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import to_dev

pytestmark = pytest.mark.gpu


def gpu_fixed(data_np, record_bytes, n, shift=0):
    buf = torch.zeros(data_np.size + shift + 16, dtype=torch.uint8, device="cuda")
    if data_np.size:
        buf[shift:shift + data_np.size] = to_dev(data_np)
    wide = torch.full((1024 + 8,), 0x3333, dtype=torch.int16, device="cuda")
    narrow = torch.full((32 + 8,), 0x3333, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_fixed(buf.data_ptr() + shift, record_bytes, n, wide.data_ptr())
    sentry.sentry_lthash32_fixed(buf.data_ptr() + shift, record_bytes, n, narrow.data_ptr())
    torch.cuda.synchronize()
    w, m = wide.cpu().numpy().view(np.uint16), narrow.cpu().numpy().view(np.uint16)
    assert (w[1024:] == 0x3333).all() and (m[32:] == 0x3333).all()
    return w[:1024], m[:32]


def oracle_fixed(data_np, record_bytes, n):
    off = np.arange(n + 1, dtype=np.uint64) * np.uint64(record_bytes)
    return oracle.lthash(data_np, off), oracle.lthash32(data_np, off)


@pytest.mark.parametrize("record_bytes", [0, 1, 3, 64, 127, 128, 129, 383, 384, 385, 3072, 16_383, 16_384, 100_003])
def test_record_sizes_and_alignments(record_bytes):
    # few records: four lanes each; sizes on both sides of every block and path boundary
    n = 37
    data = wl.uniform_bytes(6000 + record_bytes, 0, n * record_bytes)
    want = oracle_fixed(data, record_bytes, n)
    for shift in (0, 1, 2, 3):
        got = gpu_fixed(data, record_bytes, n, shift)
        assert (got[0] == want[0]).all() and (got[1] == want[1]).all(), (record_bytes, shift)


@pytest.mark.parametrize("n", [0, 1, 15, 16, 17, 32_768, 32_769, 70_001])
def test_record_counts_on_both_sides_of_the_one_lane_path(n):
    # up to 32,768 records go four lanes each, more go one lane each (short records)
    record_bytes = 100
    data = wl.uniform_bytes(6100 + n, 0, max(n * record_bytes, 1))[:n * record_bytes]
    want = oracle_fixed(data, record_bytes, n)
    got = gpu_fixed(data, record_bytes, n, shift=n % 4)
    assert (got[0] == want[0]).all() and (got[1] == want[1]).all()


def test_many_long_records_take_four_lanes():
    n, record_bytes = 33_000, 16_384
    data = wl.uniform_bytes(6200, 0, n * record_bytes)
    off = np.arange(n + 1, dtype=np.uint64) * np.uint64(record_bytes)
    got = gpu_fixed(data, record_bytes, n)
    assert (got[1] == oracle.lthash32(data, off)).all()
    # the wide hash of half a gigabyte is slow on one core: the same bytes through the call with offsets instead
    d, o = to_dev(data), to_dev(off)
    out = torch.zeros(1024, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash(d.data_ptr(), o.data_ptr(), n, out.data_ptr())
    torch.cuda.synchronize()
    assert (got[0] == out.cpu().numpy().view(np.uint16)).all()
    sample = oracle.lthash(data[:64 * record_bytes], off[:65])
    sentry.sentry_lthash_fixed(d.data_ptr(), record_bytes, 64, out.data_ptr())
    torch.cuda.synchronize()
    assert (out.cpu().numpy().view(np.uint16) == sample).all()


def test_config2_images_without_an_offsets_array():
    data, off = wl.image_records(50_000, device="cuda")
    host = data.cpu().numpy()
    wide = torch.zeros(1024, dtype=torch.int16, device="cuda")
    narrow = torch.zeros(32, dtype=torch.int16, device="cuda")
    sentry.sentry_lthash_fixed(data.data_ptr(), 3072, 50_000, wide.data_ptr())
    sentry.sentry_lthash32_fixed(data.data_ptr(), 3072, 50_000, narrow.data_ptr())
    torch.cuda.synchronize()
    assert (wide.cpu().numpy().view(np.uint16) == oracle.lthash(host, off)).all()
    assert (narrow.cpu().numpy().view(np.uint16) == oracle.lthash32(host, off)).all()


def test_bad_arguments():
    out = torch.zeros(1024, dtype=torch.int16, device="cuda")
    for call in (lambda: sentry.sentry_lthash_fixed(0, 100, 5, out.data_ptr()),
                 lambda: sentry.sentry_lthash32_fixed(0x1000, 100, 5, 0),
                 lambda: sentry.sentry_lthash_fixed(0x1000, 1 << 62, 8, out.data_ptr()),
                 lambda: sentry.sentry_lthash_fixed(0x1000, 1, 1 << 30, out.data_ptr())):
        with pytest.raises(sentry.SentryError) as e:
            call()
        assert e.value.code == sentry.ERR_INVALID_ARG

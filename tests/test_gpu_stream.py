"""GPU parity for the chunked and host-streaming entry points."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("total,leaf,chunks", [
    (4096 * 10 + 100, 4096, [4096 * 4, 4096 * 6 + 100]),
    (4096 * 10, 4096, [4096] * 10),
    (64 * 1000 + 1, 64, [64 * 256, 64 * 300, 64 * 444 + 1]),
    (100, 4096, [100]),
    (0, 64, []),
])
def test_stream_api_equals_one_shot(total, leaf, chunks):
    buf = wl.uniform_bytes(2000 + total % 13, 0, total)
    want = oracle.merkle_root(buf, leaf)
    st = sentry.sentry_merkle_stream_begin(total, leaf)
    pos = 0
    keep = []
    for c in chunks:
        d = to_dev(buf[pos:pos + c])
        keep.append(d)
        sentry.sentry_merkle_stream_update(st, d.data_ptr(), c)
        pos += c
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_stream_final(st, out.data_ptr())
    torch.cuda.synchronize()
    assert bytes(out.cpu().numpy()) == want


def test_stream_api_misuse():
    st = sentry.sentry_merkle_stream_begin(4096 * 4, 4096)
    d = torch.zeros(4096 * 4, dtype=torch.uint8, device="cuda")
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_stream_update(st, d.data_ptr(), 4096 + 64)   # only the last chunk may end inside a leaf
    sentry.sentry_merkle_stream_update(st, d.data_ptr(), 4096)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_stream_final(st, out.data_ptr())             # not everything fed
    sentry.sentry_merkle_stream_abort(st)
    st = sentry.sentry_merkle_stream_begin(4096, 4096)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_stream_update(st, d.data_ptr(), 8192)        # more than announced
    sentry.sentry_merkle_stream_abort(st)


@pytest.mark.parametrize("total,leaf,chunk", [
    (1 << 22, 4096, 1 << 20), ((1 << 22) + 4096 * 3 + 5, 4096, 1 << 20), (1 << 20, 65536, 1 << 22),
    (64 * 700, 64, 64 * 256), (0, 64, 64),
])
def test_merkle_root_h2d(total, leaf, chunk):
    buf = wl.uniform_bytes(2100, 0, total)
    want = oracle.merkle_root(buf, leaf)
    host = torch.zeros(max(total, 16), dtype=torch.uint8).pin_memory()
    host[:total] = torch.from_numpy(buf)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    s = torch.cuda.Stream()
    for stream in (0, s.cuda_stream):
        out.zero_()
        torch.cuda.synchronize()
        sentry.sentry_merkle_root_h2d(host.data_ptr(), total, leaf, chunk, out.data_ptr(), stream)
        torch.cuda.synchronize()
        assert bytes(out.cpu().numpy()) == want
    assert (host[:total].numpy() == buf).all()


def test_lthash_h2d_batches_and_running_sum():
    lens = wl.lognormal_record_lengths(400, seed=99, median=20_000, lo=100, hi=200_000)
    lens[5] = 0
    off = wl.offsets_from_lengths(lens)
    total = int(off[-1])
    data = wl.uniform_bytes(2200, 0, total)
    want = oracle.lthash(data, off)
    host = torch.zeros(total + 1, dtype=torch.uint8).pin_memory()
    for shift in (0, 1):                     # the host buffer need not be aligned either
        host[shift:shift + total] = torch.from_numpy(data)
        hoff = torch.from_numpy(off.view(np.int64)).pin_memory()
        out = torch.full((1024,), 0x1111, dtype=torch.int16, device="cuda")
        for batch in (1 << 20, 300_000, total + 5):
            sentry.sentry_lthash_h2d(host.data_ptr() + shift, hoff.data_ptr(), 400, batch, out.data_ptr())
            torch.cuda.synchronize()
            assert (out.cpu().numpy().view(np.uint16) == want).all(), (shift, batch)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_lthash_h2d(host.data_ptr(), hoff.data_ptr(), 400, 1000, out.data_ptr())
    # running sum across calls (one call per dataset batch) = one call over everything
    acc = torch.zeros(1024, dtype=torch.int16, device="cuda")
    part = torch.zeros(1024, dtype=torch.int16, device="cuda")
    host[:total] = torch.from_numpy(data)
    for a, b in ((0, 150), (150, 400)):
        sub = torch.from_numpy(off[a:b + 1].view(np.int64).copy()).pin_memory()
        sentry.sentry_lthash_h2d(host.data_ptr(), sub.data_ptr(), b - a, 1 << 20, part.data_ptr())
        sentry.sentry_lthash_combine(acc.data_ptr(), part.data_ptr())
    torch.cuda.synchronize()
    assert (acc.cpu().numpy().view(np.uint16) == want).all()


def test_h2d_from_pageable_pinned_and_device_memory():
    # pinned memory is read by the load kernel, pageable memory goes through hipMemcpyAsync,
    # and a device pointer in place of the host buffer is accepted as well
    total, leaf, chunk = 64 * 5000 + 37, 64, 64 * 512
    buf = wl.uniform_bytes(2300, 0, total)
    want = oracle.merkle_root(buf, leaf)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    pageable = np.zeros(total + 64, dtype=np.uint8)
    base = (-pageable.ctypes.data) % 16                      # numpy gives no 16-byte guarantee
    pageable[base:base + total] = buf
    pinned = torch.from_numpy(buf.copy()).pin_memory()
    device = to_dev(buf)
    for name, ptr in (("pageable", pageable.ctypes.data + base), ("pinned", pinned.data_ptr()), ("device", device.data_ptr())):
        out.zero_()
        sentry.sentry_merkle_root_h2d(ptr, total, leaf, chunk, out.data_ptr())
        torch.cuda.synchronize()
        assert bytes(out.cpu().numpy()) == want, name

    lens = wl.lognormal_record_lengths(300, seed=7, median=3_000, lo=0, hi=40_000)
    off = wl.offsets_from_lengths(lens)
    n_bytes = int(off[-1])
    data = wl.uniform_bytes(2310, 0, n_bytes)
    want_l = oracle.lthash(data, off)
    lanes = torch.zeros(1024, dtype=torch.int16, device="cuda")
    hoff = off.copy()                                         # pageable offsets
    pg = np.zeros(n_bytes + 32, dtype=np.uint8)
    pin = torch.zeros(n_bytes + 32, dtype=torch.uint8).pin_memory()
    for shift in (0, 3, 15, 16):
        pg[shift:shift + n_bytes] = data
        pin[shift:shift + n_bytes] = torch.from_numpy(data)
        for name, ptr in (("pageable", pg.ctypes.data + shift), ("pinned", pin.data_ptr() + shift)):
            for batch in (50_000, 77_777, n_bytes):
                lanes.zero_()
                sentry.sentry_lthash_h2d(ptr, hoff.ctypes.data, 300, batch, lanes.data_ptr())
                torch.cuda.synchronize()
                assert (lanes.cpu().numpy().view(np.uint16) == want_l).all(), (name, shift, batch)
    # offsets that do not start at 0: only [offsets[0], offsets[n]) of the buffer is touched
    sub = off[100:251].copy()
    want_sub = oracle.lthash(data[int(sub[0]):int(sub[-1])], sub - sub[0])
    pin[:n_bytes] = torch.from_numpy(data)
    sentry.sentry_lthash_h2d(pin.data_ptr(), sub.ctypes.data, 150, 60_000, lanes.data_ptr())
    torch.cuda.synchronize()
    assert (lanes.cpu().numpy().view(np.uint16) == want_sub).all()

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

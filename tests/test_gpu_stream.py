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


@pytest.mark.parametrize("total,leaf,chunks,pinned", [
    (4096 * 10 + 100, 4096, [4096 * 4, 4096 * 6 + 100], True),
    (4096 * 12, 4096, [4096] * 12, True),                       # both staging buffers reused many times
    (64 * 1000 + 1, 64, [64 * 256, 64 * 300, 64 * 444 + 1], True),
    ((3 << 20) + 77, 65536, [1 << 20, 1 << 16, 1 << 20, (1 << 20) - (1 << 16) + 77], True),   # growing and shrinking chunks
    (4096 * 10 + 100, 4096, [4096 * 4, 4096 * 6 + 100], False),  # pageable host memory
    (100, 4096, [100], True),
])
def test_stream_update_h2d_equals_one_shot(total, leaf, chunks, pinned):
    buf = wl.uniform_bytes(2050 + total % 13, 0, total)
    want = oracle.merkle_root(buf, leaf)
    host = torch.from_numpy(buf.copy())
    if pinned:
        host = host.pin_memory()
    s = torch.cuda.Stream()
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()     # torch fills `out` on its own stream, which s does not wait for
    st = sentry.sentry_merkle_stream_begin(total, leaf)
    pos = 0
    for c in chunks:      # fed back to back, no host wait in between: the chunks stay in place
        sentry.sentry_merkle_stream_update_h2d(st, host.data_ptr() + pos, c, s.cuda_stream)
        pos += c
    sentry.sentry_merkle_stream_final(st, out.data_ptr(), s.cuda_stream)
    torch.cuda.synchronize()
    assert bytes(out.cpu().numpy()) == want


def test_stream_update_h2d_mixed_with_device_chunks_and_two_trees_on_one_stream():
    # two trees fed in turn on one stream share that stream's two staging buffers; one of them also
    # takes a chunk that is already on the device
    leaf = 4096
    bufs = [wl.uniform_bytes(2060 + i, 0, leaf * 9 + 11 * i) for i in range(2)]
    hosts = [torch.from_numpy(b.copy()).pin_memory() for b in bufs]
    dev1 = to_dev(bufs[1][leaf * 3:leaf * 6])
    sts = [sentry.sentry_merkle_stream_begin(b.size, leaf) for b in bufs]
    for part in range(3):
        lo = leaf * 3 * part
        for i in range(2):
            n = (bufs[i].size - lo) if part == 2 else leaf * 3
            if i == 1 and part == 1:
                sentry.sentry_merkle_stream_update(sts[i], dev1.data_ptr(), n)
            else:
                sentry.sentry_merkle_stream_update_h2d(sts[i], hosts[i].data_ptr() + lo, n)
    outs = [torch.zeros(32, dtype=torch.uint8, device="cuda") for _ in range(2)]
    for i in range(2):
        sentry.sentry_merkle_stream_final(sts[i], outs[i].data_ptr())
    torch.cuda.synchronize()
    for i in range(2):
        assert bytes(outs[i].cpu().numpy()) == oracle.merkle_root(bufs[i], leaf), i


def test_merkle_root_h2d_in_the_shape_of_config_5():
    # 64 KiB leaves, 1 GiB chunks, three chunks and a ragged fourth from pinned memory, so that both
    # staging buffers are used twice; no host synchronisation while the call's pipeline runs
    leaf, chunk = 64 << 10, 1 << 30
    total = 3 * chunk + 5 * leaf + 12345
    d = wl.uniform_bytes(2070, 0, total, device="cuda")
    host = torch.empty(total, dtype=torch.uint8).pin_memory()
    host.copy_(d)
    a = torch.zeros(32, dtype=torch.uint8, device="cuda")
    b = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_root_h2d(host.data_ptr(), total, leaf, chunk, a.data_ptr())
    sentry.sentry_merkle_root(d.data_ptr(), total, leaf, b.data_ptr())
    torch.cuda.synchronize()
    assert bytes(a.cpu().numpy()) == bytes(b.cpu().numpy())
    # and against the oracle on the leaves it can afford: first, last (ragged) and one across a chunk seam
    leaves = torch.zeros(32, dtype=torch.uint8, device="cuda")
    for i in (0, chunk // leaf, total // leaf):
        n = min(leaf, total - i * leaf)
        sentry.sentry_merkle_leaves(d.data_ptr() + i * leaf, n, leaf, leaves.data_ptr())
        torch.cuda.synchronize()
        assert bytes(leaves.cpu().numpy()) == oracle.sha256(d[i * leaf:i * leaf + n].cpu().numpy()), i
    del d, host


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
    h = torch.zeros(8192, dtype=torch.uint8).pin_memory()
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_stream_update_h2d(st, h.data_ptr(), 8192)    # more than announced, host chunk
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_stream_update_h2d(st, h.data_ptr() + 8, 4096)    # misaligned host chunk
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


@pytest.mark.parametrize("pinned", [True, False])
def test_lthash_stream_running_sum_over_batches_fed_one_by_one(pinned):
    # 13 batches of unequal sizes (one empty, one of a single empty record) fed back to back on a
    # stream of their own with no host wait in between: every staging slot and every hash stream is
    # reused several times and the staging buffers grow while batches are in flight
    lens = wl.lognormal_record_lengths(1300, seed=101, median=9_000, lo=0, hi=300_000)
    lens[700] = 0
    off = wl.offsets_from_lengths(lens)
    total = int(off[-1])
    data = wl.uniform_bytes(2400, 0, total)
    want = oracle.lthash(data, off)
    host = torch.from_numpy(data.copy())
    hoff = torch.from_numpy(off.view(np.int64).copy())
    if pinned:
        host, hoff = host.pin_memory(), hoff.pin_memory()
    cuts = [0, 10, 11, 11, 300, 350, 700, 701, 900, 901, 1000, 1100, 1250, 1300]
    s = torch.cuda.Stream()
    out = torch.full((1024,), 0x2222, dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()     # torch fills `out` on its own stream, which s does not wait for
    st = sentry.sentry_lthash_stream_begin()
    for a, b in zip(cuts[:-1], cuts[1:]):
        sentry.sentry_lthash_stream_update_h2d(st, host.data_ptr(), hoff.data_ptr() + 8 * a, b - a, s.cuda_stream)
    sentry.sentry_lthash_stream_final(st, out.data_ptr(), s.cuda_stream)
    torch.cuda.synchronize()
    assert (out.cpu().numpy().view(np.uint16) == want).all()
    # a second running sum on the same stream right after, two batches; and an empty one
    st = sentry.sentry_lthash_stream_begin()
    sentry.sentry_lthash_stream_update_h2d(st, host.data_ptr(), hoff.data_ptr() + 8 * 300, 400, s.cuda_stream)
    sentry.sentry_lthash_stream_update_h2d(st, host.data_ptr(), hoff.data_ptr(), 300, s.cuda_stream)
    sentry.sentry_lthash_stream_final(st, out.data_ptr(), s.cuda_stream)
    torch.cuda.synchronize()
    assert (out.cpu().numpy().view(np.uint16) == oracle.lthash(data[:int(off[700])], off[:701])).all()
    st = sentry.sentry_lthash_stream_begin()
    sentry.sentry_lthash_stream_final(st, out.data_ptr(), s.cuda_stream)
    torch.cuda.synchronize()
    assert (out.cpu() == 0).all()


@pytest.mark.parametrize("narrow", [False, True])
def test_lthash_stream_batches_of_one_record_size_need_no_offsets_on_the_device(narrow):
    # batches in which every record has one size take the call without offsets (the host sees it);
    # here they alternate with batches of mixed sizes inside one running sum: 3072-byte samples
    # (one lane per record), 70 records of 40,000 bytes (four lanes), a batch of empty records, a
    # batch of one record, and a batch that is equal but for its last record (the ordinary path)
    lens = np.concatenate([
        np.full(500, 3072), wl.lognormal_record_lengths(200, seed=5, median=5000, lo=0, hi=60_000),
        np.full(70, 40_000), np.zeros(9, dtype=np.int64), [777], np.full(40, 1000), [1001], np.full(64, 129)]).astype(np.int64)
    cuts = np.cumsum([0, 500, 200, 70, 9, 1, 41, 64])
    off = wl.offsets_from_lengths(lens)
    data = wl.uniform_bytes(2500, 0, int(off[-1]))
    want = (oracle.lthash32 if narrow else oracle.lthash)(data, off)
    # the records start 3 bytes into the host buffer: staging keeps that alignment modulo 16
    host = torch.zeros(int(off[-1]) + 3, dtype=torch.uint8).pin_memory()
    host[3:] = torch.from_numpy(data.copy())
    hoff = torch.from_numpy(off.view(np.int64).copy())
    s = torch.cuda.Stream()
    out = torch.full((1024,), 0x3333, dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    for _ in range(2):      # the second running sum finds the staging buffers as the first left them
        st = (sentry.sentry_lthash32_stream_begin if narrow else sentry.sentry_lthash_stream_begin)()
        for a, b in zip(cuts[:-1], cuts[1:]):
            sentry.sentry_lthash_stream_update_h2d(st, host.data_ptr() + 3, hoff.data_ptr() + 8 * int(a), int(b - a), s.cuda_stream)
        sentry.sentry_lthash_stream_final(st, out.data_ptr(), s.cuda_stream)
        torch.cuda.synchronize()
        got = out.cpu().numpy().view(np.uint16)
        assert (got[:len(want)] == want).all()
        out.fill_(0x3333)
        torch.cuda.synchronize()


def test_lthash_stream_misuse():
    st = sentry.sentry_lthash_stream_begin()
    h = torch.zeros(4096, dtype=torch.uint8).pin_memory()
    o = torch.tensor([0, 100, 50], dtype=torch.int64).pin_memory()
    with pytest.raises(sentry.SentryError):
        sentry.sentry_lthash_stream_update_h2d(st, h.data_ptr(), 0, 2)                 # NULL offsets
    with pytest.raises(sentry.SentryError):
        sentry.sentry_lthash_stream_update_h2d(st, h.data_ptr(), o.data_ptr() + 4, 2)  # misaligned offsets
    with pytest.raises(sentry.SentryError):
        sentry.sentry_lthash_stream_final(st, 0)                                       # NULL lanes
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    sentry.sentry_lthash_stream_update_h2d(st, h.data_ptr(), o.data_ptr(), 1, s1.cuda_stream)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_lthash_stream_update_h2d(st, h.data_ptr(), o.data_ptr(), 1, s2.cuda_stream)   # another stream
    sentry.sentry_lthash_stream_abort(st)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_lthash_stream_update_h2d(None, h.data_ptr(), o.data_ptr(), 1)


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

"""GPU tests of the library's run-time plumbing: scratch that grows and shrinks between calls,
calls on several streams and from several host threads, release and reuse of the scratch,
error reporting.  Every result is still checked against the CPU oracle."""
import threading

import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import to_dev

pytestmark = pytest.mark.gpu


def _records(seed, n, lo, hi):
    rng = np.random.default_rng(seed)
    lens = rng.integers(lo, hi, size=n)
    off = np.zeros(n + 1, dtype=np.uint64)
    off[1:] = np.cumsum(lens)
    return wl.uniform_bytes(seed, 0, int(off[-1])), off


def test_scratch_grows_and_is_reused_with_smaller_inputs():
    s = torch.cuda.Stream()
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    lanes = torch.zeros(1024, dtype=torch.int16, device="cuda")
    # sizes go up and down so that every scratch region is regrown while earlier work of the
    # same stream may still be in flight, then reused with stale contents from a larger call
    for n_leaves in (3, 70_000, 600, 300_000, 5, 70_000):
        buf = wl.uniform_bytes(900 + n_leaves, 0, 64 * n_leaves - 7)
        d = to_dev(buf)
        sentry.sentry_merkle_root(d.data_ptr(), buf.size, 64, out.data_ptr(), s.cuda_stream)
        s.synchronize()
        assert bytes(out.cpu().numpy()) == oracle.merkle_root(buf, 64), n_leaves
    for n in (10, 5000, 40, 20_000, 1):
        data, off = _records(910 + n, n, 0, 300)
        dd, do = to_dev(data), to_dev(off)
        sentry.sentry_lthash(dd.data_ptr(), do.data_ptr(), n, lanes.data_ptr(), s.cuda_stream)
        s.synchronize()
        assert (lanes.cpu().numpy().view(np.uint16) == oracle.lthash(data, off)).all(), n


def test_calls_interleaved_on_two_streams():
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    bufs = [wl.uniform_bytes(920 + i, 0, 4096 * (300 + 37 * i) + 11 * i) for i in range(6)]
    devs = [to_dev(b) for b in bufs]
    outs = torch.zeros(len(bufs), 32, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for i, (b, d) in enumerate(zip(bufs, devs)):   # nothing waits between the calls
        st = (s1, s2)[i & 1]
        sentry.sentry_merkle_root(d.data_ptr(), b.size, 4096, outs[i].data_ptr(), st.cuda_stream)
    torch.cuda.synchronize()
    got = outs.cpu().numpy()
    for i, b in enumerate(bufs):
        assert bytes(got[i]) == oracle.merkle_root(b, 4096), i


def test_host_threads_with_a_stream_each():
    n_threads = 4
    work = []
    for t in range(n_threads):
        buf = wl.uniform_bytes(930 + t, 0, 1024 * (2000 + 100 * t) + t)
        data, off = _records(940 + t, 3000 + 10 * t, 0, 500)
        work.append((buf, data, off))
    staged = [(to_dev(b), to_dev(d), to_dev(o)) for b, d, o in work]
    roots = torch.zeros(n_threads, 32, dtype=torch.uint8, device="cuda")
    lanes = torch.zeros(n_threads, 1024, dtype=torch.int16, device="cuda")
    # per-source sums too: every stream has tables, counters and tickets of its own
    srcs = [wl.dirichlet_source_ids(len(w[2]) - 1, 5 + t, 945 + t) for t, w in enumerate(work)]
    d_srcs = [to_dev(x.view(np.int32)) for x in srcs]
    sums = [torch.zeros((5 + t) * 1024, dtype=torch.int16, device="cuda") for t in range(n_threads)]
    streams = [torch.cuda.Stream() for _ in range(n_threads)]
    torch.cuda.synchronize()
    errors = []

    def run(t):
        try:
            db, dd, do = staged[t]
            st = streams[t].cuda_stream
            for _ in range(3):
                sentry.sentry_merkle_root(db.data_ptr(), work[t][0].size, 1024, roots[t].data_ptr(), st)
                sentry.sentry_lthash(dd.data_ptr(), do.data_ptr(), len(work[t][2]) - 1, lanes[t].data_ptr(), st)
                sentry.sentry_lthash_sources(dd.data_ptr(), do.data_ptr(), d_srcs[t].data_ptr(), len(work[t][2]) - 1, 5 + t,
                                             sums[t].data_ptr(), st)
            streams[t].synchronize()
        except Exception as e:   # reported in the main thread
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=run, args=(t,)) for t in range(n_threads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    torch.cuda.synchronize()
    r, l = roots.cpu().numpy(), lanes.cpu().numpy().view(np.uint16)
    for t, (buf, data, off) in enumerate(work):
        assert bytes(r[t]) == oracle.merkle_root(buf, 1024), t
        assert (l[t] == oracle.lthash(data, off)).all(), t
        one = oracle.lthash_sources(data, off, srcs[t], 5 + t).astype(np.uint32)
        assert (sums[t].cpu().numpy().view(np.uint16).reshape(5 + t, 1024) == ((3 * one) & 0xFFFF)).all(), t


def test_release_scratch_then_reuse():
    buf = wl.uniform_bytes(950, 0, 64 * 5000 + 3)
    d = to_dev(buf)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    want = oracle.merkle_root(buf, 64)
    for _ in range(2):
        sentry.sentry_merkle_root(d.data_ptr(), buf.size, 64, out.data_ptr())
        torch.cuda.synchronize()
        assert bytes(out.cpu().numpy()) == want
        sentry.sentry_release_scratch()
    # the host-streaming paths own streams and events, which a release destroys as well
    host = torch.from_numpy(buf.copy()).pin_memory()
    for _ in range(2):
        sentry.sentry_merkle_root_h2d(host.data_ptr(), buf.size, 64, 64 * 1024, out.data_ptr())
        torch.cuda.synchronize()
        assert bytes(out.cpu().numpy()) == want
        sentry.sentry_release_scratch()


def test_scratch_bytes_is_the_extra_memory_of_a_scheme():
    # section 5.2 (memory usage): what the library holds for a stream after hashing a model of 40
    # tensors (26 MB) in 8 KiB blocks.  Per layer and in place it is the digests of the workgroups'
    # subtrees and the tables: a few pages, where one digest per block would take 1/256 of the
    # model; coalesced without a buffer it is the gathered blocks on top (at most one per tensor
    # and the padded last one).  Grow-only, the same after a second call, zero after a release.
    lens = [8192 * (5 + 7 * i % 150) + (48 * i) % 8192 for i in range(40)]      # tails of whole 16-byte words
    tensors = [to_dev(wl.uniform_bytes(970 + i, 0, n)) for i, n in enumerate(lens)]
    ptrs = [t.data_ptr() for t in tensors]
    host = [t.cpu().numpy() for t in tensors]
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    roots = torch.zeros(32 * len(lens), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    total = sum(lens)
    seen = {}
    sentry.sentry_release_scratch()      # torch hands out streams from a pool: one may have served an earlier test
    for name, call in (
            ("per layer", lambda st: sentry.sentry_merkle_segments(ptrs, lens, 8192, roots.data_ptr(), out.data_ptr(), st)),
            ("in place", lambda st: sentry.sentry_merkle_inplace(ptrs, lens, 8192, out.data_ptr(), st)),
            ("coalesced", lambda st: sentry.sentry_merkle_coalesced(ptrs, lens, 8192, 0, 0, out.data_ptr(), st))):
        s = torch.cuda.Stream()
        assert sentry.sentry_scratch_bytes(s.cuda_stream) == (0, 0)
        call(s.cuda_stream)
        s.synchronize()
        dev, pinned = sentry.sentry_scratch_bytes(s.cuda_stream)
        call(s.cuda_stream)
        s.synchronize()
        assert sentry.sentry_scratch_bytes(s.cuda_stream) == (dev, pinned)
        assert 0 < dev and 0 < pinned <= 64 * 1024
        seen[name] = dev
    assert bytes(out.cpu().numpy()) == oracle.merkle_coalesced_h(sentry.HASH_SHA256, host, 8192)
    # (every region is a whole number of 4 KiB pages: that is what shows on a model this small)
    assert seen["per layer"] < 40 * 4096 + total // 2048 and seen["in place"] < 40 * 4096 + total // 2048
    gathered, _, _ = sentry.sentry_merkle_coalesced_plan(ptrs, lens, 8192)
    assert gathered <= 8192 * (len(lens) + 1)
    assert seen["coalesced"] <= seen["in place"] + gathered + 3 * 4096 + 64 * 1024
    sentry.sentry_release_scratch()
    assert sentry.sentry_scratch_bytes(0) == (0, 0)


def test_error_text_names_the_argument_and_later_calls_still_work():
    buf = wl.uniform_bytes(960, 0, 4096)
    d = to_dev(buf)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    with pytest.raises(sentry.SentryError) as e:
        sentry.sentry_merkle_root(d.data_ptr(), buf.size, 100, out.data_ptr())
    assert e.value.code == sentry.ERR_INVALID_ARG and "leaf_bytes" in str(e.value)
    with pytest.raises(sentry.SentryError) as e:
        sentry.sentry_merkle_root(d.data_ptr() + 4, buf.size - 4, 64, out.data_ptr())
    assert "aligned" in str(e.value)
    sentry.sentry_merkle_root(d.data_ptr(), buf.size, 64, out.data_ptr())
    torch.cuda.synchronize()
    assert bytes(out.cpu().numpy()) == oracle.merkle_root(buf, 64)
    assert sentry.sentry_last_error() == ""


def test_h2d_pipeline_with_many_streams_alive():
    # HIP maps streams onto a few hardware queues; with dozens of streams alive the library's side
    # streams share queues with the caller's stream.  Kernels of streams on one queue still run
    # side by side, copies do not, which is one reason the loads are kernels; results are the same
    # either way, the time is printed for the record.
    import time
    streams = [torch.cuda.Stream() for _ in range(40)]          # fills torch's stream pool
    total, leaf, chunk = 1 << 28, 65536, 1 << 25
    buf = wl.uniform_bytes(970, 0, total)
    want = oracle.merkle_root(buf, leaf)
    host = torch.from_numpy(buf).pin_memory()
    stage = torch.empty(total, dtype=torch.uint8, device="cuda")
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    lens = wl.lognormal_record_lengths(2000, seed=5, median=100_000, lo=1000, hi=400_000)
    off = wl.offsets_from_lengths(lens)
    lt_total = int(off[-1])
    data = wl.uniform_bytes(971, 0, lt_total)
    want_l = oracle.lthash(data, off)
    lhost = torch.from_numpy(data).pin_memory()
    lanes = torch.zeros(1024, dtype=torch.int16, device="cuda")

    def wall(fn):
        torch.cuda.synchronize()
        t = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t)

    t_copy = min(wall(lambda: stage.copy_(host, non_blocking=True)) for _ in range(3))
    for s in [torch.cuda.default_stream()] + streams[:6]:
        out.zero_()
        with torch.cuda.stream(s):
            sentry.sentry_merkle_root_h2d(host.data_ptr(), total, leaf, chunk, out.data_ptr(), s.cuda_stream)   # creates the streams
            t = min(wall(lambda: sentry.sentry_merkle_root_h2d(host.data_ptr(), total, leaf, chunk, out.data_ptr(),
                                                               s.cuda_stream)) for _ in range(2))
        assert bytes(out.cpu().numpy()) == want
        print("merkle_h2d on stream %#x: %.2f ms (plain copy %.2f ms)" % (s.cuda_stream, t, t_copy))
    for s in [torch.cuda.default_stream()] + streams[6:9]:
        lanes.zero_()
        sentry.sentry_lthash_h2d(lhost.data_ptr(), off.ctypes.data, 2000, 1 << 25, lanes.data_ptr(), s.cuda_stream)
        torch.cuda.synchronize()
        assert (lanes.cpu().numpy().view(np.uint16) == want_l).all()


@pytest.mark.parametrize("schedule", ["overlap", "pair", "serial"])
def test_bench_quick_run_prints_one_valid_line(schedule):
    # bench.py at 1/64 size in a process of its own: one JSON line with the fields the contract
    # names; the run itself checks the overlapped parts against the same calls run alone and the
    # GPU against the oracle on the CPU-baseline sample
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--quick", "--steps", "2", "--warmup", "1",
                        "--schedule", schedule], capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["value"] > 0 and d["config"]["workload"].startswith("QUICK")
    assert d["roofline"]["bound"] == "alu" and 0 < d["roofline"]["frac"] and d["roofline"]["shares_the_chip"] == (schedule == "overlap")
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["cores"] == 1
    # no entry runs faster than the chip can issue its instruction mix, nor than HBM can feed it
    r = d["roofline"]
    assert r["issue_bound"] > 0 and 0 < r["issue_frac"] <= 1 and 0 < r["whole_step"]["issue_frac"] <= 1
    assert r["alone"]["issue_frac"] <= 1
    assert set(r["issue_rates_TOP/s"]["this_run"]) == set(r["issue_rates_TOP/s"]["table"])
    for name, e in d["per_config"].items():
        assert 0 < e["issue_frac"] <= 1 and 0 < e["hbm_frac"] <= 1 and e["alu_frac"] <= e["issue_bound_TOP/s"] / 39.3, name


def test_calls_can_be_captured_in_a_graph_and_replayed():
    # once a stream's scratch has its size (one eager call), the calls only launch kernels, so a
    # caller may capture them; every replay is checked against the oracle, with the inputs
    # rewritten, other work of the library and synchronisations between the replays
    s = torch.cuda.Stream()
    n_bytes, leaf, n_rec = 4096 * 700 + 100, 4096, 3000
    buf = torch.zeros(n_bytes, dtype=torch.uint8, device="cuda")
    data0, off = _records(980, n_rec, 0, 2000)
    rec = torch.zeros(data0.size, dtype=torch.uint8, device="cuda")
    d_off = to_dev(off)
    root = torch.zeros(32, dtype=torch.uint8, device="cuda")
    lanes = torch.zeros(1024, dtype=torch.int16, device="cuda")
    lanes32 = torch.zeros(32, dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()     # torch fills these on its own stream, which s does not wait for

    def calls():
        sentry.sentry_merkle_root(buf.data_ptr(), n_bytes, leaf, root.data_ptr(), s.cuda_stream)
        sentry.sentry_lthash(rec.data_ptr(), d_off.data_ptr(), n_rec, lanes.data_ptr(), s.cuda_stream)
        sentry.sentry_lthash_combine(lanes.data_ptr(), lanes.data_ptr(), s.cuda_stream)    # lanes doubled
        sentry.sentry_lthash32(rec.data_ptr(), d_off.data_ptr(), n_rec, lanes32.data_ptr(), s.cuda_stream)
        sentry.sentry_lthash32_combine(lanes32.data_ptr(), lanes32.data_ptr(), s.cuda_stream)

    with torch.cuda.stream(s):
        calls()
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        calls()
    other = wl.uniform_bytes(981, 0, 64 * 900)
    d_other, out_other = to_dev(other), torch.zeros(32, dtype=torch.uint8, device="cuda")
    for k in range(4):
        b = wl.uniform_bytes(990 + k, 0, n_bytes)
        r = wl.uniform_bytes(995 + k, 0, data0.size)
        buf.copy_(torch.from_numpy(b))
        rec.copy_(torch.from_numpy(r))
        root.zero_()
        lanes.zero_()
        lanes32.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert bytes(root.cpu().numpy()) == oracle.merkle_root(b, leaf), k
        one = oracle.lthash(r, off)
        assert (lanes.cpu().numpy().view(np.uint16) == oracle.lthash_combine(one, one)).all(), k
        one32 = oracle.lthash32(r, off)
        assert (lanes32.cpu().numpy().view(np.uint16) == oracle.lanes_add(one32, one32)).all(), k
        # eager work of the library between the replays, on another stream
        sentry.sentry_merkle_root(d_other.data_ptr(), other.size, 64, out_other.data_ptr())
        torch.cuda.synchronize()
        assert bytes(out_other.cpu().numpy()) == oracle.merkle_root(other, 64)


def test_reserved_scratch_makes_the_first_calls_on_a_stream_fit_for_capture():
    # a fresh stream has no scratch: without the reservation the first call would allocate, which a
    # capturing stream does not allow; with it the very first calls on the stream are captured
    n_bytes, leaf, n_rec = 64 * 70_000 + 9, 64, 5000
    buf_np = wl.uniform_bytes(1200, 0, n_bytes)
    data, off = _records(1201, n_rec, 0, 900)
    buf, rec, d_off = to_dev(buf_np), to_dev(data), to_dev(off)
    root = torch.zeros(32, dtype=torch.uint8, device="cuda")
    leaves = torch.zeros(32 * 70_001, dtype=torch.uint8, device="cuda")
    root2 = torch.zeros(32, dtype=torch.uint8, device="cuda")
    lanes = torch.zeros(1024, dtype=torch.int16, device="cuda")
    lanes32 = torch.zeros(32, dtype=torch.int16, device="cuda")
    rows = torch.zeros(n_rec * 1024, dtype=torch.int16, device="cuda")
    summed = torch.zeros(1024, dtype=torch.int16, device="cuda")
    fixed = torch.zeros(1024, dtype=torch.int16, device="cuda")
    # code objects are loaded by a first launch: make those on the default stream, with tiny inputs
    sentry.sentry_merkle_root(buf.data_ptr(), 64 * 700, leaf, root.data_ptr())
    sentry.sentry_merkle_root(buf.data_ptr(), 64 * 70_000, leaf, root.data_ptr())
    sentry.sentry_merkle_leaves(buf.data_ptr(), 640, leaf, leaves.data_ptr())
    sentry.sentry_merkle_reduce(leaves.data_ptr(), 10, root2.data_ptr())
    sentry.sentry_lthash(rec.data_ptr(), d_off.data_ptr(), 40_000 if n_rec > 40_000 else n_rec, lanes.data_ptr())
    sentry.sentry_lthash32(rec.data_ptr(), d_off.data_ptr(), 10, lanes32.data_ptr())
    sentry.sentry_lthash_digests(rec.data_ptr(), d_off.data_ptr(), 10, rows.data_ptr())
    sentry.sentry_lthash_sum(rows.data_ptr(), 10, summed.data_ptr())
    sentry.sentry_lthash_fixed(rec.data_ptr(), 100, 10, fixed.data_ptr())
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    sentry.sentry_reserve_scratch(n_bytes, leaf, n_rec, s.cuda_stream)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        sentry.sentry_merkle_root(buf.data_ptr(), n_bytes, leaf, root.data_ptr(), s.cuda_stream)
        sentry.sentry_merkle_leaves(buf.data_ptr(), n_bytes, leaf, leaves.data_ptr(), s.cuda_stream)
        sentry.sentry_merkle_reduce(leaves.data_ptr(), 70_001, root2.data_ptr(), s.cuda_stream)
        sentry.sentry_lthash(rec.data_ptr(), d_off.data_ptr(), n_rec, lanes.data_ptr(), s.cuda_stream)
        sentry.sentry_lthash32(rec.data_ptr(), d_off.data_ptr(), n_rec, lanes32.data_ptr(), s.cuda_stream)
        sentry.sentry_lthash_digests(rec.data_ptr(), d_off.data_ptr(), n_rec, rows.data_ptr(), s.cuda_stream)
        sentry.sentry_lthash_sum(rows.data_ptr(), n_rec, summed.data_ptr(), s.cuda_stream)
        sentry.sentry_lthash_fixed(rec.data_ptr(), 100, n_rec, fixed.data_ptr(), s.cuda_stream)
    want_root = oracle.merkle_root(buf_np, leaf)
    want_lanes = oracle.lthash(data, off)
    want_fixed = oracle.lthash(data[:100 * n_rec], np.arange(n_rec + 1, dtype=np.uint64) * np.uint64(100))
    for k in range(2):
        for t in (root, root2, lanes, lanes32, summed, fixed):
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert bytes(root.cpu().numpy()) == want_root and bytes(root2.cpu().numpy()) == want_root, k
        assert (lanes.cpu().numpy().view(np.uint16) == want_lanes).all(), k
        assert (summed.cpu().numpy().view(np.uint16) == want_lanes).all(), k
        assert (lanes32.cpu().numpy().view(np.uint16) == oracle.lthash32(data, off)).all(), k
        assert (fixed.cpu().numpy().view(np.uint16) == want_fixed).all(), k
    with pytest.raises(sentry.SentryError):
        sentry.sentry_reserve_scratch(1000, 100, 0)

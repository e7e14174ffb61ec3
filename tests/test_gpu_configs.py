"""The five target configurations at full size on the GPU, against expected values that
tests/golden/make_golden.py computed with the CPU oracle on the same synthetic inputs (the
32-partition hash of config 2 is small enough for the oracle to run inside its test)."""
import gc

import numpy as np
import pytest
import torch

import oracle
import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import workloads as wl
from conftest import golden_lines, to_dev

pytestmark = pytest.mark.gpu


def lanes_from_hex(text):
    return np.array([int(x, 16) for x in text.split()], dtype=np.uint16)


def free_gpu():
    gc.collect()
    torch.cuda.empty_cache()


def test_config1_root():
    want = bytes.fromhex(golden_lines("config1_root.txt")[0])
    buf = wl.uniform_bytes(wl.SEED_C1, 0, 16 << 20, device="cuda")
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_root(buf.data_ptr(), buf.numel(), 4096, out.data_ptr())
    torch.cuda.synchronize()
    assert sentry.sentry_verify(bytes(out.cpu().numpy()), want) == 0


def test_config2_lanes_and_halves():
    full, a, b = (lanes_from_hex(x) for x in golden_lines("config2_lanes.txt"))
    data, off = wl.image_records(50_000, device="cuda")
    d_off = to_dev(off)
    out = [torch.zeros(1024, dtype=torch.int16, device="cuda") for _ in range(3)]
    sentry.sentry_lthash(data.data_ptr(), d_off.data_ptr(), 50_000, out[0].data_ptr())
    sentry.sentry_lthash(data.data_ptr(), d_off.data_ptr(), 25_000, out[1].data_ptr())
    sentry.sentry_lthash(data.data_ptr(), d_off.data_ptr() + 8 * 25_000, 25_000, out[2].data_ptr())
    torch.cuda.synchronize()
    got = [o.cpu().numpy().view(np.uint16) for o in out]
    assert (got[0] == full).all() and (got[1] == a).all() and (got[2] == b).all()
    sentry.sentry_lthash_combine(out[1].data_ptr(), out[2].data_ptr())
    torch.cuda.synchronize()
    assert (out[1].cpu().numpy().view(np.uint16) == full).all()


def test_config2_at_the_32_partition_width():
    # the same 50,000 images under the 64-byte digest of section 4.2.2; the oracle hashes them here
    # (0.15 GB of BLAKE2b on one core), whole and in two halves
    data, off = wl.image_records(50_000, device="cuda")
    host = data.cpu().numpy()
    d_off = to_dev(off)
    out = [torch.zeros(32, dtype=torch.int16, device="cuda") for _ in range(3)]
    sentry.sentry_lthash32(data.data_ptr(), d_off.data_ptr(), 50_000, out[0].data_ptr())
    sentry.sentry_lthash32(data.data_ptr(), d_off.data_ptr(), 25_000, out[1].data_ptr())
    sentry.sentry_lthash32(data.data_ptr(), d_off.data_ptr() + 8 * 25_000, 25_000, out[2].data_ptr())
    torch.cuda.synchronize()
    got = [o.cpu().numpy().view(np.uint16) for o in out]
    assert (got[0] == oracle.lthash32(host, off)).all()
    assert (got[1] == oracle.lthash32(host, off[:25_001])).all()
    assert (got[2] == oracle.lthash32(host, off[25_000:])).all()
    sentry.sentry_lthash32_combine(out[1].data_ptr(), out[2].data_ptr())
    torch.cuda.synchronize()
    assert (out[1].cpu().numpy().view(np.uint16) == got[0]).all()
    sentry.sentry_lthash32_remove(out[1].data_ptr(), out[2].data_ptr())
    torch.cuda.synchronize()
    assert (out[1].cpu().numpy().view(np.uint16) == oracle.lthash32(host, off[:25_001])).all()


def test_config3_7b_checkpoint_per_tensor_roots():
    lines = golden_lines("config3_roots.txt")
    want_top = bytes.fromhex(lines[0])
    want_roots = [bytes.fromhex(ln.split()[1]) for ln in lines[1:]]
    lay = wl.layout_7b()
    assert len(want_roots) == len(lay) == 291
    tensors = [wl.checkpoint_tensor(lay, i, base_seed=wl.SEED_C3, device="cuda") for i in range(len(lay))]
    roots = torch.zeros(32 * len(lay), dtype=torch.uint8, device="cuda")
    top = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_segments([t.data_ptr() for t in tensors], [2 * t.numel() for t in tensors], 1 << 20,
                                  roots.data_ptr(), top.data_ptr())
    torch.cuda.synchronize()
    got = roots.cpu().numpy().reshape(len(lay), 32)
    bad = [lay[i][0] for i in range(len(lay)) if bytes(got[i]) != want_roots[i]]
    assert not bad, bad[:5]
    assert bytes(top.cpu().numpy()) == want_top
    del tensors
    free_gpu()


def test_config4_streamed_lattice_hash_with_running_sum():
    lines = golden_lines("config4_lanes.txt")
    want_total = lanes_from_hex(lines[0])
    want_batches = {}
    for ln in lines[1:]:
        _, k, a, b, lanes = ln.split(" ", 4)
        want_batches[int(k)] = (int(a), int(b), lanes_from_hex(lanes))
    off = wl.offsets_from_lengths(wl.lognormal_record_lengths(wl.C4_RECORDS))
    batches = wl.cut_batches(off, wl.C4_BATCH_BYTES)
    assert len(batches) == len(want_batches)
    host = [torch.empty(wl.C4_BATCH_BYTES, dtype=torch.uint8).pin_memory() for _ in range(2)]
    running = torch.zeros(1024, dtype=torch.int16, device="cuda")
    part = torch.zeros(1024, dtype=torch.int16, device="cuda")
    streamed = torch.zeros(1024, dtype=torch.int16, device="cuda")
    lt = sentry.sentry_lthash_stream_begin()          # the same 20 batches, fed whole to one running sum
    narrow = golden_lines("config4_lanes32.txt")      # and to one at the 32-partition width
    want_total32 = lanes_from_hex(narrow[0])
    want_batches32 = [lanes_from_hex(ln.split(" ", 4)[4]) for ln in narrow[1:]]
    lt32 = sentry.sentry_lthash32_stream_begin()
    part32 = torch.zeros(32, dtype=torch.int16, device="cuda")
    streamed32 = torch.zeros(32, dtype=torch.int16, device="cuda")
    offs_keep = []
    for k, (a, b) in enumerate(batches):
        assert (a, b) == want_batches[k][:2]
        nbytes = int(off[b] - off[a])
        dev = wl.uniform_bytes(wl.SEED_C4_BYTES, int(off[a]), nbytes, device="cuda")
        h = host[k & 1]
        h[:nbytes].copy_(dev)                      # the batch now sits in pinned host memory
        del dev
        h_off = torch.from_numpy((off[a:b + 1] - off[a]).view(np.int64).copy())
        # loaded in 1 GB pieces on the side stream while the previous piece is hashed
        sentry.sentry_lthash_h2d(h.data_ptr(), h_off.data_ptr(), b - a, 1_000_000_000, part.data_ptr())
        sentry.sentry_lthash_combine(running.data_ptr(), part.data_ptr())
        sentry.sentry_lthash_stream_update_h2d(lt, h.data_ptr(), h_off.data_ptr(), b - a)
        sentry.sentry_lthash_stream_update_h2d(lt32, h.data_ptr(), h_off.data_ptr(), b - a)
        offs_keep.append(h_off)
        torch.cuda.synchronize()
        assert (part.cpu().numpy().view(np.uint16) == want_batches[k][2]).all(), "batch %d" % k
        if k in (0, 7, len(batches) - 1):          # three batches on their own at the narrow width, resident
            d_off = h_off.cuda()
            dev = h[:nbytes].cuda()
            sentry.sentry_lthash32(dev.data_ptr(), d_off.data_ptr(), b - a, part32.data_ptr())
            torch.cuda.synchronize()
            assert (part32.cpu().numpy().view(np.uint16) == want_batches32[k]).all(), "batch %d, 32 partitions" % k
            del dev
        print("config 4: batch %d/%d ok" % (k + 1, len(batches)), flush=True)
    assert (running.cpu().numpy().view(np.uint16) == want_total).all()
    sentry.sentry_lthash_stream_final(lt, streamed.data_ptr())
    torch.cuda.synchronize()
    assert (streamed.cpu().numpy().view(np.uint16) == want_total).all()
    sentry.sentry_lthash_stream_final(lt32, streamed32.data_ptr())
    torch.cuda.synchronize()
    assert (streamed32.cpu().numpy().view(np.uint16) == want_total32).all()
    del host
    free_gpu()


def test_config5_70b_checkpoint_resident_and_streamed():
    lines = golden_lines("config5_root.txt")
    want = bytes.fromhex(lines[0])
    want_leaves = {int(ln.split()[1]): bytes.fromhex(ln.split()[2]) for ln in lines[1:]}
    lay = wl.layout_70b()
    leaf = 64 << 10
    buf, offs = wl.checkpoint_flat_torch(lay, "cuda", base_seed=wl.SEED_C5)
    total = buf.numel()
    assert total == 137_953_296_384
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    # resident, in the launch configuration bench.py times
    sentry.sentry_merkle_root(buf.data_ptr(), total, leaf, out.data_ptr())
    torch.cuda.synchronize()
    assert sentry.sentry_verify(bytes(out.cpu().numpy()), want) == 0
    # sampled leaf digests
    d = torch.zeros(32, dtype=torch.uint8, device="cuda")
    for i, dig in want_leaves.items():
        n = min(leaf, total - i * leaf)
        sentry.sentry_merkle_leaves(buf.data_ptr() + i * leaf, n, leaf, d.data_ptr())
        torch.cuda.synchronize()
        assert bytes(d.cpu().numpy()) == dig, i
    print("config 5: resident root ok", flush=True)
    # the same checkpoint per tensor (Algorithm 2): 723 roots and the root over them, where the tensors lie
    pt = golden_lines("config5_per_tensor_roots.txt")
    want_top, want_roots = bytes.fromhex(pt[0]), [bytes.fromhex(ln.split()[1]) for ln in pt[1:]]
    assert len(want_roots) == len(lay) == 723
    roots = torch.zeros(32 * len(lay), dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_segments([buf.data_ptr() + offs[i] for i in range(len(lay))],
                                  [offs[i + 1] - offs[i] for i in range(len(lay))], leaf, roots.data_ptr(), out.data_ptr())
    torch.cuda.synchronize()
    got = roots.cpu().numpy().reshape(len(lay), 32)
    bad = [lay[i][0] for i in range(len(lay)) if bytes(got[i]) != want_roots[i]]
    assert not bad, bad[:5]
    assert bytes(out.cpu().numpy()) == want_top
    print("config 5: per-tensor roots ok", flush=True)
    # streamed through the library's own load path: 1 GiB chunks in two pinned host buffers, fed to
    # sentry_merkle_stream_update_h2d, which loads chunk k on its side stream into its own staging
    # buffers while chunk k - 1 is hashed; no host wait per chunk except the one a two-buffer
    # reader needs anyway (buffer b is refilled once the update that read it has passed)
    chunk = 1 << 30
    host = [torch.empty(chunk, dtype=torch.uint8).pin_memory() for _ in range(2)]
    main = torch.cuda.current_stream()
    fill = torch.cuda.Stream()                        # stands in for the reader that fills pinned memory
    loaded = [torch.cuda.Event() for _ in range(2)]   # update k has passed: host[b] may be refilled
    filled = [torch.cuda.Event() for _ in range(2)]
    st = sentry.sentry_merkle_stream_begin(total, leaf)
    pos, k = 0, 0
    while pos < total:
        n = min(chunk, total - pos)
        b = k & 1
        with torch.cuda.stream(fill):
            fill.wait_event(loaded[b])
            host[b][:n].copy_(buf[pos:pos + n], non_blocking=True)
            filled[b].record(fill)
        filled[b].synchronize()                        # the chunk is in host memory: hand it to the library
        sentry.sentry_merkle_stream_update_h2d(st, host[b].data_ptr(), n, main.cuda_stream)
        loaded[b].record(main)
        pos += n
        k += 1
    sentry.sentry_merkle_stream_final(st, out.data_ptr(), main.cuda_stream)
    torch.cuda.synchronize()
    assert k == 129 and sentry.sentry_verify(bytes(out.cpu().numpy()), want) == 0
    print("config 5: streamed root ok (%d chunks)" % k, flush=True)
    del buf, host
    free_gpu()


def test_config3_checkpoint_inplace_flat_tree():
    # the same 291 fragmented tensors, one flat tree over all their blocks (Algorithm 3)
    want = bytes.fromhex(golden_lines("config3_inplace_root.txt")[0])
    lay = wl.layout_7b()
    tensors = [wl.checkpoint_tensor(lay, i, base_seed=wl.SEED_C3, device="cuda") for i in range(len(lay))]
    top = torch.zeros(32, dtype=torch.uint8, device="cuda")
    sentry.sentry_merkle_inplace([t.data_ptr() for t in tensors], [2 * t.numel() for t in tensors], 1 << 20,
                                 top.data_ptr())
    torch.cuda.synchronize()
    assert bytes(top.cpu().numpy()) == want
    del tensors
    free_gpu()


def test_config3_checkpoint_coalesced_tree():
    # the same 291 fragmented tensors as ONE zero-padded byte stream (Algorithm 1): hashed where they lie
    # (only the blocks that span tensors are gathered), and through a coalesced copy in a second buffer
    want = {}
    for ln in golden_lines("config3_coalesced_root.txt"):
        name, leaf, root = ln.split()
        want[(name, int(leaf))] = bytes.fromhex(root)
    lay = wl.layout_7b()
    tensors = [wl.checkpoint_tensor(lay, i, base_seed=wl.SEED_C3, device="cuda") for i in range(len(lay))]
    ptrs, lens = [t.data_ptr() for t in tensors], [2 * t.numel() for t in tensors]
    total = sum(lens)
    top = torch.zeros(64, dtype=torch.uint8, device="cuda")
    for (name, leaf), root in want.items():
        hid = {"sha256": sentry.HASH_SHA256, "blake2b": sentry.HASH_BLAKE2B}[name]
        top.zero_()
        sentry.sentry_merkle_coalesced_h(hid, ptrs, lens, leaf, 0, 0, top.data_ptr())
        torch.cuda.synchronize()
        assert bytes(top.cpu().numpy()[:len(root)]) == root, (name, leaf)
    padded = -(-total // (1 << 20)) * (1 << 20)
    buf = torch.empty(padded, dtype=torch.uint8, device="cuda")
    top.zero_()
    sentry.sentry_merkle_coalesced(ptrs, lens, 1 << 20, buf.data_ptr(), padded, top.data_ptr())
    torch.cuda.synchronize()
    assert bytes(top.cpu().numpy()[:32]) == want[("sha256", 1 << 20)]
    # the buffer now holds the stream: its plain root at another block size is the coalesced root at that size
    if padded == total:
        sentry.sentry_merkle_root(buf.data_ptr(), total, 8192, top.data_ptr())
        torch.cuda.synchronize()
        assert bytes(top.cpu().numpy()[:32]) == want[("sha256", 8192)]
    del tensors, buf
    free_gpu()

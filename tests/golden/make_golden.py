#!/usr/bin/env python3
"""Writes the expected digests of the five target configurations under tests/golden/.

Inputs come from the numpy generators of ``paper_2510_00554_amd.workloads`` (they hold no
hashing arithmetic), every digest from the CPU oracle under ``oracle/``; nothing here
touches the GPU library.  Leaves and records are independent, so the work is fanned out
over processes, each running the single-threaded oracle on its slice; the reductions are
done by the oracle in the parent.  Run from the repository root:

    python tests/golden/make_golden.py [c1 c2 c3 c3model c3coalesced c4 c4narrow c5 c5pertensor] [--procs N]
"""
import argparse
import multiprocessing as mp
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402
from paper_2510_00554_amd import workloads as wl  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def write(name, header, lines):
    with open(os.path.join(HERE, name), "w") as f:
        for h in header:
            f.write("# " + h + "\n")
        for ln in lines:
            f.write(ln + "\n")
    print("wrote", name, flush=True)


def lanes_hex(lanes):
    return " ".join("%04x" % int(v) for v in lanes)


def c1():
    buf = wl.uniform_bytes(wl.SEED_C1, 0, 16 << 20)
    write("config1_root.txt",
          ["Merkle root (oracle) of config 1: 16 MiB uniform bytes, workloads.SEED_C1, 4 KiB leaves"],
          [oracle.merkle_root(buf, 4096).hex()])


def c2():
    data, off = wl.image_records(50_000)
    full = oracle.lthash(data, off)
    a = oracle.lthash(data, off[:25_001])
    b = oracle.lthash(data, off[25_000:])
    assert (oracle.lthash_combine(a, b) == full).all()
    write("config2_lanes.txt",
          ["Lattice hash (oracle) of config 2: 50,000 samples of 3072 uniform bytes, workloads.SEED_C2",
           "line 1: all samples; line 2: samples [0, 25000); line 3: samples [25000, 50000); 1024 hex uint16 each"],
          [lanes_hex(full), lanes_hex(a), lanes_hex(b)])


# ---- config 5 / config 3: leaf digests of stream ranges --------------------------------

def _c5_task(args):
    start, nbytes, leaf = args
    lay = wl.layout_70b()
    data = wl.checkpoint_stream_np(lay, start, nbytes, base_seed=wl.SEED_C5)
    return start, oracle.merkle_leaves(data, leaf).tobytes()


def c5(pool):
    lay = wl.layout_70b()
    total = wl.checkpoint_offsets(lay)[-1]
    leaf, span = 64 << 10, 64 << 20
    tasks = [(s, min(span, total - s), leaf) for s in range(0, total, span)]
    n_leaves = -(-total // leaf)
    digests = np.empty((n_leaves, 32), np.uint8)
    t0 = time.time()
    for k, (start, blob) in enumerate(pool.imap_unordered(_c5_task, tasks, chunksize=1)):
        d = np.frombuffer(blob, np.uint8).reshape(-1, 32)
        digests[start // leaf:start // leaf + d.shape[0]] = d
        if k % 100 == 0:
            print("c5 %d/%d tasks %.0fs" % (k, len(tasks), time.time() - t0), flush=True)
    root = oracle.merkle_reduce(digests)
    sample = [0, 1, 4095, 1_000_000, n_leaves - 2, n_leaves - 1]
    write("config5_root.txt",
          ["Merkle root (oracle) of config 5: 70B checkpoint (workloads.layout_70b, SEED_C5) as one byte stream,",
           "%d bytes, 64 KiB leaves, %d leaves.  line 1: root; then 'leaf <index> <digest>' samples" % (total, n_leaves)],
          [root.hex()] + ["leaf %d %s" % (i, bytes(digests[i]).hex()) for i in sample])


def _c5pt_task(args):
    idx, e0, e1, leaf = args
    data = wl.normal_bf16_bits(wl.tensor_seed(wl.SEED_C5, idx), e0, e1 - e0).view(np.uint8)
    return idx, e0, oracle.merkle_leaves(data, leaf).tobytes()


def c5pertensor(pool):
    """Config 5 per tensor (Algorithm 2): the 723 tensor roots at 64 KiB leaves and the root over them."""
    lay = wl.layout_70b()
    leaf = 64 << 10
    per = 1024 * (leaf // 2)    # elements per task: 1024 leaves = 64 MiB
    tasks = []
    for i, (_, numel) in enumerate(lay):
        for e0 in range(0, numel, per):
            tasks.append((i, e0, min(numel, e0 + per), leaf))
    leaves = [np.empty((max(1, -(-2 * numel // leaf)), 32), np.uint8) for _, numel in lay]
    t0 = time.time()
    for k, (idx, e0, blob) in enumerate(pool.imap_unordered(_c5pt_task, tasks, chunksize=1)):
        d = np.frombuffer(blob, np.uint8).reshape(-1, 32)
        l0 = (2 * e0) // leaf
        leaves[idx][l0:l0 + d.shape[0]] = d
        if k % 200 == 0:
            print("c5pertensor %d/%d tasks %.0fs" % (k, len(tasks), time.time() - t0), flush=True)
    roots = [oracle.merkle_reduce(lv) for lv in leaves]
    top = oracle.merkle_reduce(np.frombuffer(b"".join(roots), np.uint8).reshape(-1, 32))
    write("config5_per_tensor_roots.txt",
          ["Per-tensor Merkle roots and the root over them (oracle) of config 5's checkpoint (workloads.layout_70b,",
           "SEED_C5), 64 KiB leaves.  line 1: root over the 723 tensor roots; then one tensor root per line"],
          [top.hex()] + ["%s %s" % (lay[i][0], roots[i].hex()) for i in range(len(lay))])


def _c3_task(args):
    idx, e0, e1, leaf = args
    lay = wl.layout_7b()
    data = wl.normal_bf16_bits(wl.tensor_seed(wl.SEED_C3, idx), e0, e1 - e0).view(np.uint8)
    return idx, e0, oracle.merkle_leaves(data, leaf).tobytes()


def c3(pool):
    lay = wl.layout_7b()
    leaf = 1 << 20
    per = 32 * (leaf // 2)   # elements per task: 32 leaves
    tasks = []
    for i, (_, numel) in enumerate(lay):
        for e0 in range(0, numel, per):
            tasks.append((i, e0, min(numel, e0 + per), leaf))
    leaves = [np.empty((max(1, -(-2 * numel // leaf)), 32), np.uint8) for _, numel in lay]
    for idx, e0, blob in pool.imap_unordered(_c3_task, tasks, chunksize=1):
        d = np.frombuffer(blob, np.uint8).reshape(-1, 32)
        l0 = (2 * e0) // leaf
        leaves[idx][l0:l0 + d.shape[0]] = d
    roots = [oracle.merkle_reduce(lv) for lv in leaves]
    top = oracle.merkle_reduce(np.frombuffer(b"".join(roots), np.uint8).reshape(-1, 32))
    flat = oracle.merkle_reduce(np.concatenate(leaves, axis=0))
    write("config3_inplace_root.txt",
          ["Root (oracle) of the ONE flat tree over the 1 MiB blocks of all 291 tensors of config 3 in order",
           "(Algorithm 3, in-place hashing; the 8 KiB norm tensors are short leaves)"],
          [flat.hex()])
    write("config3_roots.txt",
          ["Per-tensor Merkle roots and model root (oracle) of config 3: 7B checkpoint (workloads.layout_7b,",
           "SEED_C3), 1 MiB leaves.  line 1: model root over the 291 tensor roots; then one tensor root per line"],
          [top.hex()] + ["%s %s" % (lay[i][0], roots[i].hex()) for i in range(len(lay))])


def _c3_model_task(args):
    idx, e0, e1, first_index, block = args
    data = wl.normal_bf16_bits(wl.tensor_seed(wl.SEED_C3, idx), e0, e1 - e0).view(np.uint8)
    _, lanes = oracle.lthash_model([data], block, first_index=first_index)
    return idx, lanes.tobytes()


def c3model(pool):
    """Model lattice hash (Algorithm 4) of the 7B checkpoint at the paper's default 8 KiB blocks."""
    lay = wl.layout_7b()
    block = 8192
    per = 4096 * (block // 2)                      # elements per task: 4096 blocks
    tasks, index = [], 0
    for i, (_, numel) in enumerate(lay):
        for e0 in range(0, numel, per):
            tasks.append((i, e0, min(numel, e0 + per), index + (2 * e0) // block, block))
        index += -(-2 * numel // block)
    layers = np.zeros((len(lay), 32), np.uint16)
    for idx, blob in pool.imap_unordered(_c3_model_task, tasks, chunksize=1):
        layers[idx] = oracle.lanes_add(layers[idx], np.frombuffer(blob, np.uint16))
    total = np.zeros(32, np.uint16)
    for row in layers:
        total = oracle.lanes_add(total, row)
    write("config3_model_lthash.txt",
          ["Model lattice hash (oracle, Algorithm 4: BLAKE2b-512 of LE64(block index) || block, 32 partitions) of the",
           "config 3 checkpoint, 8 KiB blocks, %d blocks.  line 1: model digest; then one tensor digest per line" % index],
          [lanes_hex(total)] + ["%s %s" % (lay[i][0], lanes_hex(layers[i])) for i in range(len(lay))])


def _c3co_task(args):
    start, nbytes, leaf, h = args
    lay = wl.layout_7b()
    data = wl.checkpoint_stream_np(lay, start, nbytes, base_seed=wl.SEED_C3)
    if nbytes % leaf:                      # Algorithm 1: zero bytes up to a whole block
        data = np.concatenate([data, np.zeros(leaf - nbytes % leaf, np.uint8)])
    if h == oracle.HASH_SHA256:
        return start, oracle.merkle_leaves(data, leaf).tobytes()
    return start, b"".join(oracle.merkle_root_h(h, data[i:i + leaf], leaf) for i in range(0, data.size, leaf))


def c3coalesced(pool):
    """Algorithm 1 over the 7B checkpoint: the tensors as one byte stream, zero-padded to whole blocks;
    SHA-256 at 1 MiB blocks, and SHA-256 and BLAKE2b-512 at the paper's default 8 KiB."""
    lay = wl.layout_7b()
    total = wl.checkpoint_offsets(lay)[-1]
    lines = []
    for name, h, dl, leaf in (("sha256", oracle.HASH_SHA256, 32, 1 << 20), ("sha256", oracle.HASH_SHA256, 32, 8192),
                              ("blake2b", oracle.HASH_BLAKE2B, 64, 8192)):
        span = 64 << 20
        tasks = [(s, min(span, total - s), leaf, h) for s in range(0, total, span)]
        n_leaves = -(-total // leaf)
        digests = np.empty((n_leaves, dl), np.uint8)
        for start, blob in pool.imap_unordered(_c3co_task, tasks, chunksize=1):
            d = np.frombuffer(blob, np.uint8).reshape(-1, dl)
            digests[start // leaf:start // leaf + d.shape[0]] = d
        # the tree over ready-made nodes: the hash of the 2-node concatenation, level by level,
        # is what merkle_root_h does to a buffer of digests cut into leaves of two digests' size
        root = oracle.merkle_reduce(digests) if h == oracle.HASH_SHA256 else _reduce_h(h, digests)
        lines.append("%s %d %s" % (name, leaf, root.hex()))
        print("c3coalesced", name, leaf, flush=True)
    write("config3_coalesced_root.txt",
          ["Root (oracle) of the tree over the 291 tensors of config 3 laid one behind the other in one buffer,",
           "zero bytes up to a whole block (Algorithm 1, coalesced hashing); %d bytes.  '<hash> <block bytes> <root>'" % total],
          lines)


def _reduce_h(h, digests):
    level = [bytes(d) for d in digests]
    while len(level) > 1:
        nxt = [oracle.merkle_root_h(h, level[i] + level[i + 1], 2 * len(level[i])) for i in range(0, len(level) - 1, 2)]
        if len(level) % 2:
            nxt.append(level[-1])
        level = nxt
    return level[0]


# ---- config 4: lattice hash of record ranges ---------------------------------------------

_C4_OFF = None


def _c4_offsets():
    global _C4_OFF
    if _C4_OFF is None:
        _C4_OFF = wl.offsets_from_lengths(wl.lognormal_record_lengths(wl.C4_RECORDS))
    return _C4_OFF


def _c4_task(args):
    a, b = args
    off = _c4_offsets()
    data = wl.uniform_bytes(wl.SEED_C4_BYTES, int(off[a]), int(off[b] - off[a]))
    return a, oracle.lthash(data, off[a:b + 1] - off[a]).tobytes()


def c4(pool):
    off = _c4_offsets()
    batches = wl.cut_batches(off, wl.C4_BATCH_BYTES)
    tasks, owner = [], {}
    for bi, (a, b) in enumerate(batches):
        for (x, y) in [(a + p, a + q) for p, q in wl.cut_batches(off[a:b + 1] - off[a], 64_000_000)]:
            tasks.append((x, y))
            owner[x] = bi
    per_batch = [np.zeros(1024, np.uint16) for _ in batches]
    t0 = time.time()
    for k, (a, blob) in enumerate(pool.imap_unordered(_c4_task, tasks, chunksize=1)):
        bi = owner[a]
        per_batch[bi] = oracle.lthash_combine(per_batch[bi], np.frombuffer(blob, np.uint16))
        if k % 200 == 0:
            print("c4 %d/%d tasks %.0fs" % (k, len(tasks), time.time() - t0), flush=True)
    total = np.zeros(1024, np.uint16)
    for lanes in per_batch:
        total = oracle.lthash_combine(total, lanes)
    write("config4_lanes.txt",
          ["Lattice hash (oracle) of config 4: %d records, log-normal lengths (workloads.lognormal_record_lengths," % wl.C4_RECORDS,
           "SEED_C4_LEN), bytes from the uniform stream SEED_C4_BYTES cut at record boundaries; %d bytes in %d batches"
           % (int(off[-1]), len(batches)),
           "of at most 8e9 bytes.  line 1: all records; then 'batch <k> <first> <last_exclusive> <lanes>'"],
          [lanes_hex(total)] + ["batch %d %d %d %s" % (k, a, b, lanes_hex(per_batch[k]))
                                for k, (a, b) in enumerate(batches)])


def _c4n_task(args):
    a, b = args
    off = _c4_offsets()
    data = wl.uniform_bytes(wl.SEED_C4_BYTES, int(off[a]), int(off[b] - off[a]))
    return a, oracle.lthash32(data, off[a:b + 1] - off[a]).tobytes()


def c4narrow(pool):
    """Config 4 at the 32-partition width (section 4.2.2): the same records and batches."""
    off = _c4_offsets()
    batches = wl.cut_batches(off, wl.C4_BATCH_BYTES)
    tasks, owner = [], {}
    for bi, (a, b) in enumerate(batches):
        for (x, y) in [(a + p, a + q) for p, q in wl.cut_batches(off[a:b + 1] - off[a], 64_000_000)]:
            tasks.append((x, y))
            owner[x] = bi
    per_batch = [np.zeros(32, np.uint16) for _ in batches]
    t0 = time.time()
    for k, (a, blob) in enumerate(pool.imap_unordered(_c4n_task, tasks, chunksize=1)):
        per_batch[owner[a]] = oracle.lanes_add(per_batch[owner[a]], np.frombuffer(blob, np.uint16))
        if k % 200 == 0:
            print("c4narrow %d/%d tasks %.0fs" % (k, len(tasks), time.time() - t0), flush=True)
    total = np.zeros(32, np.uint16)
    for lanes in per_batch:
        total = oracle.lanes_add(total, lanes)
    write("config4_lanes32.txt",
          ["32-partition lattice hash (oracle: plain BLAKE2b-512 per record) of config 4's records, %d bytes in %d batches."
           % (int(off[-1]), len(batches)),
           "line 1: all records; then 'batch <k> <first> <last_exclusive> <32 hex uint16>'"],
          [lanes_hex(total)] + ["batch %d %d %d %s" % (k, a, b, lanes_hex(per_batch[k]))
                                for k, (a, b) in enumerate(batches)])


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("configs", nargs="*", default=["c1", "c2", "c3", "c3model", "c3coalesced", "c4", "c4narrow", "c5", "c5pertensor"])
    ap.add_argument("--procs", type=int, default=os.cpu_count())
    a = ap.parse_args()
    oracle.build()
    with mp.Pool(a.procs) as pool:
        for c in a.configs:
            t = time.time()
            {"c1": c1, "c2": c2}.get(c, lambda: {"c3": c3, "c3model": c3model, "c3coalesced": c3coalesced, "c4": c4, "c4narrow": c4narrow, "c5": c5, "c5pertensor": c5pertensor}[c](pool))()
            print("%s done in %.0fs" % (c, time.time() - t), flush=True)

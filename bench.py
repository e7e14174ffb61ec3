#!/usr/bin/env python3
"""Benchmark of the artifact-hashing hot path on one MI355X.

One step = one pass of the whole path over inputs already resident in HBM.  The three parts
belong to independent artifacts; the second and third are bound by single serial chains and
leave most of the chip idle, so they run on a second stream (one after the other) beside the
first, which can use every issue slot they leave (--schedule serial runs all three back to back
on one stream; --schedule pair runs the first alone, then the other two side by side):
  * Merkle root of the 70B-parameter bf16 checkpoint laid out as one byte stream
    (137.95 GB, 64 KiB leaves)                         -> sentry_merkle_root, sentry_verify
  * per-tensor roots + model root of the 7B checkpoint (291 tensors, 13.48 GB,
    1 MiB leaves)                                      -> sentry_merkle_segments
  * lattice hash of one 8 GB batch of variable-length records (log-normal lengths),
    folded into the running sum                        -> sentry_lthash, sentry_lthash_combine
`value` = bytes hashed per step / step time (GB = 1e9 bytes).

Beside it, in the same JSON line: `roofline` (the SHA-256 leaf kernel on the 70B stream against
the integer-ALU peak: as it runs inside the step, sharing the chip with the other two parts, with
the same kernel timed alone and the whole step's operations over the step time beside it), `per_config` (the five target configurations and the widened entry
points, each with GB/s and its fractions of the ALU and HBM rooflines), `streaming` (hashing
while loading from 16 GB of pinned host memory in the shape of configs 5 and 4, against the
plain copy of the same bytes; PCIe-bound, never part of `value`) and `cpu_baseline` (the
single-threaded oracle on a bounded sample of the same inputs).

Prints one JSON line.  --quick shrinks every input (for smoke runs; the workload name says so).
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

ALU_PEAK_OPS = 256 * 4 * 16 * 2.4e9          # CUs x SIMDs x lanes x clock: 32-bit VALU lane-ops/s (nominal)
HBM_PEAK = 8.0e12


class Mix(dict):
    """VALU instructions by opcode: the work of a hash, counted as the instructions its hot loop
    needs on gfx950 (one instruction = one operation of each of a wave's 64 lanes)."""

    def __add__(self, other):
        out = Mix(self)
        for k, v in other.items():
            out[k] = out.get(k, 0) + v
        return out

    def __mul__(self, n):
        return Mix({k: v * n for k, v in self.items()})

    __rmul__ = __mul__

    def total(self):
        return sum(self.values())


# SHA-256 on gfx950 (rotate = v_alignbit_b32, xor3/Ch/Maj = v_bitop3_b32, three-input add = v_add3_u32).
# One 64-byte block: 64 rounds x (6 rotates, 4 three-input booleans, 3 add3, 1 add) + 48 schedule steps x
# (4 rotates, 2 xor3, 2 shifts, add3 + add) + 16 byte swaps + 8 feed-forward adds = 1400; the compiled
# loop has exactly these (1384 in the loop body + the 16 v_perm_b32 of the loads).
SHA_BLOCK_MIX = Mix({"v_alignbit_b32": 64 * 6 + 48 * 4, "v_bitop3_b32": 64 * 4 + 48 * 2, "v_add3_u32": 64 * 3 + 48,
                     "v_add_u32": 64 + 48 + 8, "v_lshrrev_b32": 48 * 2, "v_perm_b32": 16})
# A block whose message schedule is a constant (the padding block of a leaf that is a whole number of
# blocks, the second block of an inner node): rounds with K + W folded into one literal, and the adds.
SHA_CONST_BLOCK_MIX = Mix({"v_alignbit_b32": 64 * 6, "v_bitop3_b32": 64 * 4, "v_add3_u32": 64 * 2, "v_add_u32": 64 * 2 + 8})
# BLAKE2b: 96 G functions x (6 64-bit adds as v_lshl_add_u64, 4 64-bit xors = 8 v_xor_b32, 3 rotations by
# 24/16/63 = 6 v_alignbit_b32; the rotation by 32 is a renaming) + 16 64-bit xors of the feed-forward.
# A 64-bit add is ONE instruction here, not two.  The one-block expansion calls have eight zero message
# words (96 of the 192 message adds vanish) and 16 packed 16-bit adds into the lane sums.
B2_BLOCK_MIX = Mix({"v_lshl_add_u64": 96 * 6, "v_xor_b32": 96 * 8 + 32, "v_alignbit_b32": 96 * 6})
B2_EXPAND_MIX = Mix({"v_lshl_add_u64": 96 * 6 - 96, "v_xor_b32": 96 * 8 + 32, "v_alignbit_b32": 96 * 6, "v_pk_add_u16": 16})
# Keccak-f[1600] on 32-bit halves: per round theta 20 xor3 + 10 rotate halves + 60 xor, rho 48 rotate halves,
# chi 50 three-input booleans, iota 2 xor; 24 rounds, plus 34 xors to absorb a 136-byte block.
KECCAK_BLOCK_MIX = Mix({"v_bitop3_b32": 24 * 70, "v_xor_b32": 24 * 62 + 34, "v_alignbit_b32": 24 * 58})
SHA_BLOCK_OPS, SHA_CONST_BLOCK_OPS = SHA_BLOCK_MIX.total(), SHA_CONST_BLOCK_MIX.total()            # 1400, 904
B2_BLOCK_OPS, B2_EXPAND_OPS, KECCAK_BLOCK_OPS = B2_BLOCK_MIX.total(), B2_EXPAND_MIX.total(), KECCAK_BLOCK_MIX.total()
SHA_NODE_MIX = SHA_BLOCK_MIX + SHA_CONST_BLOCK_MIX

# Measured issue rates of single opcodes on this chip, T lane-ops/s with four waves per SIMD (the table
# `python bench.py --valu-probe` prints; profiles/valu_issue_rates.md holds a run of it).  Two classes: the
# two-operand integer and boolean ops and v_bitop3_b32 issue at about 57 T, the three-operand adds, funnel
# shifts, byte permutes, 64-bit and packed adds at about 36 T; the nominal 39.32 T is neither.  The
# ceiling of a kernel is that of its mix: total instructions / sum(instructions of opcode / its rate).
ISSUE_RATE_TOPS = {"v_xor_b32": 57.0, "v_add_u32": 57.0, "v_lshrrev_b32": 57.0, "v_bitop3_b32": 57.0,
                   "v_alignbit_b32": 36.0, "v_add3_u32": 36.0, "v_perm_b32": 36.0, "v_lshl_add_u64": 36.0,
                   "v_pk_add_u16": 36.0}


def issue_bound(mix):
    """Lane-ops/s the chip can issue for this instruction mix (every opcode at its measured rate)."""
    return mix.total() / sum(n / (ISSUE_RATE_TOPS[op] * 1e12) for op, n in mix.items() if n)


def merkle_mix(n_leaves, leaf_bytes, n_nodes):
    per_leaf = (leaf_bytes // 64) * SHA_BLOCK_MIX + SHA_CONST_BLOCK_MIX
    return n_leaves * per_leaf + n_nodes * SHA_NODE_MIX


def sha_tree_mix(lens, leaf_bytes, flat=False):
    """SHA-256 trees over buffers of the given byte lengths: per-buffer trees plus the tree over
    their roots, or (flat) one tree over all their leaves."""
    mix, leaves_total = Mix(), 0
    for ln in lens:
        n = -(-ln // leaf_bytes) if (ln or flat) else 1
        if ln == 0 and not flat:
            mix = mix + SHA_BLOCK_MIX
        for size, count in ((leaf_bytes, ln // leaf_bytes), (ln % leaf_bytes, 1 if ln % leaf_bytes else 0)):
            # full blocks, then the padding block(s): constant when the leaf is a whole number of blocks
            if count:
                pad = SHA_CONST_BLOCK_MIX if size % 64 == 0 else (2 if size % 64 > 55 else 1) * SHA_BLOCK_MIX
                mix = mix + count * ((size // 64) * SHA_BLOCK_MIX + pad)
        leaves_total += n
        if not flat:
            mix = mix + (n - 1) * SHA_NODE_MIX
    top = leaves_total if flat else len(lens)
    return mix + (max(top, 1) - 1) * SHA_NODE_MIX


def sha_tree_ops(lens, leaf_bytes, flat=False):
    return sha_tree_mix(lens, leaf_bytes, flat).total()


def other_tree_mix(hash_name, lens, leaf_bytes, flat=False):
    unit = B2_BLOCK_MIX if hash_name == "blake2b" else KECCAK_BLOCK_MIX
    blocks, leaves_total = 0, 0
    for ln in lens:
        sizes = [(leaf_bytes, ln // leaf_bytes)] + ([(ln % leaf_bytes, 1)] if ln % leaf_bytes or (ln == 0 and not flat) else [])
        n = sum(c for _, c in sizes)
        for size, count in sizes:
            blocks += count * (max(1, -(-size // 128)) if hash_name == "blake2b" else size // 136 + 1)
        leaves_total += n
        if not flat:
            blocks += max(n - 1, 0)
    top = leaves_total if flat else len(lens)
    return (blocks + max(top, 1) - 1) * unit


def other_tree_ops(hash_name, lens, leaf_bytes, flat=False):
    return other_tree_mix(hash_name, lens, leaf_bytes, flat).total()


def lthash_mix(record_lengths):
    import numpy as np
    blocks = np.maximum(1, -(-np.asarray(record_lengths, dtype=np.int64) // 128))
    return int(blocks.sum()) * B2_BLOCK_MIX + (len(record_lengths) * 32) * B2_EXPAND_MIX


def lthash_ops(record_lengths):
    return lthash_mix(record_lengths).total()


def lthash32_mix(record_lengths):
    """The 32-partition hash: the root compressions alone, and one packed add per digest word."""
    import numpy as np
    blocks = np.maximum(1, -(-np.asarray(record_lengths, dtype=np.int64) // 128))
    return int(blocks.sum()) * B2_BLOCK_MIX + Mix({"v_pk_add_u16": 16 * len(record_lengths)})


def model_lthash_mix(lens, block_bytes):
    blocks = 0
    for ln in lens:
        for size, count in ((block_bytes, ln // block_bytes), (ln % block_bytes, 1 if ln % block_bytes else 0)):
            blocks += count * (-(-(size + 8) // 128))
    return blocks * B2_BLOCK_MIX


def model_lthash_ops(lens, block_bytes):
    return model_lthash_mix(lens, block_bytes).total()


# A launch with fewer leaves (records) than lanes is bound by the serial chain of its longest leaf:
# a wave that has a SIMD to itself issues one VALU instruction per 5.0 to 5.4 cycles on this chip,
# whatever the instruction (measured: 5.0 with the rest of its CU idle, 5.3 - 5.4 with the other SIMDs
# of the CU busy), so chain_floor = instructions on the longest chain x 5.0 cycles /
# 2.4 GHz.  Instructions per block on the critical wave: 930 for the SHA-256 rounds-only
# consumer wave, 2304 for one tree level (two compressions by one lane; 1850 where a second wave
# expands the node's message schedule, as the one-launch tree of small inputs does), 700 for one
# BLAKE2b compression spread over four lanes.
LONE_WAVE_CYCLES_PER_INSTR, CLOCK_HZ = 5.0, 2.4e9
SHA_CONSUMER_INSTRS, SHA_NODE_INSTRS, SHA_NODE_SPLIT_INSTRS, B2_FOUR_LANE_INSTRS = 930, 2304, 1850, 700


def chain_bound(entry, instrs):
    floor_ms = instrs * LONE_WAVE_CYCLES_PER_INSTR / CLOCK_HZ * 1e3
    entry["bound"] = "chain"
    entry["chain_floor_ms"] = floor_ms
    entry["chain_frac"] = floor_ms / entry["ms"]
    return entry


def tree_levels(n):
    lv = 0
    while n > 1:
        n = (n + 1) // 2
        lv += 1
    return lv


class Timed(float):
    """A time in ms that remembers the spread of the calls it is the median of."""
    spread = None


def rated(entry, mix, hbm_bytes=None):
    """Add the roofline fractions to a per-config entry: alu_frac against the nominal integer-ALU peak
    (instructions of the mix x 64 lanes / time / 39.32 T), issue_frac against the rate at which the chip
    can issue this mix (issue_bound), hbm_frac against 8 TB/s (bytes hashed unless hbm_bytes is given)."""
    if isinstance(entry["ms"], Timed) and entry["ms"].spread:
        entry.update(entry["ms"].spread)
        entry["ms"] = float(entry["ms"])
    sec = entry["ms"] * 1e-3
    ops = mix.total()
    bound = issue_bound(mix)
    entry["alu_frac"] = ops / sec / ALU_PEAK_OPS
    entry["issue_bound_TOP/s"] = bound / 1e12
    entry["issue_frac"] = ops / sec / bound
    entry["hbm_frac"] = (hbm_bytes if hbm_bytes is not None else entry["bytes"]) / sec / HBM_PEAK
    return entry


def load_probe():
    import ctypes
    path = os.path.join(ROOT, "paper_2510_00554_amd", "libsentry_probe.so")
    if not os.path.exists(path):
        from paper_2510_00554_amd import build as _build
        _build.build()
    lib = ctypes.CDLL(path)
    lib.sentry_probe_op_name.restype = ctypes.c_char_p
    lib.sentry_probe_valu.argtypes = [ctypes.c_int, ctypes.c_int] + [ctypes.POINTER(ctypes.c_double)] * 3
    return lib


def probe_issue_rates(only=None, waves=(4,)):
    """{opcode name: {waves per SIMD: (T lane-ops/s, shader MHz, cycles between a wave's instructions)}},
    measured now on the current device by the probe kernels (four independent chains of one opcode)."""
    import ctypes
    lib = load_probe()
    out = {}
    for op in range(lib.sentry_probe_op_count()):
        name = lib.sentry_probe_op_name(op).decode()
        if only is not None and name not in only:
            continue
        for w in waves:
            t, f, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
            rc = lib.sentry_probe_valu(op, w, ctypes.byref(t), ctypes.byref(f), ctypes.byref(c))
            if rc:
                sys.exit("bench.py: VALU probe failed on %s (HIP error %d)" % (name, rc))
            out.setdefault(name, {})[w] = (t.value, f.value, c.value)
    return out


def run_only_config(args, sentry, wl, torch, np, dev, stream):
    """One configuration alone, args.steps timed calls after args.warmup: one short JSON line."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.only_config == "a1":
        # coalesced hashing with the copy (Algorithm 1) of the 7B checkpoint, 8 KiB blocks
        lay7 = wl.layout_7b()
        t7 = [wl.checkpoint_tensor(lay7, i, base_seed=wl.SEED_C3, device=dev) for i in range(len(lay7))]
        ptrs, lens = [t.data_ptr() for t in t7], [t.numel() * 2 for t in t7]
        nbytes = sum(lens)
        padded = -(-nbytes // 8192) * 8192
        cbuf = torch.empty(padded, dtype=torch.uint8, device=dev)
        out = torch.zeros(32, dtype=torch.uint8, device=dev)
        mix = sha_tree_mix([padded], 8192, flat=True)
        if args.copy_probe:
            src = torch.ones(1 << 30, dtype=torch.int32, device=dev)
            dst = torch.empty_like(src)
            torch.add(src, 1, out=dst)
            torch.cuda.synchronize()
            del src, dst

        def call():
            sentry.sentry_merkle_coalesced(ptrs, lens, 8192, cbuf.data_ptr(), padded, out.data_ptr(), stream)
    elif args.only_config == "c1":
        buf = wl.uniform_bytes(wl.SEED_C1, 0, 16 << 20, device=dev)
        out = torch.zeros(32, dtype=torch.uint8, device=dev)
        nbytes, mix = buf.numel(), sha_tree_mix([buf.numel()], 4096, flat=True)

        def call():
            sentry.sentry_merkle_root(buf.data_ptr(), nbytes, 4096, out.data_ptr(), stream)
    else:
        img, ioff = wl.image_records(50_000, device=dev)
        d_ioff = torch.from_numpy(ioff.view(np.int64).copy()).to(dev)
        lanes, half_a, half_b = (torch.zeros(1024, dtype=torch.int16, device=dev) for _ in range(3))
        nbytes, mix = img.numel(), lthash_mix([3072] * 50_000)

        def call():
            sentry.sentry_lthash(img.data_ptr(), d_ioff.data_ptr(), 50_000, lanes.data_ptr(), stream)
    for _ in range(max(args.warmup, 1)):
        call()
    torch.cuda.synchronize()
    ts = []
    for _ in range(args.steps):
        a.record()
        call()
        b.record()
        b.synchronize()
        ts.append(a.elapsed_time(b))
    entry = rated({"ms": statistics.median(ts), "ms_min": min(ts), "ms_max": max(ts), "calls": len(ts), "bytes": nbytes,
                   "GB/s": nbytes / statistics.median(ts) / 1e6}, mix)
    if args.only_config == "c2":
        # the two disjoint halves, combined, equal the whole (checked here as well as in tests/)
        sentry.sentry_lthash(img.data_ptr(), d_ioff.data_ptr(), 25_000, half_a.data_ptr(), stream)
        sentry.sentry_lthash(img.data_ptr(), d_ioff.data_ptr() + 8 * 25_000, 25_000, half_b.data_ptr(), stream)
        sentry.sentry_lthash_combine(half_a.data_ptr(), half_b.data_ptr(), stream)
        torch.cuda.synchronize()
        if not torch.equal(half_a, lanes):
            sys.exit("bench.py: combine of the halves differs from the whole")
        entry["samples/s"] = 50_000 / (entry["ms"] * 1e-3)
    print(json.dumps({"config": args.only_config, **entry}))


def print_valu_probe():
    """The table behind ISSUE_RATE_TOPS (profiles/valu_issue_rates.md is one run of this)."""
    rates = probe_issue_rates(waves=(1, 2, 4, 8))
    print("| opcode | " + " | ".join("%d waves/SIMD: T lane-ops/s (MHz, clk/instr/wave)" % w for w in (1, 2, 4, 8)) + " |")
    print("|---|---|---|---|---|")
    for name, by_w in rates.items():
        print("| %s | " % name + " | ".join("%.1f (%.0f, %.2f)" % by_w[w] for w in (1, 2, 4, 8)) + " |")
    for label, mix in (("sha-256 block", SHA_BLOCK_MIX), ("blake2b compression", B2_BLOCK_MIX), ("keccak block", KECCAK_BLOCK_MIX)):
        live = {k: v[4][0] for k, v in rates.items()}
        measured = mix.total() / sum(n / live[op] for op, n in mix.items())
        print("mix ceiling, %s: %.1f T lane-ops/s from this run's single-opcode rates at 4 waves/SIMD, %.1f from the table in bench.py"
              % (label, measured, issue_bound(mix) / 1e12))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--quick", action="store_true", help="1/64-size inputs (not the reported workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--schedule", choices=("overlap", "pair", "serial"), default="overlap",
                    help="overlap: the 70B root on one stream, the other two parts one after the other on a second; "
                         "pair: the 70B root alone, then the other two side by side; serial: one stream")
    ap.add_argument("--no-extras", action="store_true", help="skip per-config and streaming side measurements")
    ap.add_argument("--no-streaming", action="store_true", help="skip the host-to-device streaming legs (for counter runs)")
    ap.add_argument("--no-graph", action="store_true", help="skip the entry that captures and replays a HIP graph (for profiler runs)")
    ap.add_argument("--merkle-prefix-gib", type=int, default=0,
                    help="hash only the first N GiB of the 70B stream (for counter runs; the workload name says so)")
    ap.add_argument("--only-config", choices=("c1", "c2", "a1"), default=None,
                    help="run only config 1 (16 MiB Merkle, 4 KiB leaves), config 2 (50,000 images, lattice hash, and "
                         "the two halves combined) or a1 (coalesced hashing of the 7B checkpoint with the copy, 8 KiB "
                         "blocks) --steps times and print its own short line (for kernel traces)")
    ap.add_argument("--valu-probe", action="store_true",
                    help="print the measured issue rate of every VALU opcode the hash kernels use, and exit")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 4 GiB device copy kernel (calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (got --gpus %d); no multi-GPU figure exists" % args.gpus)

    import numpy as np
    import torch

    import paper_2510_00554_amd as sentry
    from paper_2510_00554_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    sentry.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.valu_probe:
        print_valu_probe()
        return
    if args.only_config:
        run_only_config(args, sentry, wl, torch, np, dev, torch.cuda.current_stream().cuda_stream)
        return
    # the issue rates of the opcodes in the hash kernels' mixes, measured now (a few ms each): printed
    # beside the table the fractions are computed against, as a check on that table
    live_rates = {k: round(v[4][0], 2) for k, v in probe_issue_rates(only=set(ISSUE_RATE_TOPS)).items()}
    stream = torch.cuda.current_stream().cuda_stream
    t_setup = time.time()

    def log(msg):
        print("[bench %6.1fs] %s" % (time.time() - t_setup, msg), file=sys.stderr, flush=True)

    # ---------------- inputs, resident in HBM ----------------
    if args.quick:
        lay70, lay7 = wl.llama_layout(4, 4096, 14336, 32000, kv_dim=512), wl.llama_layout(2, 2048, 5504, 32000)
        batch_bytes, n_records_total = 128_000_000, 20_000
    else:
        lay70, lay7 = wl.layout_70b(), wl.layout_7b()
        batch_bytes, n_records_total = 8_000_000_000, 1_281_167
    if args.merkle_prefix_gib:
        # cut the layout after the tensors that cover the prefix, so that no more is generated
        acc, cut = 0, []
        for name, numel in lay70:
            cut.append((name, numel))
            acc += 2 * numel
            if acc >= args.merkle_prefix_gib << 30:
                break
        lay70 = cut
    # resident inputs, plus (side measurements) a 16 GB copy target, three staging buffers of one batch and two of one chunk
    need = 2 * sum(n for _, n in lay70) + 2 * sum(n for _, n in lay7) + batch_bytes + (2 << 30)
    if not args.no_extras and not args.no_streaming and not args.quick:
        need += (16 << 30) + 3 * batch_bytes + (4 << 30)
    free, _ = torch.cuda.mem_get_info()
    if free < need:
        sys.exit("bench.py: needs %.1f GB of free HBM, %.1f GB available" % (need / 1e9, free / 1e9))

    log("generating the 70B-shaped checkpoint (%d tensors)" % len(lay70))
    ckpt70, _ = wl.checkpoint_flat_torch(lay70, dev, base_seed=wl.SEED_C5)
    log("generating the 7B-shaped checkpoint (%d tensors, one allocation each)" % len(lay7))
    t7 = [wl.checkpoint_tensor(lay7, i, base_seed=wl.SEED_C3, device=dev) for i in range(len(lay7))]
    t7_ptrs = [t.data_ptr() for t in t7]
    t7_lens = [t.numel() * 2 for t in t7]
    log("generating one batch of variable-length records")
    lengths = wl.lognormal_record_lengths(n_records_total)
    offsets = wl.offsets_from_lengths(lengths)
    b0, b1 = wl.cut_batches(offsets, batch_bytes)[0]
    rec_off = offsets[b0:b1 + 1]
    rec_bytes = int(rec_off[-1] - rec_off[0])
    n_rec = b1 - b0
    records = wl.uniform_bytes(wl.SEED_C4_BYTES, int(rec_off[0]), rec_bytes, device=dev)
    d_off = torch.from_numpy(rec_off.view(np.int64).copy()).to(dev)
    torch.cuda.synchronize()

    LEAF70, LEAF7 = 64 << 10, 1 << 20
    root70 = torch.zeros(32, dtype=torch.uint8, device=dev)
    root7 = torch.zeros(32, dtype=torch.uint8, device=dev)
    seg_roots = torch.zeros(32 * len(t7), dtype=torch.uint8, device=dev)
    lanes = torch.zeros(1024, dtype=torch.int16, device=dev)
    running = torch.zeros(1024, dtype=torch.int16, device=dev)
    host_root = torch.zeros(32, dtype=torch.uint8).pin_memory()

    bytes70, bytes7 = ckpt70.numel(), sum(t7_lens)
    if args.merkle_prefix_gib:
        bytes70 = min(bytes70, args.merkle_prefix_gib << 30)
    step_bytes = bytes70 + bytes7 + rec_bytes
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
    # The per-tensor pass over the 7B checkpoint and the lattice hash of the batch are both bound by
    # single serial chains and leave most of the chip idle; the 70B root is bound by instruction issue.
    # They are independent artifacts (two models, a dataset), so the step runs the chain-bound parts
    # on a second stream while the 70B root fills whatever they leave free.
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()

    def part_7b(st):
        sentry.sentry_merkle_segments(t7_ptrs, t7_lens, LEAF7, seg_roots.data_ptr(), root7.data_ptr(), st)

    def part_batch(st):
        sentry.sentry_lthash(records.data_ptr(), d_off.data_ptr(), n_rec, lanes.data_ptr(), st)
        sentry.sentry_lthash_combine(running.data_ptr(), lanes.data_ptr(), st)

    def part_70b(st):
        sentry.sentry_merkle_root(ckpt70.data_ptr(), bytes70, LEAF70, root70.data_ptr(), st)

    def step(expected=None, timed=None):
        ev[0].record()
        if args.schedule == "serial":
            part_70b(stream)
            ev[1].record()
            part_7b(stream)
            ev[2].record()
            part_batch(stream)
            ev[3].record()
            spans = ((0, 1), (1, 2), (2, 3))
        elif args.schedule == "pair":
            part_70b(stream)
            ev[1].record()
            side.wait_event(ev[1])
            part_7b(stream)
            ev[2].record()
            part_batch(side.cuda_stream)
            ev[3].record(side)
            main.wait_event(ev[3])
            spans = ((0, 1), (1, 2), (1, 3))
        else:
            # the two chain-bound parts, one after the other, on the side stream; they are queued first
            # so that their few waves are resident when the 70B root's workgroups fill the rest of the chip
            side.wait_event(ev[0])
            part_7b(side.cuda_stream)
            ev[2].record(side)
            part_batch(side.cuda_stream)
            ev[3].record(side)
            part_70b(stream)
            ev[1].record()
            main.wait_event(ev[3])
            spans = ((0, 1), (0, 2), (2, 3))
        ev[4].record()
        host_root.copy_(root70, non_blocking=True)
        torch.cuda.synchronize()
        got = bytes(host_root.numpy())
        if expected is not None and sentry.sentry_verify(got, expected) != 0:
            sys.exit("bench.py: root changed between steps")
        if timed is not None:
            # per part: from the event it starts after to its own end; then all three parts
            timed.append(tuple(ev[a].elapsed_time(ev[b]) for a, b in spans) + (ev[0].elapsed_time(ev[4]),))
        return got

    def alone(fn, reps=3):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ts = []
        for _ in range(reps):
            torch.cuda.synchronize()
            a.record()
            fn()
            b.record()
            b.synchronize()
            ts.append(a.elapsed_time(b))
        return statistics.median(ts)

    if args.copy_probe:
        # a plain copy of known size: 2^30 int32 elements read and written once by one kernel
        src = torch.ones(1 << 30, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # what the other two parts give when each runs with the chip to itself, to hold the overlapped
    # steps against
    part_7b(stream)
    part_batch(stream)
    torch.cuda.synchronize()
    alone_out = [t.clone() for t in (root7, seg_roots, lanes)]

    log("warm-up")
    expected = step()
    for _ in range(max(args.warmup - 1, 0)):
        step(expected)
    log("timing %d steps" % args.steps)
    parts = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(expected, parts)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    for t, ref, what in zip((root7, seg_roots, lanes), alone_out, ("model root", "per-tensor roots", "batch lanes")):
        if not torch.equal(t, ref):
            sys.exit("bench.py: %s of the overlapped step differ from the same call run alone" % what)
    ms_per_step = 1e3 * dt / args.steps
    value = step_bytes / (dt / args.steps) / 1e9
    ms70_in_step = statistics.mean(p[0] for p in parts)
    ms_gpu_step = statistics.mean(p[3] for p in parts)
    ms7_in_step = statistics.mean(p[1] for p in parts)
    mslt_in_step = statistics.mean(p[2] for p in parts)
    # each part on its own, the chip to itself (--no-extras: the step and nothing else is launched)
    ms70 = ms7 = mslt = None
    if not args.no_extras:
        ms70 = alone(lambda: part_70b(stream))
        ms7 = alone(lambda: part_7b(stream))
        mslt = alone(lambda: part_batch(stream))

    # ---------------- roofline of the dominant kernel (SHA-256 leaf kernel, 70B stream) ----------------
    n_leaves70 = -(-bytes70 // LEAF70)
    full_leaves = bytes70 // LEAF70
    # the leaf kernel hashes every leaf and folds each group of 64 leaf digests (one wave) in LDS
    groups = -(-n_leaves70 // 64)
    mix_leaf_kernel = merkle_mix(full_leaves, LEAF70, n_leaves70 - groups)
    if n_leaves70 != full_leaves:
        mix_leaf_kernel = mix_leaf_kernel + ((bytes70 - full_leaves * LEAF70) // 64 + 1) * SHA_BLOCK_MIX
    ops_leaf_kernel = mix_leaf_kernel.total()
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath) and not args.quick:
        traffic = json.load(open(tpath)).get("merkle_leaf_kernel_c5_bytes_per_launch")
    # Inside the step the kernel shares the chip with the other two parts (unless --schedule serial or
    # pair), so its launch takes longer than it does alone while the chip as a whole does more: the
    # kernel's own figures come first, as it runs in the timed region; beside them the same launch with
    # the chip to itself, and all the operations of the step over the step's time.  `frac` is against the
    # nominal peak (one instruction per SIMD per four cycles at 2.4 GHz), `issue_frac` against
    # `issue_bound`, the rate at which the chip can issue this kernel's instruction mix.
    achieved = ops_leaf_kernel / (ms70_in_step * 1e-3)
    bound_leaf = issue_bound(mix_leaf_kernel)
    mix_step = (sha_tree_mix([bytes70], LEAF70, flat=True) + sha_tree_mix(t7_lens, LEAF7) + lthash_mix(lengths[b0:b1]))
    ops_step, bound_step = mix_step.total(), issue_bound(mix_step)
    roofline = {"kernel": "merkle_leaf_kernel (SHA-256 leaves + 6 in-LDS tree levels), 70B stream, 64 KiB leaves",
                "bound": "alu", "achieved": achieved / 1e12, "peak": ALU_PEAK_OPS / 1e12, "unit": "TOP/s",
                "frac": achieved / ALU_PEAK_OPS, "issue_bound": bound_leaf / 1e12, "issue_frac": achieved / bound_leaf,
                "traffic": traffic,
                "ms_per_launch": ms70_in_step, "algorithmic_ops_per_launch": ops_leaf_kernel,
                "algorithmic_bytes_per_launch": bytes70 + 32 * groups,
                "hbm_frac": (bytes70 + 32 * groups) / (ms70_in_step * 1e-3) / HBM_PEAK,
                "shares_the_chip": args.schedule == "overlap",
                "alone": None if ms70 is None else {"ms_per_launch": ms70, "achieved": ops_leaf_kernel / (ms70 * 1e-3) / 1e12,
                                                    "frac": ops_leaf_kernel / (ms70 * 1e-3) / ALU_PEAK_OPS,
                                                    "issue_frac": ops_leaf_kernel / (ms70 * 1e-3) / bound_leaf},
                "whole_step": {"algorithmic_ops": ops_step, "ms": ms_gpu_step,
                               "achieved": ops_step / (ms_gpu_step * 1e-3) / 1e12,
                               "frac": ops_step / (ms_gpu_step * 1e-3) / ALU_PEAK_OPS,
                               "issue_bound": bound_step / 1e12,
                               "issue_frac": ops_step / (ms_gpu_step * 1e-3) / bound_step},
                "issue_rates_TOP/s": {"table": ISSUE_RATE_TOPS, "this_run": live_rates}}

    # every entry: GB/s hashed, and the fractions of the integer-ALU roofline (instructions of the hash's
    # mix x 64 lanes / time: against the nominal 39.3 T and against the issue rate of that mix) and of the
    # HBM roofline (bytes hashed / time / 8 TB/s)
    per_config = {}
    if not args.no_extras:
        per_config = {
            "C5_merkle_70b_64KiB_resident": rated({"GB/s": bytes70 / ms70 / 1e6, "ms": ms70, "bytes": bytes70},
                                                  sha_tree_mix([bytes70], LEAF70, flat=True)),
            "C3_merkle_7b_segments_1MiB": rated({"GB/s": bytes7 / ms7 / 1e6, "ms": ms7, "bytes": bytes7,
                                                 "leaves": sum(max(1, -(-l // LEAF7)) for l in t7_lens)},
                                                sha_tree_mix(t7_lens, LEAF7)),
            "C4_lthash_one_8GB_batch_resident": rated({"GB/s": rec_bytes / mslt / 1e6, "ms": mslt, "bytes": rec_bytes,
                                                       "samples/s": n_rec / (mslt * 1e-3), "records": n_rec,
                                                       "longest_record": int(lengths[b0:b1].max())},
                                                      lthash_mix(lengths[b0:b1])),
        }
        # the chain floors of the two chain-bound parts of the step: a full 1 MiB leaf and its tensor's tree
        # levels; the longest record of the batch
        max_leaves7 = max(-(-l // LEAF7) for l in t7_lens)
        chain_bound(per_config["C3_merkle_7b_segments_1MiB"],
                    (LEAF7 // 64 + 1) * SHA_CONSUMER_INSTRS + (tree_levels(max_leaves7) + tree_levels(len(t7_lens))) * SHA_NODE_INSTRS)
        chain_bound(per_config["C4_lthash_one_8GB_batch_resident"],
                    -(-int(lengths[b0:b1].max()) // 128) * B2_FOUR_LANE_INSTRS)


    def timed_call(fn, reps, warm=2):
        """Time of one call in ms: the median over all timed calls.  Short calls (reps >= 30) are timed in
        three series, because now and then a whole series of sub-millisecond calls runs some 10 us per call
        slower than the next one in the same process; the medians of the series and the fastest and slowest
        single call go into the entry beside the overall median (rated() copies them)."""
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        series = []
        for _ in range(3 if reps >= 30 else 1):
            ts = []
            for _ in range(reps):
                a.record()
                fn()
                b.record()
                b.synchronize()
                ts.append(a.elapsed_time(b))
            series.append(ts)
        every = [t for ts in series for t in ts]
        ms = Timed(statistics.median(every))
        ms.spread = {"ms_min": min(every), "ms_max": max(every), "calls": len(every),
                     "ms_series_medians": [statistics.median(ts) for ts in series]}
        return ms

    streaming = None
    if not args.no_extras:
        log("side measurements: configs 1 and 2, streaming legs")
        c1 = wl.uniform_bytes(wl.SEED_C1, 0, 16 << 20, device=dev)
        ms = timed_call(lambda: sentry.sentry_merkle_root(c1.data_ptr(), c1.numel(), 4096, root7.data_ptr(), stream), 50)
        per_config["C1_merkle_16MiB_4KiB"] = chain_bound(
            rated({"GB/s": c1.numel() / ms / 1e6, "ms": ms, "bytes": c1.numel()}, sha_tree_mix([c1.numel()], 4096, flat=True)),
            (4096 // 64 + 1) * SHA_CONSUMER_INSTRS + tree_levels(c1.numel() // 4096) * SHA_NODE_SPLIT_INSTRS)
        img, ioff = wl.image_records(50_000, device=dev)
        d_ioff = torch.from_numpy(ioff.view(np.int64).copy()).to(dev)
        ms = timed_call(lambda: sentry.sentry_lthash(img.data_ptr(), d_ioff.data_ptr(), 50_000, lanes.data_ptr(), stream), 50)
        per_config["C2_lthash_50k_images"] = rated({"GB/s": img.numel() / ms / 1e6, "ms": ms, "bytes": img.numel(),
                                                    "samples/s": 50_000 / (ms * 1e-3)}, lthash_mix([3072] * 50_000))
        # config 5 per tensor as well (Algorithm 2 over the 723 tensors of the 70B checkpoint where they lie
        # in the resident buffer, 64 KiB leaves): per-tensor roots and the root over them
        if not args.merkle_prefix_gib:
            offs70 = wl.checkpoint_offsets(lay70)
            p70 = [ckpt70.data_ptr() + offs70[i] for i in range(len(lay70))]
            l70 = [offs70[i + 1] - offs70[i] for i in range(len(lay70))]
            roots70 = torch.zeros(32 * len(lay70), dtype=torch.uint8, device=dev)
            ms = timed_call(lambda: sentry.sentry_merkle_segments(p70, l70, LEAF70, roots70.data_ptr(), root7.data_ptr(), stream), 3)
            per_config["C5_merkle_70b_per_tensor_64KiB"] = rated({"GB/s": bytes70 / ms / 1e6, "ms": ms, "bytes": bytes70,
                                                                  "tensors": len(lay70)}, sha_tree_mix(l70, LEAF70))
        # the 7B checkpoint as one flat tree over all blocks of all tensors (Algorithm 3)
        ms = timed_call(lambda: sentry.sentry_merkle_inplace(t7_ptrs, t7_lens, LEAF7, root7.data_ptr(), stream), 5)
        per_config["F3_merkle_7b_inplace_flat_1MiB"] = rated({"GB/s": bytes7 / ms / 1e6, "ms": ms, "bytes": bytes7},
                                                             sha_tree_mix(t7_lens, LEAF7, flat=True))
        ms = timed_call(lambda: sentry.sentry_merkle_inplace(t7_ptrs, t7_lens, 8192, root7.data_ptr(), stream), 5)
        per_config["F3_merkle_7b_inplace_flat_8KiB"] = rated({"GB/s": bytes7 / ms / 1e6, "ms": ms, "bytes": bytes7},
                                                             sha_tree_mix(t7_lens, 8192, flat=True))
        # the same checkpoint as one zero-padded byte stream (Algorithm 1, coalesced hashing), 8 KiB blocks:
        # hashed where the tensors lie (only blocks that span tensors are gathered), and the scheme as
        # stated, through a coalesced copy in a second buffer (the copy reads and writes every byte once more)
        pad7 = -(-bytes7 // 8192) * 8192
        ms = timed_call(lambda: sentry.sentry_merkle_coalesced(t7_ptrs, t7_lens, 8192, 0, 0, root7.data_ptr(), stream), 5)
        per_config["A1_merkle_7b_coalesced_in_place_8KiB"] = rated({"GB/s": bytes7 / ms / 1e6, "ms": ms, "bytes": bytes7},
                                                                    sha_tree_mix([pad7], 8192, flat=True))
        cbuf = torch.empty(pad7, dtype=torch.uint8, device=dev)
        ms_c = timed_call(lambda: sentry.sentry_merkle_coalesced(t7_ptrs, t7_lens, 8192, cbuf.data_ptr(), pad7,
                                                                 root7.data_ptr(), stream), 5)
        ms_r = timed_call(lambda: sentry.sentry_merkle_root(cbuf.data_ptr(), pad7, 8192, root7.data_ptr(), stream), 5)
        e = rated({"GB/s": bytes7 / ms_c / 1e6, "ms": ms_c, "bytes": bytes7}, sha_tree_mix([pad7], 8192, flat=True),
                  hbm_bytes=3 * bytes7)
        e["copy_ms"] = ms_c - ms_r            # the gather kernel: the call less the tree over the filled buffer
        e["copy_TB/s_read_plus_write"] = 2 * bytes7 / (ms_c - ms_r) / 1e9
        per_config["A1_merkle_7b_coalesced_with_copy_8KiB"] = e
        del cbuf
        # small models in the shapes of the paper's own model runs (transformer stacks of BERT-base and GPT2-XL size,
        # synthetic bf16 weights, one allocation per tensor), the paper's default 8 KiB blocks, the four schemes.
        # Launches with fewer leaves than lanes: one 8 KiB leaf is a serial chain of 129 compressions (0.25 ms).
        for shape, lay_s in (("bert_base_like_12x768", wl.llama_layout(12, 768, 3072, 30522)),
                             ("gpt2_xl_like_48x1600", wl.llama_layout(48, 1600, 6400, 50257))):
            ts = [wl.checkpoint_tensor(lay_s, i, base_seed=wl.SEED_C3 + 5, device=dev) for i in range(len(lay_s))]
            ps, ls = [t.data_ptr() for t in ts], [t.numel() * 2 for t in ts]
            nb = sum(ls)
            roots_s = torch.zeros(32 * len(ls), dtype=torch.uint8, device=dev)
            lanes_s = torch.zeros(32, dtype=torch.int16, device=dev)
            for scheme, call, mix in (
                    ("coalesced_alg1", lambda st: sentry.sentry_merkle_coalesced(ps, ls, 8192, 0, 0, root7.data_ptr(), st),
                     sha_tree_mix([-(-nb // 8192) * 8192], 8192, flat=True)),
                    ("per_layer_alg2", lambda st: sentry.sentry_merkle_segments(ps, ls, 8192, roots_s.data_ptr(), root7.data_ptr(), st),
                     sha_tree_mix(ls, 8192)),
                    ("in_place_alg3", lambda st: sentry.sentry_merkle_inplace(ps, ls, 8192, root7.data_ptr(), st),
                     sha_tree_mix(ls, 8192, flat=True)),
                    ("lattice_alg4", lambda st: sentry.sentry_lthash_model(ps, ls, 8192, 0, lanes_s.data_ptr(), st),
                     model_lthash_mix(ls, 8192))):
                ms = timed_call(lambda: call(stream), 20)
                # the scheme's extra GPU memory (section 5.2, memory usage): what the library holds for a stream
                # that has made this one call
                own = torch.cuda.Stream()
                unused = sentry.sentry_scratch_bytes(own.cuda_stream) == (0, 0)    # torch hands out streams from a pool
                call(own.cuda_stream)
                own.synchronize()
                extra = sentry.sentry_scratch_bytes(own.cuda_stream)[0] if unused else None
                per_config["E1_%s_%s_8KiB" % (shape, scheme)] = rated(
                    {"GB/s": nb / ms / 1e6, "ms": ms, "bytes": nb, "tensors": len(ls), "extra_device_bytes": extra,
                     "extra_per_model_byte": extra / nb if unused else None}, mix)
            del ts, roots_s
        # the three leaf functions of section 4.2.1 on the first 16 GiB of the 70B stream, 8 KiB leaves
        f4_bytes = min(bytes70, 16 << 30)
        big_root = torch.zeros(64, dtype=torch.uint8, device=dev)
        for name, hid in (("sha256", sentry.HASH_SHA256), ("blake2b", sentry.HASH_BLAKE2B), ("sha3_256", sentry.HASH_SHA3_256)):
            ms = timed_call(lambda: sentry.sentry_merkle_root_h(hid, ckpt70.data_ptr(), f4_bytes, 8192,
                                                                big_root.data_ptr(), stream), 5)
            ops = (sha_tree_mix([f4_bytes], 8192, flat=True) if name == "sha256"
                   else other_tree_mix(name, [f4_bytes], 8192, flat=True))
            per_config["F4_merkle_%s_16GiB_8KiB" % name] = rated({"GB/s": f4_bytes / ms / 1e6, "ms": ms, "bytes": f4_bytes}, ops)
        # the paper's three schemes' hardest case: fragmented 7B checkpoint, per-tensor and flat trees, 8 KiB blocks
        seg_roots = torch.zeros(64 * len(t7_ptrs), dtype=torch.uint8, device=dev)
        for name, hid in (("blake2b", sentry.HASH_BLAKE2B), ("sha3_256", sentry.HASH_SHA3_256)):
            ms = timed_call(lambda: sentry.sentry_merkle_segments_h(hid, t7_ptrs, t7_lens, 8192, seg_roots.data_ptr(),
                                                                    big_root.data_ptr(), stream), 5)
            per_config["F4_merkle_%s_7b_per_tensor_8KiB" % name] = rated(
                {"GB/s": bytes7 / ms / 1e6, "ms": ms, "bytes": bytes7}, other_tree_mix(name, t7_lens, 8192))
            ms = timed_call(lambda: sentry.sentry_merkle_inplace_h(hid, t7_ptrs, t7_lens, 8192, big_root.data_ptr(),
                                                                   stream), 5)
            per_config["F4_merkle_%s_7b_inplace_flat_8KiB" % name] = rated(
                {"GB/s": bytes7 / ms / 1e6, "ms": ms, "bytes": bytes7}, other_tree_mix(name, t7_lens, 8192, flat=True))
        # lattice hash of the 7B checkpoint (Algorithm 4), the paper's default 8 KiB blocks
        mlanes = torch.zeros(32, dtype=torch.int16, device=dev)
        ms = timed_call(lambda: sentry.sentry_lthash_model(t7_ptrs, t7_lens, 8192, 0, mlanes.data_ptr(), stream), 5)
        per_config["F2_lthash_model_7b_8KiB"] = rated({"GB/s": bytes7 / ms / 1e6, "ms": ms, "bytes": bytes7},
                                                      model_lthash_mix(t7_lens, 8192))
        # mixed-source batches (section 4.3): the same 50,000 samples from 1, 16 and 128 sources whose shares
        # are drawn from a Dirichlet distribution with concentration 1, as in the paper's run over the number of sources
        for n_src in (1, 16, 128):
            ids = torch.from_numpy(wl.dirichlet_source_ids(50_000, n_src, wl.SEED_C2 + 7).view(np.int32)).to(dev)
            acc = torch.zeros(n_src * 1024, dtype=torch.int16, device=dev)
            ms = timed_call(lambda: sentry.sentry_lthash_sources(img.data_ptr(), d_ioff.data_ptr(), ids.data_ptr(),
                                                                 50_000, n_src, acc.data_ptr(), stream), 30)
            per_config["F1_lthash_50k_images_%d_sources" % n_src] = rated(
                {"GB/s": img.numel() / ms / 1e6, "ms": ms, "bytes": img.numel(), "samples/s": 50_000 / (ms * 1e-3)},
                lthash_mix([3072] * 50_000))
            acc32 = torch.zeros(n_src * 32, dtype=torch.int16, device=dev)
            ms = timed_call(lambda: sentry.sentry_lthash32_sources(img.data_ptr(), d_ioff.data_ptr(), ids.data_ptr(),
                                                                   50_000, n_src, acc32.data_ptr(), stream), 30)
            per_config["F1_lthash32_50k_images_%d_sources" % n_src] = rated(
                {"GB/s": img.numel() / ms / 1e6, "ms": ms, "bytes": img.numel(), "samples/s": 50_000 / (ms * 1e-3)},
                lthash32_mix([3072] * 50_000))
        # the same 50,000 samples through the call for samples of one size (no offsets array: the host knows
        # the batch and launches only the kernels that have work)
        ms = timed_call(lambda: sentry.sentry_lthash_fixed(img.data_ptr(), 3072, 50_000, lanes.data_ptr(), stream), 50)
        per_config["C2_lthash_50k_images_fixed_size_call"] = rated(
            {"GB/s": img.numel() / ms / 1e6, "ms": ms, "bytes": img.numel(), "samples/s": 50_000 / (ms * 1e-3)},
            lthash_mix([3072] * 50_000))
        # the same 50,000 samples at the paper's own digest width: plain BLAKE2b-512, 32 partitions (section 4.2.2)
        lanes32 = torch.zeros(32, dtype=torch.int16, device=dev)
        ms = timed_call(lambda: sentry.sentry_lthash32_fixed(img.data_ptr(), 3072, 50_000, lanes32.data_ptr(), stream), 50)
        per_config["F2_lthash32_50k_images_fixed_size_call"] = rated(
            {"GB/s": img.numel() / ms / 1e6, "ms": ms, "bytes": img.numel(), "samples/s": 50_000 / (ms * 1e-3)},
            lthash32_mix([3072] * 50_000))
        ms = timed_call(lambda: sentry.sentry_lthash32(img.data_ptr(), d_ioff.data_ptr(), 50_000, lanes32.data_ptr(), stream), 50)
        per_config["F2_lthash32_50k_images"] = rated(
            {"GB/s": img.numel() / ms / 1e6, "ms": ms, "bytes": img.numel(), "samples/s": 50_000 / (ms * 1e-3)},
            lthash32_mix([3072] * 50_000))
        # the lane sum taken alone, over digests that are already in memory (any 2048 bytes are a valid
        # digest row: the first 2 GiB of the 70B stream stand in for 2^20 of them): bound by HBM
        n_rows = min(1 << 20, bytes70 // 2048)
        ms = timed_call(lambda: sentry.sentry_lthash_sum(ckpt70.data_ptr(), n_rows, lanes.data_ptr(), stream), 20)
        per_config["L3_lane_sum_alone_%d_digests" % n_rows] = rated(
            {"GB/s": 2048 * n_rows / ms / 1e6, "ms": ms, "bytes": 2048 * n_rows, "samples/s": n_rows / (ms * 1e-3),
             "bound": "hbm"}, Mix({"v_pk_add_u16": 512 * n_rows}))
        # and the digests of the 50,000 images written out one by one (2048 bytes per sample)
        rows = torch.empty(50_000 * 2048, dtype=torch.uint8, device=dev)
        ms = timed_call(lambda: sentry.sentry_lthash_digests(img.data_ptr(), d_ioff.data_ptr(), 50_000, rows.data_ptr(), stream), 50)
        per_config["L2_digests_50k_images"] = rated(
            {"GB/s": img.numel() / ms / 1e6, "ms": ms, "bytes": img.numel(), "samples/s": 50_000 / (ms * 1e-3)},
            lthash_mix([3072] * 50_000), hbm_bytes=img.numel() + rows.numel())
        del rows
        # the 50,000 images as a data pipeline hands them over (batches of 128 samples from 16 sources, as in the
        # paper's pipeline runs): one per-source call per batch into running sums, 391 calls back to back on one
        # stream, and dealt over four streams (each with running sums of its own, which add up); host time included
        ids16 = torch.from_numpy(wl.dirichlet_source_ids(50_000, 16, wl.SEED_C2 + 9).view(np.int32)).to(dev)
        # (batches of 32 and 512, the ends of the paper's range of batch sizes, on one stream at 1024 lanes)
        for n_streams, batch in ((1, 128), (4, 128), (1, 32), (1, 512)):
            pipe_streams = [torch.cuda.Stream() for _ in range(n_streams)]
            for name, call, lanes_per in (("lthash", sentry.sentry_lthash_sources, 1024), ("lthash32", sentry.sentry_lthash32_sources, 32)):
                if batch != 128 and name != "lthash":
                    continue
                accs = [torch.zeros(16 * lanes_per, dtype=torch.int16, device=dev) for _ in range(n_streams)]
                torch.cuda.synchronize()
                n_calls = -(-50_000 // batch)

                def whole_dataset():
                    for k, a in enumerate(range(0, 50_000, batch)):
                        n = min(batch, 50_000 - a)
                        call(img.data_ptr() + 3072 * a, d_ioff.data_ptr(), ids16.data_ptr() + 4 * a, n, 16,
                             accs[k % n_streams].data_ptr(), pipe_streams[k % n_streams].cuda_stream)
                    torch.cuda.synchronize()

                whole_dataset()
                ts = []
                for _ in range(3):
                    t0 = time.perf_counter()
                    whole_dataset()
                    ts.append((time.perf_counter() - t0) * 1e3)
                ms = statistics.median(ts)
                per_config["E4_%s_50k_images_batches_of_%d_16_sources_%d_stream%s" % (name, batch, n_streams, "s" if n_streams > 1 else "")] = rated(
                    {"GB/s": img.numel() / ms / 1e6, "ms": ms, "bytes": img.numel(), "samples/s": 50_000 / (ms * 1e-3), "calls": n_calls,
                     "us_per_call": ms * 1e3 / n_calls, "clock": "host wall time around all calls and the final synchronisation"},
                    (lthash_mix if name == "lthash" else lthash32_mix)([3072] * 50_000))
        # the same for a text data set in the shape of the paper's second one (section 5: 40,000 samples of varying
        # length, padded to one length inside a batch, which is then the block size of the dataset kernel; batches of
        # 128 from 16 sources): lengths log-normal around 600 bytes, every batch padded to its longest sample
        t_lens = wl.lognormal_record_lengths(40_000, seed=wl.SEED_C2 + 21, median=600, sigma=0.4, lo=64, hi=4096)
        t_pad = [(int(t_lens[a:a + 128].max()) + 15) // 16 * 16 for a in range(0, 40_000, 128)]
        t_cnt = [min(128, 40_000 - a) for a in range(0, 40_000, 128)]
        t_base = np.concatenate([[0], np.cumsum([p * c for p, c in zip(t_pad, t_cnt)])]).astype(np.int64)
        text = wl.uniform_bytes(wl.SEED_C2 + 22, 0, int(t_base[-1]), device=dev)
        t_off = torch.from_numpy(np.concatenate([np.arange(129, dtype=np.int64) * p for p in t_pad])).to(dev)
        t_ids = torch.from_numpy(wl.dirichlet_source_ids(40_000, 16, wl.SEED_C2 + 23).view(np.int32)).to(dev)
        t_mix_lens = [p for p, c in zip(t_pad, t_cnt) for _ in range(c)]
        text_stream = torch.cuda.Stream()
        for name, call, lanes_per in (("lthash", sentry.sentry_lthash_sources, 1024), ("lthash32", sentry.sentry_lthash32_sources, 32)):
            acc_t = torch.zeros(16 * lanes_per, dtype=torch.int16, device=dev)
            torch.cuda.synchronize()

            def whole_text_set():
                for k in range(len(t_pad)):
                    call(text.data_ptr() + int(t_base[k]), t_off.data_ptr() + 8 * 129 * k, t_ids.data_ptr() + 4 * 128 * k,
                         t_cnt[k], 16, acc_t.data_ptr(), text_stream.cuda_stream)
                torch.cuda.synchronize()

            whole_text_set()
            ts = []
            for _ in range(3):
                t0 = time.perf_counter()
                whole_text_set()
                ts.append((time.perf_counter() - t0) * 1e3)
            ms = statistics.median(ts)
            per_config["E4_%s_40k_text_samples_batches_of_128_16_sources_1_stream" % name] = rated(
                {"GB/s": int(t_base[-1]) / ms / 1e6, "ms": ms, "bytes": int(t_base[-1]), "samples/s": 40_000 / (ms * 1e-3),
                 "calls": len(t_pad), "us_per_call": ms * 1e3 / len(t_pad), "mean_padded_bytes": int(t_base[-1]) // 40_000,
                 "clock": "host wall time around all calls and the final synchronisation"},
                (lthash_mix if name == "lthash" else lthash32_mix)(t_mix_lens))
        del text, t_off, t_ids
        # what a HIP graph buys such a pipeline: the per-source call on a batch buffer (a pipeline hands every batch
        # over in the same buffer) captured once and replayed 391 times, against the same 391 calls issued one by one;
        # both running sums must come out equal
        gs = torch.cuda.Stream()
        for name, call, lanes_per in (() if args.no_graph else
                                      (("lthash", sentry.sentry_lthash_sources, 1024), ("lthash32", sentry.sentry_lthash32_sources, 32))):
            acc_e = torch.zeros(16 * lanes_per, dtype=torch.int16, device=dev)
            acc_g = torch.zeros(16 * lanes_per, dtype=torch.int16, device=dev)
            torch.cuda.synchronize()

            def one_batch(acc):
                call(img.data_ptr(), d_ioff.data_ptr(), ids16.data_ptr(), 128, 16, acc.data_ptr(), gs.cuda_stream)

            one_batch(acc_e)                      # the stream's scratch has its size before the capture
            torch.cuda.synchronize()
            try:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=gs):
                    one_batch(acc_g)
            except Exception as e:                # a side measurement: the line does not depend on it
                log("graph capture of %s failed, entry left out: %s" % (name, e))
                torch.cuda.synchronize()
                continue
            ms_by = {}
            acc_e.zero_()
            acc_g.zero_()
            torch.cuda.synchronize()
            for kind in ("calls", "graph_replays"):
                ts = []
                for _ in range(4):                # the first pass warms up
                    t0 = time.perf_counter()
                    for _k in range(391):
                        if kind == "calls":
                            one_batch(acc_e)
                        else:
                            graph.replay()
                    torch.cuda.synchronize()
                    ts.append((time.perf_counter() - t0) * 1e3)
                ms_by[kind] = statistics.median(ts[1:])
            torch.cuda.synchronize()
            if not torch.equal(acc_e, acc_g):
                raise SystemExit("bench: the replayed graph and the eager calls disagree (%s)" % name)
            ms = ms_by["graph_replays"]
            per_config["E4_%s_batch_of_128_16_sources_graph_replayed_391_times" % name] = rated(
                {"GB/s": 391 * 128 * 3072 / ms / 1e6, "ms": ms, "bytes": 391 * 128 * 3072, "samples/s": 391 * 128 / (ms * 1e-3),
                 "calls": 391, "us_per_call": ms * 1e3 / 391, "us_per_call_without_graph": ms_by["calls"] * 1e3 / 391,
                 "clock": "host wall time around all replays and the final synchronisation"},
                (lthash_mix if name == "lthash" else lthash32_mix)([3072] * (391 * 128)))
            del graph
        del ids16
        if not args.no_streaming:
            # host-to-device streaming in the shape of configs 5 and 4, from a pinned host buffer of 16 GB:
            # Merkle while loading in 1 GiB chunks, and the lattice hash of 8 GB batches, each against the
            # plain copy of the same bytes; then one full streamed pass of each configuration (137.95 GB in
            # 129 chunks; 159.64 GB in the 20 batches of config 4, with their true record boundaries), fed
            # chunk by chunk from the same pinned buffer used round-robin (the bytes repeat, which the time
            # does not see; the full-size digests are checked against the oracle's in tests/).
            if args.quick:
                hbytes, chunk = 1 << 28, 1 << 26
            else:
                hbytes, chunk = 16 << 30, 1 << 30
            hbytes = max(hbytes, 2 * rec_bytes)
            host = torch.empty(hbytes, dtype=torch.uint8).pin_memory()
            stage = torch.empty(hbytes, dtype=torch.uint8, device=dev)
            m_bytes = min(hbytes, bytes70) // LEAF70 * LEAF70
            host[:m_bytes].copy_(ckpt70[:m_bytes])
            ms_copy = timed_call(lambda: stage[:m_bytes].copy_(host[:m_bytes], non_blocking=True), 3)

            def merkle_fed(total):
                """`total` bytes fed in chunks to one tree through the library's load path."""
                state = sentry.sentry_merkle_stream_begin(total, LEAF70)
                pos = 0
                while pos < total:
                    n = min(chunk, total - pos)
                    at = pos % m_bytes
                    if at + n > m_bytes:
                        at = 0
                    sentry.sentry_merkle_stream_update_h2d(state, host.data_ptr() + at, n, stream)
                    pos += n
                sentry.sentry_merkle_stream_final(state, root7.data_ptr(), stream)

            ms_m = timed_call(lambda: merkle_fed(m_bytes), 3)
            sentry.sentry_merkle_root(ckpt70.data_ptr(), m_bytes, LEAF70, root70.data_ptr(), stream)
            torch.cuda.synchronize()
            if bytes(root7.cpu().numpy()) != bytes(root70.cpu().numpy()):
                sys.exit("bench.py: Merkle root while loading differs from the root of the resident bytes")
            ms_m_call = timed_call(lambda: sentry.sentry_merkle_root_h2d(host.data_ptr(), m_bytes, LEAF70, chunk,
                                                                         root7.data_ptr(), stream), 3)
            full_m = bytes70 if not args.merkle_prefix_gib else m_bytes
            ms_m_full = timed_call(lambda: merkle_fed(full_m), 1, warm=0)
            # lattice: the resident batch twice in pinned memory
            lt_bytes = 2 * rec_bytes
            host[:rec_bytes].copy_(records)
            host[rec_bytes:lt_bytes].copy_(records)
            rel = rec_off - rec_off[0]
            h_off = torch.from_numpy(np.concatenate([rel, rel[1:] + np.uint64(rec_bytes)]).view(np.int64).copy()).pin_memory()
            ms_copy_l = timed_call(lambda: stage[:lt_bytes].copy_(host[:lt_bytes], non_blocking=True), 3)
            lanes2 = torch.zeros(1024, dtype=torch.int16, device=dev)
            ms_l = timed_call(lambda: sentry.sentry_lthash_h2d(host.data_ptr(), h_off.data_ptr(), 2 * n_rec, rec_bytes,
                                                               lanes2.data_ptr(), stream), 3)
            sentry.sentry_lthash(records.data_ptr(), d_off.data_ptr(), n_rec, lanes.data_ptr(), stream)
            sentry.sentry_lthash_combine(lanes.data_ptr(), lanes.data_ptr(), stream)      # the batch twice
            torch.cuda.synchronize()
            if (lanes.cpu() != lanes2.cpu()).any():
                sys.exit("bench.py: lattice hash while loading differs from the hash of the resident batch")
            # the full pass: every batch of the configuration with its own record boundaries, batch k read from
            # half k % 2 of the pinned buffer
            all_batches = wl.cut_batches(offsets, batch_bytes)
            half = hbytes // 2
            b_offs = []
            for k, (a0, a1) in enumerate(all_batches):
                o = offsets[a0:a1 + 1] - offsets[a0] + np.uint64((k & 1) * half)
                b_offs.append((torch.from_numpy(o.view(np.int64).copy()).pin_memory(), a1 - a0, int(offsets[a1] - offsets[a0])))

            def lattice_fed(n_batches):
                state = sentry.sentry_lthash_stream_begin()
                for o, cnt, _ in b_offs[:n_batches]:
                    sentry.sentry_lthash_stream_update_h2d(state, host.data_ptr(), o.data_ptr(), cnt, stream)
                sentry.sentry_lthash_stream_final(state, lanes2.data_ptr(), stream)

            lattice_fed(min(3, len(b_offs)))      # sizes the staging buffers
            torch.cuda.synchronize()
            ms_l2 = timed_call(lambda: lattice_fed(2), 3, warm=1)
            ms_l_full = timed_call(lambda: lattice_fed(len(b_offs)), 1, warm=0)
            full_l = sum(nb for _, _, nb in b_offs)
            two_l = sum(nb for _, _, nb in b_offs[:2])
            copy_rate_l = lt_bytes / ms_copy_l / 1e6       # GB/s of the plain copy
            steady = (ms_l_full - ms_l2) / max(len(b_offs) - 2, 1)      # ms per further batch once the pipeline runs
            # top level of each leg: the full streamed pass of the configuration; beside it the short runs
            copy_rate_m = m_bytes / ms_copy / 1e6
            streaming = {"pinned_bytes": hbytes,
                         "merkle": {"entry_point": "sentry_merkle_stream_update_h2d per chunk", "bytes": full_m,
                                    "chunk_bytes": chunk, "chunks": -(-full_m // chunk), "ms": float(ms_m_full),
                                    "copy_only_GB/s": copy_rate_m, "h2d_GB/s": full_m / ms_m_full / 1e6,
                                    "overlap_efficiency": (full_m / ms_m_full / 1e6) / copy_rate_m,
                                    "sixteen_chunks": {"bytes": m_bytes, "h2d_GB/s": m_bytes / ms_m / 1e6,
                                                       "overlap_efficiency": ms_copy / ms_m,
                                                       "one_call_sentry_merkle_root_h2d_GB/s": m_bytes / ms_m_call / 1e6}},
                         "lthash": {"entry_point": "sentry_lthash_stream_update_h2d per batch", "bytes": full_l,
                                    "batch_bytes": batch_bytes, "batches": len(b_offs), "records": int(sum(c for _, c, _ in b_offs)),
                                    "ms": float(ms_l_full), "copy_only_GB/s": copy_rate_l, "h2d_GB/s": full_l / ms_l_full / 1e6,
                                    "overlap_efficiency": (full_l / ms_l_full / 1e6) / copy_rate_l,
                                    "first_two_batches_ms": float(ms_l2), "steady_state_ms_per_batch": steady,
                                    "steady_state_efficiency": ((full_l - two_l) / max(len(b_offs) - 2, 1) / steady / 1e6) / copy_rate_l
                                    if steady > 0 else None,
                                    "tail_ms": float(ms_l2) - two_l / 1e6 / copy_rate_l,
                                    "two_batches_one_call_sentry_lthash_h2d": {"bytes": lt_bytes, "h2d_GB/s": lt_bytes / ms_l / 1e6,
                                                                               "overlap_efficiency": ms_copy_l / ms_l}}}
            del host, stage

    # ---------------- CPU baseline: the oracle, one thread, on a bounded sample ----------------
    # Configs 1 and 2 in full; of the three big configurations the first 4 GiB of the 70B stream (config 5),
    # the first 2 GB of the 7B checkpoint's tensors (config 3, per-tensor roots) and the first 2 GB of the
    # batch (config 4): about 20 s of single-thread work.  More is not run: the default bench run has to
    # finish within minutes, and the oracle's rate does not depend on how much it is given.
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        log("CPU baseline (oracle, 1 thread)")
        m_bytes = (64 << 20) if args.quick else (4 << 30)
        l_bytes = (32 << 20) if args.quick else 2_000_000_000
        s_bytes = (32 << 20) if args.quick else 2_000_000_000
        parts = {}

        def cpu_leg(name, nbytes, cpu_fn, gpu_fn):
            t = time.perf_counter()
            want = cpu_fn()
            sec = time.perf_counter() - t
            got = gpu_fn()
            if got != want:
                sys.exit("bench.py: GPU result differs from the oracle on the CPU-baseline sample (%s)" % name)
            parts[name] = {"bytes": nbytes, "s": sec, "GB/s": nbytes / sec / 1e9}

        def gpu_root(ptr, n, leaf):
            sentry.sentry_merkle_root(ptr, n, leaf, root7.data_ptr(), stream)
            torch.cuda.synchronize()
            return bytes(root7.cpu().numpy())

        def gpu_lanes(d, o, n):
            sentry.sentry_lthash(d.data_ptr(), o.data_ptr(), n, lanes.data_ptr(), stream)
            torch.cuda.synchronize()
            return lanes.cpu().numpy().view(np.uint16).tobytes()

        sample_m = ckpt70[:m_bytes].cpu().numpy()
        cpu_leg("c5_prefix", m_bytes, lambda: oracle.merkle_root(sample_m, LEAF70), lambda: gpu_root(ckpt70.data_ptr(), m_bytes, LEAF70))
        nb = int(np.searchsorted(rec_off - rec_off[0], np.uint64(l_bytes), side="right")) - 1
        lt_b = int(rec_off[nb] - rec_off[0])
        sample_l = records[:lt_b].cpu().numpy()
        sample_off = (rec_off[:nb + 1] - rec_off[0]).copy()
        cpu_leg("c4_prefix", lt_b, lambda: oracle.lthash(sample_l, sample_off).tobytes(), lambda: gpu_lanes(records, d_off, nb))
        # config 3: the tensors of the 7B checkpoint in order until the sample is full
        n_t, acc_b = 0, 0
        while n_t < len(t7) and (n_t == 0 or acc_b + t7_lens[n_t] <= s_bytes):
            acc_b += t7_lens[n_t]
            n_t += 1
        segs = [t7[i].view(torch.uint8).reshape(-1).cpu().numpy() for i in range(n_t)]

        def gpu_segments():
            sentry.sentry_merkle_segments(t7_ptrs[:n_t], t7_lens[:n_t], LEAF7, 0, root7.data_ptr(), stream)
            torch.cuda.synchronize()
            return bytes(root7.cpu().numpy())

        cpu_leg("c3_first_%d_tensors" % n_t, acc_b, lambda: oracle.merkle_segments(segs, LEAF7)[1], gpu_segments)
        if not args.quick:
            c1_np = wl.uniform_bytes(wl.SEED_C1, 0, 16 << 20)
            c1_d = torch.from_numpy(c1_np).to(dev)
            cpu_leg("c1_full", c1_np.size, lambda: oracle.merkle_root(c1_np, 4096), lambda: gpu_root(c1_d.data_ptr(), c1_np.size, 4096))
            img_np, ioff_np = wl.image_records(50_000)
            img_d = torch.from_numpy(img_np).to(dev)
            ioff_d = torch.from_numpy(ioff_np.view(np.int64).copy()).to(dev)
            cpu_leg("c2_full", img_np.size, lambda: oracle.lthash(img_np, ioff_np).tobytes(), lambda: gpu_lanes(img_d, ioff_d, 50_000))
        t_m, t_l = parts["c5_prefix"]["s"], parts["c4_prefix"]["s"]
        # context, not baselines: the same oracle on every host core at once (leaves and records are
        # independent: one slice per thread, the C oracle runs outside the interpreter lock), and the
        # host's hashing library on one core (the paper's CPU baseline is that library)
        import hashlib
        from concurrent.futures import ThreadPoolExecutor
        n_thr = max(1, min(os.cpu_count() or 1, 16))
        cut = [(m_bytes // LEAF70) * k // n_thr * LEAF70 for k in range(n_thr + 1)]
        rcut = [nb * k // n_thr for k in range(n_thr + 1)]

        def slice_job(k):
            oracle.merkle_root(sample_m[cut[k]:cut[k + 1]], LEAF70)
            o = sample_off[rcut[k]:rcut[k + 1] + 1]
            oracle.lthash(sample_l[int(o[0]):int(o[-1])], o - o[0])

        t = time.perf_counter()
        with ThreadPoolExecutor(n_thr) as pool:
            list(pool.map(slice_job, range(n_thr)))
        t_all = time.perf_counter() - t
        t = time.perf_counter()
        hashlib.sha256(sample_m[:1 << 29]).digest()
        t_hs = time.perf_counter() - t
        t = time.perf_counter()
        hashlib.blake2b(sample_l[:1 << 29]).digest()
        t_hb = time.perf_counter() - t
        context = {"oracle_all_cores_GB/s": (m_bytes + lt_b) / t_all / 1e9, "threads": n_thr,
                   "hashlib_sha256_1_core_GB/s": min(m_bytes, 1 << 29) / t_hs / 1e9,
                   "hashlib_blake2b_1_core_GB/s": min(lt_b, 1 << 29) / t_hb / 1e9}
        all_b, all_s = sum(v["bytes"] for v in parts.values()), sum(v["s"] for v in parts.values())
        cpu = {"value": all_b / all_s / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "configs 1 and 2 in full; Merkle over the first %d bytes of the 70B stream (64 KiB leaves); "
                         "per-tensor roots and model root of the first %d tensors (%d bytes) of the 7B checkpoint; lattice "
                         "hash of the first %d records (%d bytes) of the batch; %.0f s of oracle time in all, bounded so "
                         "that the default run ends within minutes; GPU results on every sample match"
                         % (m_bytes, n_t, acc_b, nb, lt_b, all_s),
               "merkle_GB/s": m_bytes / t_m / 1e9, "lthash_GB/s": lt_b / t_l / 1e9, "parts": parts,
               "host_cpus": os.cpu_count(), "context": context}

    out = {
        "metric": "GB/s hashed on 1 MI355X (Merkle and lattice hash); fraction of ALU/HBM roofline",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": ("QUICK (1/64-size smoke inputs): " if args.quick else "") +
                   ("PREFIX RUN (first %d GiB of the 70B stream only): " % args.merkle_prefix_gib
                    if args.merkle_prefix_gib else "") +
                   "Merkle root of the 70B bf16 checkpoint stream resident in HBM (config 5 shape, 64 KiB leaves) + "
                   "per-tensor roots and model root of the 7B checkpoint (config 3, 1 MiB leaves) + lattice hash of "
                   "one 8 GB batch of log-normal records folded into the running sum (config 4 shape)",
                   "bytes_per_step": step_bytes, "records_per_step": n_rec,
                   "schedule": {"serial": "one stream, parts back to back",
                                "pair": "70B root, then the 7B per-tensor pass and the batch hash side by side on two streams",
                                "overlap": "70B root on one stream; beside it, on a second stream, the 7B per-tensor pass, "
                                           "then the batch hash"}[args.schedule],
                   "step_parts_ms": {"merkle_70b_in_step": ms70_in_step, "merkle_7b_in_step": ms7_in_step,
                                     "lthash_batch_in_step": mslt_in_step, "all_on_gpu": ms_gpu_step}},
        "roofline": roofline, "cpu_baseline": cpu, "per_config": per_config, "streaming": streaming,
        "root_70b": expected.hex(),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()

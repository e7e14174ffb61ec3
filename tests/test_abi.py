"""The C-ABI library loads without a GPU, exports every entry point the header declares,
and rejects bad arguments on the host before any GPU work (no compute calls here)."""
import ctypes
import os
import re

import pytest

import paper_2510_00554_amd as sentry
from paper_2510_00554_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sentry.h")).read()
    return sorted(set(re.findall(r"SENTRY_API[^;(]*?\b(sentry_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    lib = ctypes.CDLL(sentry.lib_path())
    names = declared_symbols()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.PROTOTYPES) == names
    for n in names:
        assert callable(getattr(sentry, n)), n


def test_verify_is_host_only():
    a = bytes(range(32))
    assert sentry.sentry_verify(a, a) == 0
    b = bytearray(a)
    b[31] ^= 0x80
    assert sentry.sentry_verify(a, bytes(b)) == 1
    with pytest.raises(sentry.SentryError) as e:
        sentry.sentry_verify(None, a)
    assert e.value.code == binding.ERR_INVALID_ARG and "NULL" in str(e.value)


@pytest.mark.parametrize("call", [
    lambda: sentry.sentry_merkle_root(0x1000, 4096, 0, 0x2000),          # leaf_bytes == 0
    lambda: sentry.sentry_merkle_root(0x1000, 4096, 100, 0x2000),        # not a multiple of 64
    lambda: sentry.sentry_merkle_root(0x1004, 4096, 64, 0x2000),         # misaligned buffer
    lambda: sentry.sentry_merkle_root(0, 4096, 64, 0x2000),              # NULL with len > 0
    lambda: sentry.sentry_merkle_root(0x1000, 4096, 64, 0),              # NULL output
    lambda: sentry.sentry_merkle_root_noalloc(0x1000, 64 * ((1 << 22) + 1), 64, 0x2000),   # beyond the fixed scratch
    lambda: sentry.sentry_merkle_root_noalloc(0x1000, 4096, 96, 0x2000),  # bad leaf size
    lambda: sentry.sentry_merkle_root_h(1, 0x1000, 4096, 100, 0x2000),   # BLAKE2b tree, bad leaf size
    lambda: sentry.sentry_merkle_root_h(2, 0x1008, 4096, 64, 0x2000),    # SHA-3 tree, misaligned buffer
    lambda: sentry.sentry_merkle_root_h(9, 0x1000, 4096, 64, 0x2000),    # unknown leaf function
    lambda: sentry.sentry_merkle_leaves(0x1000, 4096, 64, 0x2008),       # misaligned output
    lambda: sentry.sentry_merkle_reduce(0x1000, 0, 0x2000),              # n == 0
    lambda: sentry.sentry_merkle_reduce(0x1008, 4, 0x2000),              # misaligned nodes
    lambda: sentry.sentry_merkle_segments([], [], 64, 0, 0x2000),        # no segments
    lambda: sentry.sentry_merkle_segments([0x1000, 0x3008], [64, 64], 64, 0, 0x2000),
    lambda: sentry.sentry_merkle_segments([0x1000], [64], 96, 0, 0x2000),
    lambda: sentry.sentry_merkle_inplace([], [], 64, 0x2000),            # no segments
    lambda: sentry.sentry_merkle_inplace([0x1000, 0x3008], [64, 64], 64, 0x2000),
    lambda: sentry.sentry_merkle_inplace([0x1000], [64], 64, 0),         # NULL output
    lambda: sentry.sentry_merkle_segments_h(1, [], [], 64, 0, 0x2000),   # BLAKE2b, no segments
    lambda: sentry.sentry_merkle_segments_h(2, [0x1000, 0x3008], [64, 64], 64, 0, 0x2000),
    lambda: sentry.sentry_merkle_segments_h(5, [0x1000], [64], 64, 0, 0x2000),        # unknown leaf function
    lambda: sentry.sentry_merkle_inplace_h(1, [0x1000], [64], 100, 0x2000),           # bad leaf size
    lambda: sentry.sentry_merkle_inplace_h(2, [0], [64], 64, 0x2000),                 # NULL tensor with bytes
    lambda: sentry.sentry_merkle_inplace_h(2, [0x1000], [64], 64, 0),                 # NULL output
    lambda: sentry.sentry_merkle_root_h2d(0x1000, 4096, 64, 100, 0x2000),  # chunk not a leaf multiple
    lambda: sentry.sentry_lthash(0x1000, 0, 5, 0x2000),                  # NULL offsets with n > 0
    lambda: sentry.sentry_lthash(0x1000, 0x3004, 5, 0x2000),             # misaligned offsets
    lambda: sentry.sentry_lthash(0x1000, 0x3000, 5, 0),                  # NULL lanes
    lambda: sentry.sentry_lthash_digests(0x1000, 0x3000, 5, 0x2004),     # misaligned digest rows
    lambda: sentry.sentry_lthash_digests(0x1000, 0, 5, 0x2000),          # NULL offsets
    lambda: sentry.sentry_lthash_sum(0, 5, 0x2000),                      # NULL digests with n > 0
    lambda: sentry.sentry_lthash_sum(0x1008, 5, 0x2000),                 # misaligned digests
    lambda: sentry.sentry_lthash_sum(0x1000, 5, 0),                      # NULL lanes
    lambda: sentry.sentry_lthash_sources(0x1000, 0x3000, 0x4000, 5, 0, 0x2000),       # no sources
    lambda: sentry.sentry_lthash_sources(0x1000, 0x3000, 0x4000, 5, 5000, 0x2000),    # too many sources
    lambda: sentry.sentry_lthash_sources(0x1000, 0x3000, 0x4002, 5, 4, 0x2000),       # misaligned ids
    lambda: sentry.sentry_lthash_sources(0x1000, 0x3000, 0, 5, 4, 0x2000),            # NULL ids
    lambda: sentry.sentry_lthash_model([], [], 8192, 0, 0x2000),                      # no tensors
    lambda: sentry.sentry_lthash_model([0x1000], [64], 100, 0, 0x2000),               # block not a multiple of 16
    lambda: sentry.sentry_lthash_model([0x1008], [64], 8192, 0, 0x2000),              # misaligned tensor
    lambda: sentry.sentry_lthash_model([0x1000], [64], 8192, 0, 0),                   # NULL output
    lambda: sentry.sentry_merkle_coalesced([0x1000], [64], 100, 0, 0, 0x2000),         # leaf_bytes not a multiple of 64
    lambda: sentry.sentry_merkle_coalesced([], [], 64, 0, 0, 0x2000),                  # no tensors
    lambda: sentry.sentry_merkle_coalesced([0], [64], 64, 0, 0, 0x2000),               # NULL tensor with bytes
    lambda: sentry.sentry_merkle_coalesced([0x1000], [64], 64, 0, 0, 0),               # NULL output
    lambda: sentry.sentry_merkle_coalesced([0x1000], [65], 64, 0x4000, 64, 0x2000),    # buffer too small for the padding
    lambda: sentry.sentry_merkle_coalesced([0x1000], [64], 64, 0x4004, 64, 0x2000),    # misaligned buffer
    lambda: sentry.sentry_merkle_coalesced([0x1000], [64], 64, 0x1020, 64, 0x2000),    # buffer inside the tensor
    lambda: sentry.sentry_merkle_coalesced_h(7, [0x1000], [64], 64, 0, 0, 0x2000),     # unknown hash
    lambda: sentry.sentry_lthash_combine(0, 0x2000),
    lambda: sentry.sentry_lthash_remove(0x2001, 0x2000),
    lambda: sentry.sentry_lthash32(0x1000, 0x3000, 5, 0),                # NULL output
    lambda: sentry.sentry_lthash32(0x1000, 0x3000, 5, 0x2001),           # misaligned output
    lambda: sentry.sentry_lthash32(0x1000, 0x3004, 5, 0x2000),           # misaligned offsets
    lambda: sentry.sentry_lthash32(0x1000, 0, 5, 0x2000),                # NULL offsets with n > 0
    lambda: sentry.sentry_lthash32(0x1000, 0x3000, 1 << 30, 0x2000),     # too many records
    lambda: sentry.sentry_reserve_scratch(1000, 100, 0),                              # leaf size not a multiple of 64
    lambda: sentry.sentry_reserve_scratch(0, 0, 1 << 30),                             # too many records
    lambda: sentry.sentry_lthash_fixed(0, 100, 5, 0x2000),                            # NULL records with bytes to read
    lambda: sentry.sentry_lthash_fixed(0x1000, 100, 5, 0x2001),                       # misaligned output
    lambda: sentry.sentry_lthash32_fixed(0x1000, 1 << 62, 8, 0x2000),                 # n * record_bytes overflows
    lambda: sentry.sentry_lthash32_fixed(0x1000, 1, 1 << 30, 0x2000),                 # too many records
    lambda: sentry.sentry_lthash32_sources(0x1000, 0x3000, 0x4000, 5, 0, 0x2000),     # no sources
    lambda: sentry.sentry_lthash32_sources(0x1000, 0x3000, 0x4000, 5, 4097, 0x2000),  # too many sources
    lambda: sentry.sentry_lthash32_sources(0x1000, 0x3000, 0x4002, 5, 4, 0x2000),     # misaligned ids
    lambda: sentry.sentry_lthash32_sources(0x1000, 0x3000, 0, 5, 4, 0x2000),          # NULL ids
    lambda: sentry.sentry_lthash32_sources(0x1000, 0x3000, 0x4000, 5, 4, 0),          # NULL sums
    lambda: sentry.sentry_lthash32_combine(0x2000, 0),
    lambda: sentry.sentry_lthash32_remove(0x2000, 0x2003),
    lambda: sentry.sentry_lthash_h2d(0x1000, 0x3000, 5, 0, 0x2000),      # batch_bytes == 0
    lambda: binding._check(binding.load().sentry_scratch_bytes(None, None, None)),    # nowhere to write to
])
def test_bad_arguments_are_rejected_on_the_host(call):
    with pytest.raises(sentry.SentryError) as e:
        call()
    assert e.value.code == binding.ERR_INVALID_ARG
    assert sentry.sentry_last_error() != ""


def test_stream_state_checks():
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_stream_begin(1000, 65)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_stream_update(None, 0x1000, 64)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_stream_update_h2d(None, 0x1000, 64)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_lthash_stream_update_h2d(None, 0x1000, 0x2000, 4)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_lthash_stream_final(None, 0x1000)


def test_header_is_plain_c_and_a_c_program_can_use_the_library(tmp_path):
    import subprocess
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "abi_smoke.c")
    exe = str(tmp_path / "abi_smoke")
    libdir = os.path.dirname(binding.lib_path())
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    src, "-o", exe, "-L", libdir, "-l:libsentry_hip.so", "-Wl,-rpath," + libdir],
                   check=True, capture_output=True, text=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "abi smoke ok" in r.stdout, r.stdout + r.stderr


def test_coalesced_plan_against_a_block_by_block_model():
    """Host logic of the coalesced scheme without a buffer (no GPU work): which blocks are put
    together in scratch.  Model, block by block: a block of the zero-padded concatenation is
    gathered when it holds bytes of more than one tensor, when it is the padded last block, or when
    its first byte is not 16-byte aligned where it lies."""
    import random
    rng = random.Random(11)
    for trial in range(300):
        leaf = rng.choice([64, 128, 1024])
        n = rng.randrange(1, 12)
        aligned = trial % 3 != 0
        lens, ptrs, at = [], [], 0x10000
        for _ in range(n):
            ln = rng.choice([0, 1, 16, leaf, leaf - 16, 3 * leaf, rng.randrange(0, 5 * leaf), 16 * rng.randrange(0, 300)])
            ptr = at if aligned else at + rng.randrange(0, 16)
            lens.append(ln)
            ptrs.append(ptr if ln else 0)
            at += (ln + 0x1000) // 0x1000 * 0x1000 + 0x1000
        total = sum(lens)
        # owner[i] = (tensor, offset in it) of byte i of the concatenation
        gathered = copied = runs = 0
        kinds = []
        starts = [sum(lens[:t]) for t in range(n)]
        for b0 in range(0, total, leaf):
            b1 = b0 + leaf
            owners = [t for t in range(n) if lens[t] and starts[t] < b1 and starts[t] + lens[t] > b0]
            where = None
            if len(owners) == 1 and b1 <= total:
                t = owners[0]
                addr = ptrs[t] + (b0 - starts[t])
                if addr % 16 == 0:
                    where = ("tensor", addr)
            if where is None:
                where = ("scratch", gathered)
                gathered += leaf
                copied += min(b1, total) - b0
            kinds.append(where)
        for k, (kind, addr) in enumerate(kinds):
            if k == 0 or kinds[k - 1][0] != kind or kinds[k - 1][1] + leaf != addr:
                runs += 1
        assert sentry.sentry_merkle_coalesced_plan(ptrs, lens, leaf) == (gathered, copied, runs), (trial, leaf, lens, ptrs)
    # aligned tensors whose lengths are multiples of the block size: nothing is gathered
    assert sentry.sentry_merkle_coalesced_plan([0x1000, 0x9000], [4096, 8192], 1024) == (0, 0, 2)
    # tensors that touch in memory are one run
    assert sentry.sentry_merkle_coalesced_plan([0x1000, 0x2000], [4096, 8192], 1024) == (0, 0, 1)
    with pytest.raises(sentry.SentryError):
        sentry.sentry_merkle_coalesced_plan([0x1000], [64], 100)

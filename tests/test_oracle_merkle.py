"""Pins for the oracle's Merkle tree: special cases that reduce to hashlib, hand
trees, a brute-force tree written over hashlib, and the path-update property
(section 2.2 "Merkle Tree": a changed block only changes its path to the root)."""
import hashlib
import random

import numpy as np
import pytest

import oracle


def H(b):
    return hashlib.sha256(b).digest()


def brute_root(buf, L):
    """Level-by-level tree over hashlib; odd node promoted unchanged."""
    n = max(1, -(-len(buf) // L))
    level = [H(buf[i * L:(i + 1) * L]) for i in range(n)]
    while len(level) > 1:
        nxt = [H(level[i] + level[i + 1]) for i in range(0, len(level) - 1, 2)]
        if len(level) % 2:
            nxt.append(level[-1])
        level = nxt
    return level[0]


def test_single_leaf_is_plain_sha256():
    rng = random.Random(3)
    for n in (0, 1, 63, 64, 65, 4095, 4096):
        buf = rng.randbytes(n)
        assert oracle.merkle_root(buf, 4096) == H(buf)


def test_empty_buffer_is_hash_of_empty_string():
    assert oracle.merkle_root(b"", 64).hex() == \
        "e3b0c44298fc1c149afbf4c8996fb92427ae41e4649b934ca495991b7852b855"


def test_hand_trees():
    rng = random.Random(4)
    L = 64
    buf = rng.randbytes(5 * L)
    h = [H(buf[i * L:(i + 1) * L]) for i in range(5)]
    assert oracle.merkle_root(buf[:2 * L], L) == H(h[0] + h[1])
    assert oracle.merkle_root(buf[:3 * L], L) == H(H(h[0] + h[1]) + h[2])
    assert oracle.merkle_root(buf[:4 * L], L) == H(H(h[0] + h[1]) + H(h[2] + h[3]))
    assert oracle.merkle_root(buf, L) == H(H(H(h[0] + h[1]) + H(h[2] + h[3])) + h[4])
    # order of the two children matters
    assert oracle.merkle_root(buf[:2 * L], L) != H(h[1] + h[0])


@pytest.mark.parametrize("L", [64, 128, 192])
def test_brute_force_1_to_33_leaves_with_short_tails(L):
    rng = random.Random(5)
    for n in range(1, 34):
        for tail in (0, 1, 55, 56, 63):
            size = (n - 1) * L + (tail if tail else L)
            buf = rng.randbytes(size)
            assert oracle.merkle_root(buf, L) == brute_root(buf, L), (n, tail)


def test_leaves_and_reduce_compose_to_root():
    rng = random.Random(6)
    buf = rng.randbytes(64 * 37 + 5)
    leaves = oracle.merkle_leaves(buf, 64)
    assert leaves.shape == (38, 32)
    assert bytes(leaves[37]) == H(buf[64 * 37:])
    assert oracle.merkle_reduce(leaves) == brute_root(buf, 64)


def test_byte_flip_changes_only_its_path():
    rng = np.random.default_rng(7)
    L, n = 256, 16
    buf = rng.integers(0, 256, L * n, dtype=np.uint8)
    root = oracle.merkle_root(buf, L)
    flipped = buf.copy()
    flipped[5 * L + 17] ^= 0x40                       # leaf 5
    assert oracle.merkle_root(flipped, L) != root
    # subtrees that do not contain leaf 5 are unchanged: leaves 8..15, 0..3, 6..7, 4
    for lo, hi in ((8, 16), (0, 4), (6, 8), (4, 5)):
        assert oracle.merkle_root(flipped[lo * L:hi * L], L) == oracle.merkle_root(buf[lo * L:hi * L], L)
    for lo, hi in ((0, 8), (4, 8), (4, 6), (5, 6)):
        assert oracle.merkle_root(flipped[lo * L:hi * L], L) != oracle.merkle_root(buf[lo * L:hi * L], L)
    # the root is the hash of the two half-tree roots
    assert root == H(oracle.merkle_root(buf[:8 * L], L) + oracle.merkle_root(buf[8 * L:], L))


def test_segments_match_brute_force():
    # Algorithm 2: per-tensor roots, then a reduction over them as ready-made nodes
    rng = random.Random(8)
    L = 128
    sizes = [L * 5, 17, L * 2 + 1, L, 0, L * 8]
    segs = [rng.randbytes(s) for s in sizes]
    roots, top = oracle.merkle_segments(segs, L)
    assert roots == [brute_root(s, L) for s in segs]
    level = list(roots)
    while len(level) > 1:
        nxt = [H(level[i] + level[i + 1]) for i in range(0, len(level) - 1, 2)]
        if len(level) % 2:
            nxt.append(level[-1])
        level = nxt
    assert top == level[0]
    # one segment: the global root is that segment's root, not a hash of it
    r1, t1 = oracle.merkle_segments([segs[0]], L)
    assert t1 == r1[0] == oracle.merkle_root(segs[0], L)


def test_verify():
    a = bytes(range(32))
    assert oracle.verify(a, a) == 0
    for i in (0, 13, 31):
        b = bytearray(a)
        b[i] ^= 1
        assert oracle.verify(a, bytes(b)) == 1


def test_inplace_flat_tree_over_fragmented_tensors():
    # Algorithm 3: one tree over the blocks of all tensors, short last blocks kept short
    rng = random.Random(9)
    L = 128
    # every tensor a multiple of the block size: same as hashing the concatenation (Algorithm 1)
    segs = [rng.randbytes(L * k) for k in (3, 1, 7, 2)]
    assert oracle.merkle_inplace(segs, L) == brute_root(b"".join(segs), L)
    # ragged tensors: leaves are the per-tensor blocks, in order, short tails included
    sizes = [L * 5 + 1, 17, L * 2, 0, L - 1, L * 3 + 64]
    segs = [rng.randbytes(s) for s in sizes]
    level = []
    for s in segs:
        level += [H(s[i:i + L]) for i in range(0, len(s), L)]
    assert len(level) == 6 + 1 + 2 + 0 + 1 + 4
    while len(level) > 1:
        nxt = [H(level[i] + level[i + 1]) for i in range(0, len(level) - 1, 2)]
        if len(level) % 2:
            nxt.append(level[-1])
        level = nxt
    assert oracle.merkle_inplace(segs, L) == level[0]
    assert oracle.merkle_inplace(segs, L) != oracle.merkle_segments(segs, L)[1]   # not the per-tensor scheme
    # one tensor: the plain root; nothing at all: the empty leaf
    assert oracle.merkle_inplace([segs[0]], L) == oracle.merkle_root(segs[0], L)
    assert oracle.merkle_inplace([b"", b""], L) == H(b"")

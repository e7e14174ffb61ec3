"""Pins for the oracle's SHA3-256 and for Merkle trees over BLAKE2b-512 and SHA3-256
(section 4.2.1 lists SHA256, BLAKE2B and SHA3 as leaf functions)."""
import hashlib
import random

import numpy as np
import pytest

import oracle
from conftest import golden_lines


def test_keccak_constants_match_fips202_definitions():
    rc, rho = oracle.keccak_constants()
    # anchors printed in FIPS 202 / the Keccak reference: first, second and last round constant
    assert int(rc[0]) == 0x0000000000000001 and int(rc[1]) == 0x0000000000008082
    assert int(rc[23]) == 0x8000000080008008
    # every constant has bits only at positions 2^j - 1
    allowed = sum(1 << ((1 << j) - 1) for j in range(7))
    assert all(int(c) & ~allowed == 0 for c in rc)
    rho = rho.reshape(5, 5)           # [y][x]
    assert rho[0][0] == 0 and rho[0][1] == 1 and rho[2][0] == 3 and rho[1][1] == 44 and rho[0][2] == 62
    assert sorted(int(v) for v in rho.reshape(-1)) == sorted([0] + [((t + 1) * (t + 2) // 2) % 64 for t in range(24)])


def test_sha3_fips202_examples():
    for ln in golden_lines("sha3_fips202.txt"):
        _, text, dig = ln.split(" ")
        assert oracle.sha3_256(text.encode()).hex() == dig


def test_sha3_against_hashlib():
    rng = random.Random(41)
    for n in list(range(0, 300)) + [135, 136, 137, 271, 272, 273, 4096, 8192, 65536, 100003]:
        msg = rng.randbytes(n)
        assert oracle.sha3_256(msg) == hashlib.sha3_256(msg).digest(), n


def brute(hfun, buf, L):
    n = max(1, -(-len(buf) // L))
    level = [hfun(buf[i * L:(i + 1) * L]) for i in range(n)]
    while len(level) > 1:
        nxt = [hfun(level[i] + level[i + 1]) for i in range(0, len(level) - 1, 2)]
        if len(level) % 2:
            nxt.append(level[-1])
        level = nxt
    return level[0]


@pytest.mark.parametrize("hid,hfun", [
    (oracle.HASH_SHA256, lambda b: hashlib.sha256(b).digest()),
    (oracle.HASH_BLAKE2B, lambda b: hashlib.blake2b(b).digest()),
    (oracle.HASH_SHA3_256, lambda b: hashlib.sha3_256(b).digest()),
])
def test_merkle_trees_over_each_leaf_function(hid, hfun):
    rng = random.Random(42 + hid)
    for L in (64, 192):
        for n in list(range(1, 20)) + [33]:
            for tail in (0, 1, 63):
                size = (n - 1) * L + (tail if tail else L)
                buf = rng.randbytes(size)
                assert oracle.merkle_root_h(hid, buf, L) == brute(hfun, buf, L), (hid, L, n, tail)
    assert oracle.merkle_root_h(hid, b"", 64) == hfun(b"")
    if hid == oracle.HASH_SHA256:
        buf = rng.randbytes(5000)
        assert oracle.merkle_root_h(hid, buf, 256) == oracle.merkle_root(buf, 256)


HASHES = [
    (oracle.HASH_SHA256, lambda b: hashlib.sha256(b).digest()),
    (oracle.HASH_BLAKE2B, lambda b: hashlib.blake2b(b).digest()),
    (oracle.HASH_SHA3_256, lambda b: hashlib.sha3_256(b).digest()),
]


def brute_nodes(hfun, level):
    while len(level) > 1:
        nxt = [hfun(level[i] + level[i + 1]) for i in range(0, len(level) - 1, 2)]
        if len(level) % 2:
            nxt.append(level[-1])
        level = nxt
    return level[0]


@pytest.mark.parametrize("hid,hfun", HASHES)
def test_per_tensor_and_flat_trees_over_each_leaf_function(hid, hfun):
    # Algorithm 2 (a tree per tensor, then a tree over the roots as ready-made nodes) and
    # Algorithm 3 (one flat tree over all blocks, short blocks kept short, empty tensors skipped)
    rng = random.Random(50 + hid)
    L = 128
    for sizes in ([1], [0], [L], [L + 1, 0, 3 * L, 5], [0, 0], [7 * L - 1, L, 2 * L + 9, 0, 64, 33 * L],
                  [rng.randrange(0, 6 * L) for _ in range(13)]):
        segs = [rng.randbytes(n) for n in sizes]
        roots, root = oracle.merkle_segments_h(hid, segs, L)
        want_roots = [brute(hfun, s, L) for s in segs]
        assert roots == want_roots, (hid, sizes)
        assert root == brute_nodes(hfun, list(want_roots)), (hid, sizes)
        leaves = [hfun(s[i:i + L]) for s in segs for i in range(0, len(s), L)]
        want_flat = brute_nodes(hfun, leaves) if leaves else hfun(b"")
        assert oracle.merkle_inplace_h(hid, segs, L) == want_flat, (hid, sizes)
        if hid == oracle.HASH_SHA256:
            assert (roots, root) == oracle.merkle_segments(segs, L)
            assert want_flat == oracle.merkle_inplace(segs, L)


@pytest.mark.parametrize("hid,hfun", HASHES)
def test_coalesced_tree_is_the_tree_over_the_zero_padded_concatenation(hid, hfun):
    # Algorithm 1: tensors copied one behind the other, the buffer a whole number of blocks long
    # (zero bytes behind the last tensor), one tree over it; rebuilt here with bytes.join, hashlib
    # and a Python list of nodes
    rng = random.Random(70 + hid)
    L = 128
    for sizes in ([1], [0], [], [L], [L - 1, 1], [L + 1, 0, 3 * L, 5], [0, 0], [3, 5, 7, 11, 13],
                  [7 * L - 1, L, 2 * L + 9, 0, 64, 33 * L], [rng.randrange(0, 6 * L) for _ in range(13)]):
        segs = [rng.randbytes(n) for n in sizes]
        cat = b"".join(segs)
        cat += bytes(-len(cat) % L)
        want = brute(hfun, cat, L)
        assert oracle.merkle_coalesced_h(hid, segs, L) == want, (hid, sizes)
        assert len(cat) % L == 0
    # blocks run across tensor boundaries: the same bytes cut differently give the same root ...
    buf = rng.randbytes(5 * L + 17)
    a = oracle.merkle_coalesced_h(hid, [buf[:100], buf[100:101], buf[101:]], L)
    b = oracle.merkle_coalesced_h(hid, [buf], L)
    assert a == b
    # ... which is not the in-place root of the same tensors (short last blocks, Algorithm 3),
    # and the padding is part of what is hashed: a buffer of whole blocks has none
    assert a != oracle.merkle_inplace_h(hid, [buf[:100], buf[100:101], buf[101:]], L)
    assert b != oracle.merkle_root_h(hid, buf, L)
    whole = rng.randbytes(4 * L)
    assert oracle.merkle_coalesced_h(hid, [whole[:L + 5], whole[L + 5:]], L) == oracle.merkle_root_h(hid, whole, L)
    # one short tensor: the hash of its bytes and the zeros up to the block size
    assert oracle.merkle_coalesced_h(hid, [b"abc"], L) == hfun(b"abc" + bytes(L - 3))
    assert oracle.merkle_coalesced_h(hid, [], L) == hfun(b"")

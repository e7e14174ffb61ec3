"""Pins for the oracle's BLAKE2b and BLAKE2Xb: the RFC 7693 example, the IV's
definition, hashlib on many lengths and on every parameter-block field hashlib
accepts, and hashlib for the BLAKE2Xb root hash.

PARITY UNPINNED: the values of the expansion-node parameter block (fanout 0,
depth 0, leaf length 64, inner length 64).  hashlib rejects depth 0 and no
BLAKE2Xb known-answer vector exists in this environment; what is pinned is the
function "BLAKE2b under an arbitrary parameter block" and the wiring of the
expansion (message = H0, node offset = block index, last block shortened)."""
import hashlib
import math
import random
import struct

import numpy as np
import pytest

import oracle
from conftest import golden_lines


def param_block(digest=64, key=0, fanout=1, depth=1, leaf=0, node_offset=0, node_depth=0,
                inner=0, salt=b"", person=b""):
    # RFC 7693 section 2.5 / BLAKE2 specification, table of the parameter block
    return (struct.pack("<BBBBIQBB", digest, key, fanout, depth, leaf, node_offset, node_depth, inner)
            + bytes(14) + salt.ljust(16, b"\0") + person.ljust(16, b"\0"))


def test_iv_is_fractional_sqrt_of_primes():
    # RFC 7693 section 2.6: the IV is that of SHA-512, the first 64 fractional bits
    # of the square roots of the first eight primes
    iv, sigma = oracle.blake2b_constants()
    primes = [2, 3, 5, 7, 11, 13, 17, 19]
    assert [int(x) for x in iv] == [math.isqrt(p << 128) & (2 ** 64 - 1) for p in primes]
    for row in sigma:
        assert sorted(int(x) for x in row) == list(range(16))
    assert [int(x) for x in sigma[0]] == list(range(16))


def test_rfc7693_abc():
    for ln in golden_lines("blake2b_rfc7693.txt"):
        _, text, dig = ln.split(" ")
        assert oracle.blake2b_param(param_block(), text.encode()).hex() == dig


def test_against_hashlib_lengths():
    rng = random.Random(11)
    for n in list(range(0, 301)) + [383, 384, 385, 3072, 8000, 1 << 16]:
        msg = rng.randbytes(n)
        assert oracle.blake2b_param(param_block(), msg) == hashlib.blake2b(msg).digest(), n


def test_counter_passes_32_bits():
    # 2^32 + 5 bytes: the byte counter t needs more than 32 bits
    msg = np.zeros((1 << 32) + 5, np.uint8)
    assert oracle.blake2b_param(param_block(), msg) == hashlib.blake2b(msg).digest()


@pytest.mark.parametrize("kw", [
    dict(digest_size=32), dict(digest_size=1), dict(digest_size=63),
    dict(fanout=0), dict(fanout=255), dict(depth=2), dict(depth=255),
    dict(leaf_size=64), dict(leaf_size=0xDEADBEEF),
    dict(node_offset=1), dict(node_offset=31), dict(node_offset=2048 << 32),
    dict(node_offset=(2048 << 32) | 17), dict(node_offset=2 ** 64 - 1),
    dict(node_depth=1), dict(node_depth=255), dict(inner_size=64), dict(inner_size=1),
    dict(salt=b"0123456789abcdef"), dict(person=b"fedcba9876543210"),
    dict(digest_size=48, fanout=0, depth=3, leaf_size=64, node_offset=(2048 << 32) | 5,
         node_depth=2, inner_size=64, salt=b"s" * 16, person=b"p" * 16),
])
def test_parameter_block_fields_against_hashlib(kw):
    rng = random.Random(12)
    p = param_block(digest=kw.get("digest_size", 64), fanout=kw.get("fanout", 1),
                    depth=kw.get("depth", 1), leaf=kw.get("leaf_size", 0),
                    node_offset=kw.get("node_offset", 0), node_depth=kw.get("node_depth", 0),
                    inner=kw.get("inner_size", 0), salt=kw.get("salt", b""),
                    person=kw.get("person", b""))
    for n in (0, 64, 129, 1000):
        msg = rng.randbytes(n)
        want = hashlib.blake2b(msg, **kw).digest()
        assert oracle.blake2b_param(p, msg, out_len=len(want)) == want, (kw, n)


def test_blake2xb_root_against_hashlib():
    # BLAKE2X: the root hash is a sequential BLAKE2b-512 whose parameter block holds the
    # XOF length in bytes 12..15, i.e. in the upper half of hashlib's 64-bit node_offset
    rng = random.Random(13)
    for xof in (2048, 100, 65535):
        for n in (0, 1, 64, 128, 3072, 5000):
            msg = rng.randbytes(n)
            want = hashlib.blake2b(msg, digest_size=64, node_offset=xof << 32).digest()
            assert oracle.blake2xb_root(msg, xof) == want, (xof, n)


def test_blake2xb_expansion_wiring():
    rng = random.Random(14)
    msg = rng.randbytes(777)
    for xof in (2048, 64, 65, 100, 128, 1000):
        h0 = oracle.blake2xb_root(msg, xof)
        out = oracle.blake2xb(msg, xof)
        assert len(out) == xof
        blocks = -(-xof // 64)
        for j in range(blocks):
            want_len = min(64, xof - 64 * j)
            # expansion node: fanout 0, depth 0, leaf length 64, node offset j, XOF length, inner 64
            p = struct.pack("<BBBBIIIBB", want_len, 0, 0, 0, 64, j, xof, 0, 64) + bytes(46)
            assert out[64 * j:64 * j + want_len] == oracle.blake2b_param(p, h0, out_len=want_len)
    # blocks differ from each other and from H0 (node offset really enters)
    out = oracle.blake2xb(msg, 2048)
    assert len({out[64 * j:64 * j + 64] for j in range(32)}) == 32
    assert oracle.blake2xb_root(msg, 2048) not in {out[64 * j:64 * j + 64] for j in range(32)}


def test_blake2xb_depends_on_requested_length():
    msg = b"sentry"
    assert oracle.blake2xb(msg, 128)[:64] != oracle.blake2xb(msg, 2048)[:64]

"""Pins for the oracle's SHA-256: the standard's constants and example digests,
and an independent library (hashlib / OpenSSL) on many lengths."""
import hashlib
import math
import random

import numpy as np

import oracle
from conftest import golden_lines


def _primes(n):
    out, c = [], 2
    while len(out) < n:
        if all(c % p for p in out if p * p <= c):
            out.append(c)
        c += 1
    return out


def _icbrt(v):
    x = int(round(v ** (1.0 / 3.0)))
    while x ** 3 > v:
        x -= 1
    while (x + 1) ** 3 <= v:
        x += 1
    return x


def test_constants_are_fractional_roots_of_primes():
    # FIPS 180-4 section 4.2.2 (K: cube roots of the first 64 primes) and
    # section 5.3.3 (H0: square roots of the first 8 primes), first 32 fractional bits
    k, h0 = oracle.sha256_constants()
    pr = _primes(64)
    assert [int(x) for x in k] == [_icbrt(p << 96) & 0xFFFFFFFF for p in pr]
    assert [int(x) for x in h0] == [math.isqrt(p << 64) & 0xFFFFFFFF for p in pr[:8]]
    # anchors as printed in the standard
    assert int(k[0]) == 0x428A2F98 and int(k[63]) == 0xC67178F2
    assert int(h0[0]) == 0x6A09E667 and int(h0[7]) == 0x5BE0CD19


def test_fips_180_4_examples():
    for ln in golden_lines("sha256_fips180_4.txt"):
        parts = ln.split(" ")
        if parts[0] == "ascii":
            msg, dig = parts[1].encode(), parts[2]
        else:
            msg, dig = parts[1].encode() * int(parts[2]), parts[3]
        assert oracle.sha256(msg).hex() == dig, (parts[0], len(msg))


def test_against_hashlib_all_short_lengths():
    rng = random.Random(1)
    for n in range(0, 301):
        msg = rng.randbytes(n)
        assert oracle.sha256(msg) == hashlib.sha256(msg).digest(), n


def test_against_hashlib_block_sizes():
    rng = np.random.default_rng(2)
    for n in (4096, 8192, 65536, 1 << 20, (1 << 20) + 55, (1 << 20) + 56, 1000003):
        msg = rng.integers(0, 256, n, dtype=np.uint8)
        assert oracle.sha256(msg) == hashlib.sha256(msg).digest(), n


def test_length_field_is_64_bit_big_endian():
    # 2^29 bytes = 2^32 bits: the bit length no longer fits 32 bits
    msg = np.zeros(1 << 29, np.uint8)
    assert oracle.sha256(msg) == hashlib.sha256(msg).digest()

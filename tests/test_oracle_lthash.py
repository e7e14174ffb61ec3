"""Pins for the oracle's lattice hash (section 2.2, Eq. (1); section 4.2.2): the
set-homomorphism identities the paper states, closed forms, the modulus, and a
brute-force sum in Python integers."""
import hashlib
import random

import numpy as np

import oracle


def pack(records):
    off = np.zeros(len(records) + 1, np.uint64)
    off[1:] = np.cumsum([len(r) for r in records])
    return b"".join(records), off


def lanes_via_xof(rec):
    return np.frombuffer(oracle.blake2xb(rec, 2048), dtype="<u2").astype(np.int64)


def test_empty_set_is_zero():
    assert not oracle.lthash(b"", np.zeros(1, np.uint64)).any()
    assert not oracle.lthash(b"", np.zeros(0, np.uint64)).any()


def test_single_record_is_its_xof_lanes():
    rec = random.Random(21).randbytes(3072)
    data, off = pack([rec])
    got = oracle.lthash(data, off)
    assert (got == lanes_via_xof(rec)).all()
    assert (oracle.lthash_one(rec) == got).all()
    # first lane = first two XOF bytes, little endian; the XOF's first block hangs off H0,
    # and H0 is pinned by hashlib
    x = oracle.blake2xb(rec, 2048)
    assert int(got[0]) == x[0] | (x[1] << 8)
    assert int(got[1023]) == x[2046] | (x[2047] << 8)
    assert oracle.blake2xb_root(rec, 2048) == hashlib.blake2b(rec, node_offset=2048 << 32).digest()


def test_brute_force_sum_small_sets():
    rng = random.Random(22)
    for n in (1, 2, 3, 16):
        recs = [rng.randbytes(rng.randrange(0, 400)) for _ in range(n)]
        data, off = pack(recs)
        want = sum(lanes_via_xof(r) for r in recs) % 65536
        assert (oracle.lthash(data, off).astype(np.int64) == want).all()


def test_union_of_disjoint_sets_is_sum():
    rng = random.Random(23)
    recs = [rng.randbytes(rng.randrange(1, 300)) for _ in range(40)]
    a, b = recs[:17], recs[17:]
    ha, hb, hab = (oracle.lthash(*pack(x)) for x in (a, b, recs))
    assert (oracle.lthash_combine(ha, hb) == hab).all()
    assert (oracle.lthash_remove(hab, ha) == hb).all()       # LtHash(S1 u S2) - LtHash(S1) = LtHash(S2)
    assert (oracle.lthash_remove(oracle.lthash_combine(ha, hb), hb) == ha).all()


def test_order_invariance_and_multiset():
    rng = random.Random(24)
    recs = [rng.randbytes(rng.randrange(0, 200)) for _ in range(30)]
    h = oracle.lthash(*pack(recs))
    shuffled = recs[:]
    rng.shuffle(shuffled)
    assert (oracle.lthash(*pack(shuffled)) == h).all()
    # a record present twice counts twice
    twice = oracle.lthash(*pack(recs + [recs[3]]))
    assert (twice == oracle.lthash_combine(h, oracle.lthash_one(recs[3]))).all()


def test_offsets_need_not_start_at_zero_and_empty_records_count():
    rng = random.Random(25)
    blob = rng.randbytes(1000)
    off = np.array([100, 100, 350, 900], np.uint64)          # first record is empty
    want = sum(lanes_via_xof(blob[int(off[i]):int(off[i + 1])]) for i in range(3)) % 65536
    assert (oracle.lthash(blob, off).astype(np.int64) == want).all()
    assert lanes_via_xof(b"").any()                          # h(empty record) is not zero


def test_modulus_is_2_to_16():
    rec = b"wraparound"
    one = oracle.lthash_one(rec)
    # 65,536 copies of one record sum to zero in every lane
    data, off = pack([rec] * 65536)
    assert not oracle.lthash(data, off).any()
    # per-lane carries are dropped, lanes do not leak into their neighbours
    a = np.full(1024, 0xFFFF, np.uint16)
    b = np.zeros(1024, np.uint16)
    b[::2] = 1
    s = oracle.lthash_combine(a, b)
    assert (s[::2] == 0).all() and (s[1::2] == 0xFFFF).all()
    d = oracle.lthash_remove(np.zeros(1024, np.uint16), b)
    assert (d[::2] == 0xFFFF).all() and (d[1::2] == 0).all()
    assert (oracle.lthash_combine(one, one).astype(np.int64) == (2 * one.astype(np.int64)) % 65536).all()


def test_per_source_sums_are_the_hashes_of_the_sub_multisets():
    # section 4.1.2 / 4.3: a shuffled batch holds samples of several providers; each provider's
    # running sum must equal the lattice hash of exactly its samples
    rng = random.Random(26)
    nprng = np.random.default_rng(26)
    recs = [rng.randbytes(rng.randrange(0, 300)) for _ in range(60)]
    src = nprng.integers(0, 5, 60).astype(np.uint32)
    src[7] = 9                                   # an id outside the table is left out
    data, off = pack(recs)
    acc = oracle.lthash_sources(data, off, src, 5)
    for s in range(5):
        mine = [r for r, k in zip(recs, src) if k == s]
        assert (acc[s] == oracle.lthash(*pack(mine))).all(), s
    # the sources partition the batch (minus the dropped record)
    total = np.zeros(1024, np.uint16)
    for s in range(5):
        total = oracle.lthash_combine(total, acc[s])
    kept = [r for r, k in zip(recs, src) if k < 5]
    assert (total == oracle.lthash(*pack(kept))).all()
    # running sums: a second batch adds on top, batch order does not matter
    acc2 = oracle.lthash_sources(data, off, src, 5, acc=acc)
    assert (acc2 == (2 * acc.astype(np.int64)) % 65536).all()
    # one source is the plain lattice hash
    one = oracle.lthash_sources(data, off, np.zeros(60, np.uint32), 1)
    assert (one[0] == oracle.lthash(data, off)).all()


def test_model_lattice_hash_against_hashlib():
    # section 4.2.2 / Algorithm 4 with the block index in front of every block: brute force
    # over hashlib.blake2b (digest 64 bytes = 32 partitions of 16 bits)
    import struct
    rng = random.Random(27)
    B = 256
    sizes = [B * 3, 17, B * 2 + 9, 0, B, B * 4 - 1]
    segs = [rng.randbytes(s) for s in sizes]
    layer, total = oracle.lthash_model(segs, B)
    k = 0
    want_total = np.zeros(32, np.int64)
    for t, s in enumerate(segs):
        want = np.zeros(32, np.int64)
        for start in range(0, len(s), B):
            dig = hashlib.blake2b(struct.pack("<Q", k) + s[start:start + B]).digest()
            want += np.frombuffer(dig, "<u2")
            k += 1
        assert (layer[t].astype(np.int64) == want % 65536).all(), t
        want_total += want
    assert (total.astype(np.int64) == want_total % 65536).all()
    assert k == 3 + 1 + 3 + 0 + 1 + 4
    # the index matters: swapping two equal-sized blocks of one tensor changes nothing in the
    # multiset of blocks, but changes the digest
    a = bytearray(segs[0])
    a[0:B], a[B:2 * B] = segs[0][B:2 * B], segs[0][0:B]
    assert (oracle.lthash_model([bytes(a)] + segs[1:], B)[1] != total).any()
    # the homomorphism still holds per block: the model digest is the sum of the layer digests
    acc = np.zeros(32, np.int64)
    for row in layer:
        acc += row
    assert (acc % 65536 == total).all()


def test_model_hash_of_slices_adds_up():
    rng = random.Random(28)
    B = 64
    segs = [rng.randbytes(B * 5 + 3), rng.randbytes(B * 2), rng.randbytes(7)]
    layer, total = oracle.lthash_model(segs, B)
    # second and third tensor on their own, starting at block 6, plus the first tensor cut in two
    l_a, t_a = oracle.lthash_model([segs[0][:B * 2]], B)
    l_b, t_b = oracle.lthash_model([segs[0][B * 2:]], B, first_index=2)
    l_c, t_c = oracle.lthash_model(segs[1:], B, first_index=6)
    assert (oracle.lanes_add(l_a[0], l_b[0]) == layer[0]).all() and (l_c == layer[1:]).all()
    assert (oracle.lanes_add(oracle.lanes_add(t_a, t_b), t_c) == total).all()


def test_digests_one_by_one_and_their_sum():
    # row i of the digest matrix is the XOF output of record i (H0 pinned by hashlib above), in
    # the order given; summing the rows is Eq. (1) again
    rng = random.Random(29)
    recs = [rng.randbytes(rng.randrange(0, 500)) for _ in range(37)] + [b"", b"same", b"same"]
    data, off = pack(recs)
    d = oracle.lthash_digests(data, off)
    assert d.shape == (40, 1024) and d.dtype == np.uint16
    for i, r in enumerate(recs):
        assert (d[i] == lanes_via_xof(r)).all(), i
    assert (d[38] == d[39]).all() and (d[37] != d[38]).any()
    assert (oracle.lthash_sum(d) == oracle.lthash(data, off)).all()
    assert oracle.lthash_digests(b"", np.zeros(1, np.uint64)).shape == (0, 1024)


def test_sum_of_given_digests_in_python_integers():
    rng = np.random.default_rng(30)
    for n in (0, 1, 2, 255, 1000):
        d = rng.integers(0, 65536, size=(n, 1024)).astype(np.uint16)
        want = [sum(int(x) for x in d[:, l]) % 65536 for l in range(1024)]
        assert oracle.lthash_sum(d).tolist() == want, n
    # carries stay inside their lane; 65,536 equal rows cancel; row order does not matter
    d = np.zeros((3, 1024), np.uint16)
    d[:, 0::2] = 0xFFFF
    s = oracle.lthash_sum(d)
    assert (s[0::2] == 0xFFFD).all() and (s[1::2] == 0).all()
    row = rng.integers(0, 65536, size=1024).astype(np.uint16)
    assert not oracle.lthash_sum(np.tile(row, (65536, 1))).any()
    d = rng.integers(0, 65536, size=(50, 1024)).astype(np.uint16)
    assert (oracle.lthash_sum(d) == oracle.lthash_sum(d[::-1].copy())).all()


# ---------------------------------------------------------------------------
# the dataset lattice hash at the paper's own digest width: one plain BLAKE2b-512 digest per
# sample = 32 partitions of 16 bits (section 4.2.2).  Pinned by hashlib all the way: no XOF.
# ---------------------------------------------------------------------------

def lanes32_via_hashlib(rec):
    return np.frombuffer(hashlib.blake2b(rec).digest(), dtype="<u2").astype(np.int64)


def test_lthash32_is_the_sum_of_hashlib_digests():
    rng = random.Random(31)
    assert not oracle.lthash32(b"", np.zeros(1, np.uint64)).any()       # the empty set
    assert not oracle.lthash32(b"", np.zeros(0, np.uint64)).any()
    for n in (1, 2, 3, 17, 200):
        recs = [rng.randbytes(rng.choice([0, 1, 127, 128, 129, 255, 256, 3072, rng.randrange(0, 700)])) for _ in range(n)]
        data, off = pack(recs)
        want = sum(lanes32_via_hashlib(r) for r in recs) % 65536
        got = oracle.lthash32(data, off)
        assert got.dtype == np.uint16 and got.shape == (32,)
        assert (got.astype(np.int64) == want).all(), n
    # one record: the 32 partitions are the digest's bytes, little endian, in order
    rec = rng.randbytes(3072)
    d = hashlib.blake2b(rec).digest()
    got = oracle.lthash32(*pack([rec]))
    assert int(got[0]) == d[0] | (d[1] << 8) and int(got[31]) == d[62] | (d[63] << 8)
    # the empty record counts: its digest is that of the empty message, not zero
    assert (oracle.lthash32(*pack([b""])).astype(np.int64) == lanes32_via_hashlib(b"")).all()


def test_lthash32_set_identities_and_modulus():
    rng = random.Random(32)
    recs = [rng.randbytes(rng.randrange(0, 500)) for _ in range(60)]
    a, b = recs[:23], recs[23:]
    ha, hb, hab = (oracle.lthash32(*pack(x)) for x in (a, b, recs))
    assert (oracle.lanes_add(ha, hb) == hab).all()                  # union of disjoint sets = sum
    assert (oracle.lanes_sub(hab, ha) == hb).all()                  # removal = subtraction
    shuffled = recs[:]
    rng.shuffle(shuffled)
    assert (oracle.lthash32(*pack(shuffled)) == hab).all()          # order does not matter
    twice = oracle.lthash32(*pack(recs + recs[:5]))                  # a multiset: duplicates count
    assert (twice == oracle.lanes_add(hab, oracle.lthash32(*pack(recs[:5])))).all()
    # offsets need not start at zero
    data, off = pack(recs)
    shifted = b"\xee" * 13 + data
    assert (oracle.lthash32(shifted, off + np.uint64(13)) == hab).all()
    # 65,536 copies of one record sum to zero in every partition; 65,537 to the record itself
    rec = rng.randbytes(40)
    many = np.arange(65537, dtype=np.uint64) * np.uint64(0)
    off1 = np.concatenate([many, np.array([40], np.uint64)])       # 65,536 empty records and then the record once
    base = oracle.lthash32(rec, off1)
    want = (65536 * lanes32_via_hashlib(b"") + lanes32_via_hashlib(rec)) % 65536
    assert (base.astype(np.int64) == want).all()


def test_lthash32_per_source_sums_against_hashlib():
    # every provider's row is the sum of hashlib's BLAKE2b-512 digests of exactly its samples,
    # partition by partition in Python integers; a second batch adds on top
    import hashlib
    rng = random.Random(36)
    nprng = np.random.default_rng(36)
    recs = [rng.randbytes(rng.randrange(0, 300)) for _ in range(70)]
    src = nprng.integers(0, 6, 70).astype(np.uint32)
    src[11] = 6                                  # an id outside the table is left out
    src[12] = 0xFFFFFFFF
    data, off = pack(recs)
    acc = oracle.lthash32_sources(data, off, src, 6)
    want = [[0] * 32 for _ in range(6)]
    for r, k in zip(recs, src):
        if k < 6:
            d = hashlib.blake2b(r).digest()
            for l in range(32):
                want[k][l] = (want[k][l] + d[2 * l] + 256 * d[2 * l + 1]) % 65536
    assert acc.tolist() == want
    acc2 = oracle.lthash32_sources(data, off, src, 6, acc=acc)
    assert (acc2 == (2 * acc.astype(np.int64)) % 65536).all()
    one = oracle.lthash32_sources(data, off, np.zeros(70, np.uint32), 1)
    assert (one[0] == oracle.lthash32(data, off)).all()
    # rows that wrap: 65,536 copies of one record in one source give zero, one fewer gives minus its digest
    rec = rng.randbytes(33)
    data, off = pack([rec] * 65536)
    src = np.ones(65536, np.uint32)
    acc = oracle.lthash32_sources(data, off, src, 2)
    assert not acc.any()
    acc = oracle.lthash32_sources(data, off[:-1], src[:-1], 2)
    assert (acc[1] == oracle.lanes_sub(np.zeros(32, np.uint16), oracle.lthash32(*pack([rec])))).all() and not acc[0].any()

"""Are the pins tight?  Each case below plants one plausible mistake in a copy of the oracle's C
source (a wrong rotation, a swapped operand, a dropped term, an off-by-one), builds it, and runs
the pins of the other test files against that build: at least one of them has to fail.  The
unedited source has to pass the same pins, so that a pin which always fails proves nothing here.
Everything runs on the CPU; the GPU library is not involved.

Not covered, because no pin exists for it (see the oracle's header): the parameter values of the
BLAKE2Xb expansion nodes."""
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle_blake2 as t_b2
import test_oracle_lthash as t_lt
import test_oracle_merkle as t_mk
import test_oracle_other_hashes as t_oh
import test_oracle_sha256 as t_sha

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "sentry_oracle.c")

# the pins, cheapest first; the parametrised ones with their parameters written out
PINS = [
    t_sha.test_constants_are_fractional_roots_of_primes, t_sha.test_fips_180_4_examples,
    t_sha.test_against_hashlib_all_short_lengths, t_sha.test_against_hashlib_block_sizes,
    t_mk.test_single_leaf_is_plain_sha256, t_mk.test_empty_buffer_is_hash_of_empty_string, t_mk.test_hand_trees,
    lambda: t_mk.test_brute_force_1_to_33_leaves_with_short_tails(64),
    lambda: t_mk.test_brute_force_1_to_33_leaves_with_short_tails(192),
    t_mk.test_leaves_and_reduce_compose_to_root, t_mk.test_byte_flip_changes_only_its_path,
    t_mk.test_segments_match_brute_force, t_mk.test_verify, t_mk.test_inplace_flat_tree_over_fragmented_tensors,
    t_b2.test_iv_is_fractional_sqrt_of_primes, t_b2.test_rfc7693_abc, t_b2.test_against_hashlib_lengths,
    t_b2.test_blake2xb_root_against_hashlib, t_b2.test_blake2xb_expansion_wiring,
    t_b2.test_blake2xb_depends_on_requested_length,
    t_lt.test_empty_set_is_zero, t_lt.test_single_record_is_its_xof_lanes, t_lt.test_brute_force_sum_small_sets,
    t_lt.test_union_of_disjoint_sets_is_sum, t_lt.test_order_invariance_and_multiset,
    t_lt.test_offsets_need_not_start_at_zero_and_empty_records_count,
    t_lt.test_per_source_sums_are_the_hashes_of_the_sub_multisets, t_lt.test_model_lattice_hash_against_hashlib,
    t_lt.test_model_hash_of_slices_adds_up, t_lt.test_digests_one_by_one_and_their_sum,
    t_lt.test_sum_of_given_digests_in_python_integers, t_lt.test_modulus_is_2_to_16,
    t_lt.test_lthash32_is_the_sum_of_hashlib_digests, t_lt.test_lthash32_set_identities_and_modulus,
    t_lt.test_lthash32_per_source_sums_against_hashlib,
    t_oh.test_keccak_constants_match_fips202_definitions, t_oh.test_sha3_fips202_examples, t_oh.test_sha3_against_hashlib,
] + [(lambda h=h, f=f: t_oh.test_merkle_trees_over_each_leaf_function(h, f)) for h, f in t_oh.HASHES] \
  + [(lambda h=h, f=f: t_oh.test_per_tensor_and_flat_trees_over_each_leaf_function(h, f)) for h, f in t_oh.HASHES] \
  + [(lambda h=h, f=f: t_oh.test_coalesced_tree_is_the_tree_over_the_zero_padded_concatenation(h, f)) for h, f in t_oh.HASHES]

# (what is planted, text in the source, replacement); every text occurs exactly once
MUTANTS = [
    ("SHA-256: a rotation of Sigma1 off by one", "rotr32(e, 6) ^ rotr32(e, 11)", "rotr32(e, 6) ^ rotr32(e, 12)"),
    ("SHA-256: a rotation of Sigma0 off by one", "rotr32(a, 13) ^ rotr32(a, 22)", "rotr32(a, 13) ^ rotr32(a, 21)"),
    ("SHA-256: shift instead of rotation in sigma0", "rotr32(W[t - 15], 18) ^ (W[t - 15] >> 3)", "rotr32(W[t - 15], 18) ^ rotr32(W[t - 15], 3)"),
    ("SHA-256: schedule takes W[t-6]", "W[t] = s1 + W[t - 7] + s0 + W[t - 16];", "W[t] = s1 + W[t - 6] + s0 + W[t - 16];"),
    ("SHA-256: Ch without the complement", "(e & f) ^ (~e & g)", "(e & f) ^ (e & g)"),
    ("SHA-256: Maj with a term dropped", "(a & b) ^ (a & c) ^ (b & c)", "(a & b) ^ (a & c)"),
    ("SHA-256: T2 left out of a", "a = T1 + T2;", "a = T1;"),
    ("SHA-256: length in bytes, not bits", "uint64_t bits = (uint64_t)len * 8u;", "uint64_t bits = (uint64_t)len;"),
    ("SHA-256: second padding block one byte late", "size_t tail_len = (rem < 56) ? 64 : 128;", "size_t tail_len = (rem < 57) ? 64 : 128;"),
    ("SHA-256: little-endian message words", "W[t] = ((uint32_t)block[4 * t] << 24) | ((uint32_t)block[4 * t + 1] << 16) |\n               ((uint32_t)block[4 * t + 2] << 8) | (uint32_t)block[4 * t + 3];",
     "W[t] = ((uint32_t)block[4 * t + 3] << 24) | ((uint32_t)block[4 * t + 2] << 16) |\n               ((uint32_t)block[4 * t + 1] << 8) | (uint32_t)block[4 * t];"),
    ("Merkle: the lone last node is hashed with itself instead of moving up", "if (n & 1) memmove(nodes + 32 * pairs, nodes + 32 * (n - 1), 32);",
     "if (n & 1) { uint8_t cat[64], dig[32]; memcpy(cat, nodes + 32 * (n - 1), 32); memcpy(cat + 32, nodes + 32 * (n - 1), 32); oracle_sha256(cat, 64, dig); memcpy(nodes + 32 * pairs, dig, 32); }"),
    ("Merkle: right child first", "memcpy(cat, nodes + 64 * i, 64);          /* node[2i] || node[2i+1] */",
     "memcpy(cat, nodes + 64 * i + 32, 32); memcpy(cat + 32, nodes + 64 * i, 32);"),
    ("Merkle: the last leaf reads a full leaf", "if (stop > len) stop = len;\n        oracle_sha256(buf + start, stop - start, digests + 32 * i);",
     "if (stop > len) stop = len;\n        oracle_sha256(buf + start, i + 1 == n && n > 1 ? stop - start - 1 : stop - start, digests + 32 * i);"),
    ("Merkle (per tensor): the roots are hashed again as leaves", "memcpy(nodes, seg_roots, 32 * n_seg);",
     "for (size_t t = 0; t < n_seg; t++) oracle_sha256(seg_roots + 32 * t, 32, nodes + 32 * t);"),
    ("Merkle (flat): an empty tensor contributes an empty leaf", "for (size_t t = 0; t < n_seg; t++) total += (lens[t] + leaf_bytes - 1) / leaf_bytes;\n    if (total == 0) { oracle_sha256(NULL, 0, out); return 0; }",
     "for (size_t t = 0; t < n_seg; t++) total += lens[t] ? (lens[t] + leaf_bytes - 1) / leaf_bytes : 1;\n    if (total == 0) { oracle_sha256(NULL, 0, out); return 0; }"),
    ("Merkle (coalesced): no padding behind the last tensor", "int rc = oracle_merkle_root_h(hash, buffer, padded, leaf_bytes, out);\n    free(buffer);",
     "int rc = oracle_merkle_root_h(hash, buffer, at, leaf_bytes, out);\n    free(buffer);"),
    ("Merkle (coalesced): the padding is not zero", "memset(buffer + at, 0, padded - at);", "memset(buffer + at, 0x80, padded - at);"),
    ("Merkle (coalesced): a whole extra block when the total is a multiple of the block size",
     "const size_t padded = (total + leaf_bytes - 1) / leaf_bytes * leaf_bytes;", "const size_t padded = (total / leaf_bytes + 1) * leaf_bytes;"),
    ("Merkle (coalesced): the tensors are laid down last to first", "for (size_t t = 0; t < n_seg; t++) {\n        if (lens[t]) memcpy(buffer + at, ptrs[t], lens[t]);",
     "for (size_t t = n_seg; t-- > 0;) {\n        if (lens[t]) memcpy(buffer + at, ptrs[t], lens[t]);"),
    ("lattice, 32 partitions per source: ids outside the table are counted for source 0",
     "if (src[i] >= n_sources) continue;\n        uint8_t dig[64];\n        oracle_blake2b_param(param, records + offsets[i], (size_t)(offsets[i + 1] - offsets[i]), dig, 64);\n        uint16_t *mine = acc + (size_t)src[i] * ORACLE_MODEL_LANES;",
     "uint8_t dig[64];\n        oracle_blake2b_param(param, records + offsets[i], (size_t)(offsets[i + 1] - offsets[i]), dig, 64);\n        uint16_t *mine = acc + (size_t)(src[i] >= n_sources ? 0 : src[i]) * ORACLE_MODEL_LANES;"),
    ("lattice, 32 partitions per source: rows saturate", "mine[l] = (uint16_t)((mine[l] + v) & 0xFFFFu);", "mine[l] = (uint16_t)(mine[l] + v > 0xFFFF ? 0xFFFF : mine[l] + v);"),
    ("lattice, 32 partitions per source: rows 16 partitions apart", "acc + (size_t)src[i] * ORACLE_MODEL_LANES;", "acc + (size_t)src[i] * 16;"),
    ("verify: the last byte is not looked at", "for (int i = 0; i < 32; i++) diff |= (unsigned)(a[i] ^ b[i]);", "for (int i = 0; i < 31; i++) diff |= (unsigned)(a[i] ^ b[i]);"),
    ("BLAKE2b: a rotation of G off by one", "v[b] = rotr64(v[b] ^ v[c], 24);", "v[b] = rotr64(v[b] ^ v[c], 25);"),
    ("BLAKE2b: G adds x twice", "v[a] = v[a] + v[b] + y;", "v[a] = v[a] + v[b] + x;"),
    ("BLAKE2b: a diagonal step on the wrong words", "blake2b_G(v, 1, 6, 11, 12, m[s[10]], m[s[11]]);", "blake2b_G(v, 1, 6, 11, 13, m[s[10]], m[s[11]]);"),
    ("BLAKE2b: eleven rounds", "for (int r = 0; r < 12; r++) {\n        const uint8_t *s = blake2b_sigma[r % 10];", "for (int r = 0; r < 11; r++) {\n        const uint8_t *s = blake2b_sigma[r % 10];"),
    ("BLAKE2b: counter counts blocks", "blake2b_compress(h, msg + done - 128, (uint64_t)done, 0);", "blake2b_compress(h, msg + done - 128, (uint64_t)(done / 128), 0);"),
    ("BLAKE2b: a message of whole blocks ends with an empty block", "while (len - done > 128) {", "while (len - done >= 128) {"),
    ("BLAKE2b: the finalisation flag inverts v[15]", "if (last) v[14] = ~v[14];", "if (last) v[15] = ~v[15];"),
    ("BLAKE2Xb root: XOF length in the wrong field", "p[12 + i] = (uint8_t)(xof_len >> (8 * i));", "p[20 + i] = (uint8_t)(xof_len >> (8 * i));"),
    ("lattice: big-endian lanes", "lanes[l] = (uint16_t)(x[2 * l] | ((uint16_t)x[2 * l + 1] << 8));", "lanes[l] = (uint16_t)(x[2 * l + 1] | ((uint16_t)x[2 * l] << 8));"),
    ("lattice: lanes saturate instead of wrapping", "            acc[l] = (uint16_t)((acc[l] + lanes[l]) & 0xFFFFu);\n    }\n}\n\n/* The digests of Eq. (1)",
     "            acc[l] = (uint16_t)((acc[l] + lanes[l]) > 0xFFFFu ? 0xFFFFu : (acc[l] + lanes[l]));\n    }\n}\n\n/* The digests of Eq. (1)"),
    ("lattice: the last record is left out", "    for (size_t i = 0; i < n; i++) {\n        uint16_t lanes[ORACLE_LANES];\n        oracle_lthash_one(records + offsets[i], (size_t)(offsets[i + 1] - offsets[i]), lanes);\n        for (int l = 0; l < ORACLE_LANES; l++)\n            acc[l]",
     "    for (size_t i = 0; i + 1 < n; i++) {\n        uint16_t lanes[ORACLE_LANES];\n        oracle_lthash_one(records + offsets[i], (size_t)(offsets[i + 1] - offsets[i]), lanes);\n        for (int l = 0; l < ORACLE_LANES; l++)\n            acc[l]"),
    ("lattice: remove adds", "    for (int l = 0; l < ORACLE_LANES; l++)\n        acc[l] = (uint16_t)((acc[l] + 0x10000u - x[l]) & 0xFFFFu);",
     "    for (int l = 0; l < ORACLE_LANES; l++)\n        acc[l] = (uint16_t)((acc[l] + x[l]) & 0xFFFFu);"),
    ("lattice: the sum of given digests skips row 0", "    for (size_t i = 0; i < n; i++)\n        for (int l = 0; l < ORACLE_LANES; l++)\n            acc[l] = (uint16_t)((acc[l] + digests[i * ORACLE_LANES + l]) & 0xFFFFu);",
     "    for (size_t i = 1; i < n; i++)\n        for (int l = 0; l < ORACLE_LANES; l++)\n            acc[l] = (uint16_t)((acc[l] + digests[i * ORACLE_LANES + l]) & 0xFFFFu);"),
    ("per source: records go to the next source", "uint16_t *row = acc + (size_t)src[i] * ORACLE_LANES;", "uint16_t *row = acc + (size_t)((src[i] + 1) % n_sources) * ORACLE_LANES;"),
    ("model lattice: the index restarts in every tensor", "        for (size_t start = 0; start < lens[t]; start += block_bytes, k++) {", "        k = first_index;\n        for (size_t start = 0; start < lens[t]; start += block_bytes, k++) {"),
    ("model lattice: big-endian index", "for (int i = 0; i < 8; i++) msg[i] = (uint8_t)(k >> (8 * i));", "for (int i = 0; i < 8; i++) msg[7 - i] = (uint8_t)(k >> (8 * i));"),
    ("32-partition lattice: big-endian partitions", "            uint16_t v = (uint16_t)(dig[2 * l] | ((uint16_t)dig[2 * l + 1] << 8));\n            acc[l] = (uint16_t)((acc[l] + v) & 0xFFFFu);",
     "            uint16_t v = (uint16_t)(dig[2 * l + 1] | ((uint16_t)dig[2 * l] << 8));\n            acc[l] = (uint16_t)((acc[l] + v) & 0xFFFFu);"),
    ("32-partition lattice: the XOF root's parameter block instead of the plain hash", "    param[0] = 64; param[2] = 1; param[3] = 1;\n    memset(acc, 0, ORACLE_MODEL_LANES * sizeof(uint16_t));",
     "    param[0] = 64; param[2] = 1; param[3] = 1; param[13] = 8;\n    memset(acc, 0, ORACLE_MODEL_LANES * sizeof(uint16_t));"),
    ("32-partition lattice: subtraction adds", "acc[l] = (uint16_t)((acc[l] + 0x10000u - x[l]) & 0xFFFFu);\n}\n\nvoid oracle_lthash_combine", "acc[l] = (uint16_t)((acc[l] + x[l]) & 0xFFFFu);\n}\n\nvoid oracle_lthash_combine"),
    ("SHA-3: SHAKE's domain byte", "last[len] ^= 0x06;", "last[len] ^= 0x1f;"),
    ("SHA-3: theta rotates by two", "D[x] = C[(x + 4) % 5] ^ rotl64(C[(x + 1) % 5], 1);", "D[x] = C[(x + 4) % 5] ^ rotl64(C[(x + 1) % 5], 2);"),
    ("SHA-3: chi without the complement", "B[x + 5 * y] ^ (~B[(x + 1) % 5 + 5 * y] & B[(x + 2) % 5 + 5 * y]);", "B[x + 5 * y] ^ (B[(x + 1) % 5 + 5 * y] & B[(x + 2) % 5 + 5 * y]);"),
    ("SHA-3: pi walks the other way", "B[y + 5 * ((2 * x + 3 * y) % 5)] = rotl64(A[x + 5 * y], keccak_rho[x][y]);", "B[y + 5 * ((3 * x + 2 * y) % 5)] = rotl64(A[x + 5 * y], keccak_rho[x][y]);"),
    ("SHA-3: the closing padding bit one byte early", "last[rate - 1] ^= 0x80;", "last[rate - 2] ^= 0x80;"),
    ("SHA-3: rate of SHA3-224", "const size_t rate = 136;\n    while (len >= rate) {", "const size_t rate = 128;\n    while (len >= rate) {"),
]


def build_variant(text, tmpdir, tag):
    c = os.path.join(tmpdir, "oracle_%s.c" % tag)
    so = os.path.join(tmpdir, "liboracle_%s.so" % tag)
    with open(c, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-std=gnu99", "-O1", "-fPIC", "-shared", "-o", so, c], check=True)
    return so


def first_failing_pin(path):
    """Index of the first pin that fails against the library at `path`, or None."""
    with oracle.use_library(path):
        for k, pin in enumerate(PINS):
            try:
                pin()
            except AssertionError:
                return k
    return None


def test_unedited_source_passes_every_pin():
    with tempfile.TemporaryDirectory() as d:
        so = build_variant(open(SRC).read(), d, "plain")
        assert first_failing_pin(so) is None


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(what, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, "the text to edit must occur exactly once: %r" % old
    with tempfile.TemporaryDirectory() as d:
        so = build_variant(src.replace(old, new), d, "edited")
        assert first_failing_pin(so) is not None, "no pin notices: " + what
    # and the real oracle is back
    assert oracle.sha256(b"abc").hex().startswith("ba7816bf")

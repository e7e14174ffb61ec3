/*
 * CPU oracle for Sentry's artifact hashing: TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded C99 statement of what the GPU library must
 * compute, written from the definitions and checked against published vectors
 * and independent libraries by the CPU tests.  Nothing in the product path may
 * call, link or import this file; it shares no code, table or helper with the
 * HIP sources.
 *
 * What follows which passage of the paper (Sentry, CCS '25):
 *   - Merkle tree over fixed-size blocks, neighbouring nodes hashed pairwise
 *     level by level up to one root:   section 2.2 "Merkle Tree", section 4.2.1.
 *   - a short last block is hashed at its true length, the buffer is never
 *     padded or modified:              section 4.2.1 "In-place Hashing".
 *   - per-tensor digests, then one reduction over the list of per-tensor
 *     digests:                         Algorithm 2 (per-layer hashing).
 *   - one flat tree over the blocks of all fragmented tensors: Algorithm 3.
 *   - all tensors copied into one buffer padded to whole blocks, one tree over it: Algorithm 1.
 *   - lattice hash = component-wise sum of per-item digests mod 2^d, d = 16:
 *                                      section 2.2 Eq. (1), section 4.2.2.
 *   - one digest per dataset sample, running sum over batches: section 4.3.
 *   - batches that mix data sources, one running sum per source: section 4.1.2, 4.3.
 *   - lattice hash of a model, block index mixed into each block digest: section 4.2.2,
 *     Algorithm 4.
 *   - Merkle trees with BLAKE2b and SHA-3 as the leaf function: section 4.2.1 (which names
 *     the three hash functions).
 *   - the dataset lattice hash at the paper's own digest width, one 64-byte BLAKE2b digest per
 *     sample = 32 partitions of 16 bits: section 4.2.2 (oracle_lthash32).
 *
 * Readings fixed where the paper leaves the point open (the build's target
 * configurations fix them):
 *   - the node function is the full padded SHA-256 (FIPS 180-4), an inner node
 *     is SHA-256(left || right) over the 64-byte concatenation;
 *   - a level with an odd number of nodes promotes its last node unchanged;
 *   - len == 0 is one empty leaf, so the root is SHA-256 of the empty string;
 *   - the per-sample digest h(M) is BLAKE2Xb(M) with 2048 output bytes, read as
 *     1024 little-endian uint16 lanes (the paper's own h is one 64-byte BLAKE2b
 *     digest = 32 lanes; the target configurations ask for 1024 lanes);
 *   - no index is mixed into a dataset sample's digest;
 *   - the padding behind the last tensor in Algorithm 1's buffer is zero bytes.
 *
 * Pins (tests/test_oracle_*.py): FIPS 180-4 vectors, RFC 7693 vector, hashlib
 * on random inputs and on every parameter block hashlib accepts, brute-force
 * trees over hashlib, the lattice invariants.  PARITY UNPINNED: the parameter
 * values of the BLAKE2Xb expansion nodes (fanout 0, depth 0, leaf length 64,
 * inner length 64) follow the BLAKE2X specification as read; no known-answer
 * vector for BLAKE2Xb exists in this environment and hashlib refuses depth 0.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* SHA-256, FIPS 180-4                                                      */
/* ------------------------------------------------------------------------ */

static uint32_t sha256_K[64];   /* frac(cbrt(prime_i)) * 2^32, i < 64 */
static uint32_t sha256_H0[8];   /* frac(sqrt(prime_i)) * 2^32, i < 8  */
static int sha256_tables_ready = 0;

/* floor(root_k(v)) for k = 2 or 3 by bisection; v < 2^106 */
static uint64_t int_root(unsigned __int128 v, int k)
{
    uint64_t lo = 0, hi = (uint64_t)1 << 36;   /* root < 2^36 for our inputs */
    while (lo + 1 < hi) {
        uint64_t mid = lo + (hi - lo) / 2;
        unsigned __int128 p = (unsigned __int128)mid * mid;
        if (k == 3) p *= mid;
        if (p <= v) lo = mid; else hi = mid;
    }
    return lo;
}

static void sha256_make_tables(void)
{
    int count = 0;
    for (uint32_t c = 2; count < 64; c++) {
        int is_prime = 1;
        for (uint32_t d = 2; d * d <= c; d++)
            if (c % d == 0) { is_prime = 0; break; }
        if (!is_prime) continue;
        /* first 32 fractional bits of the cube root: floor(cbrt(c * 2^96)) mod 2^32 */
        sha256_K[count] = (uint32_t)int_root((unsigned __int128)c << 96, 3);
        if (count < 8)  /* same for the square root: floor(sqrt(c * 2^64)) mod 2^32 */
            sha256_H0[count] = (uint32_t)int_root((unsigned __int128)c << 64, 2);
        count++;
    }
    sha256_tables_ready = 1;
}

void oracle_sha256_constants(uint32_t k_out[64], uint32_t h0_out[8])
{
    if (!sha256_tables_ready) sha256_make_tables();
    memcpy(k_out, sha256_K, sizeof sha256_K);
    memcpy(h0_out, sha256_H0, sizeof sha256_H0);
}

static uint32_t rotr32(uint32_t x, int n) { return (x >> n) | (x << (32 - n)); }

/* one application of the compression function to a 64-byte block */
static void sha256_block(uint32_t H[8], const uint8_t block[64])
{
    uint32_t W[64];
    for (int t = 0; t < 16; t++)
        W[t] = ((uint32_t)block[4 * t] << 24) | ((uint32_t)block[4 * t + 1] << 16) |
               ((uint32_t)block[4 * t + 2] << 8) | (uint32_t)block[4 * t + 3];
    for (int t = 16; t < 64; t++) {
        uint32_t s0 = rotr32(W[t - 15], 7) ^ rotr32(W[t - 15], 18) ^ (W[t - 15] >> 3);
        uint32_t s1 = rotr32(W[t - 2], 17) ^ rotr32(W[t - 2], 19) ^ (W[t - 2] >> 10);
        W[t] = s1 + W[t - 7] + s0 + W[t - 16];
    }
    uint32_t a = H[0], b = H[1], c = H[2], d = H[3];
    uint32_t e = H[4], f = H[5], g = H[6], h = H[7];
    for (int t = 0; t < 64; t++) {
        uint32_t S1 = rotr32(e, 6) ^ rotr32(e, 11) ^ rotr32(e, 25);
        uint32_t ch = (e & f) ^ (~e & g);
        uint32_t T1 = h + S1 + ch + sha256_K[t] + W[t];
        uint32_t S0 = rotr32(a, 2) ^ rotr32(a, 13) ^ rotr32(a, 22);
        uint32_t maj = (a & b) ^ (a & c) ^ (b & c);
        uint32_t T2 = S0 + maj;
        h = g; g = f; f = e; e = d + T1;
        d = c; c = b; b = a; a = T1 + T2;
    }
    H[0] += a; H[1] += b; H[2] += c; H[3] += d;
    H[4] += e; H[5] += f; H[6] += g; H[7] += h;
}

void oracle_sha256(const uint8_t *msg, size_t len, uint8_t out[32])
{
    if (!sha256_tables_ready) sha256_make_tables();
    uint32_t H[8];
    memcpy(H, sha256_H0, sizeof H);
    size_t full = len / 64;
    for (size_t i = 0; i < full; i++) sha256_block(H, msg + 64 * i);
    /* padding: 0x80, zeros, 64-bit big-endian bit length */
    uint8_t tail[128];
    size_t rem = len - 64 * full;
    memset(tail, 0, sizeof tail);
    if (rem) memcpy(tail, msg + 64 * full, rem);
    tail[rem] = 0x80;
    size_t tail_len = (rem < 56) ? 64 : 128;
    uint64_t bits = (uint64_t)len * 8u;
    for (int i = 0; i < 8; i++) tail[tail_len - 1 - i] = (uint8_t)(bits >> (8 * i));
    sha256_block(H, tail);
    if (tail_len == 128) sha256_block(H, tail + 64);
    for (int i = 0; i < 8; i++) {
        out[4 * i] = (uint8_t)(H[i] >> 24); out[4 * i + 1] = (uint8_t)(H[i] >> 16);
        out[4 * i + 2] = (uint8_t)(H[i] >> 8); out[4 * i + 3] = (uint8_t)H[i];
    }
}

/* ------------------------------------------------------------------------ */
/* Merkle tree (section 2.2, section 4.2.1, Algorithms 1 and 2)             */
/* ------------------------------------------------------------------------ */

/* Reduce n ready-made 32-byte nodes to one, in place: neighbours are hashed
 * pairwise, a lone last node moves up unchanged.  n >= 1. */
void oracle_merkle_reduce(uint8_t *nodes, size_t n, uint8_t out[32])
{
    while (n > 1) {
        size_t pairs = n / 2;
        for (size_t i = 0; i < pairs; i++) {
            uint8_t cat[64], dig[32];
            memcpy(cat, nodes + 64 * i, 64);          /* node[2i] || node[2i+1] */
            oracle_sha256(cat, 64, dig);
            memcpy(nodes + 32 * i, dig, 32);
        }
        if (n & 1) memmove(nodes + 32 * pairs, nodes + 32 * (n - 1), 32);
        n = pairs + (n & 1);
    }
    memcpy(out, nodes, 32);
}

/* Leaf digests of one buffer: leaf i = bytes [i*L, min((i+1)*L, len)).
 * Writes max(1, ceil(len/L)) digests; returns that count. */
size_t oracle_merkle_leaves(const uint8_t *buf, size_t len, size_t leaf_bytes, uint8_t *digests)
{
    size_t n = (len + leaf_bytes - 1) / leaf_bytes;
    if (n == 0) n = 1;
    for (size_t i = 0; i < n; i++) {
        size_t start = i * leaf_bytes;
        size_t stop = start + leaf_bytes;
        if (stop > len) stop = len;
        oracle_sha256(buf + start, stop - start, digests + 32 * i);
    }
    return n;
}

int oracle_merkle_root(const uint8_t *buf, size_t len, size_t leaf_bytes, uint8_t out[32])
{
    if (leaf_bytes == 0) return -1;
    size_t n = (len + leaf_bytes - 1) / leaf_bytes;
    if (n == 0) n = 1;
    uint8_t *nodes = (uint8_t *)malloc(32 * n);
    if (!nodes) return -3;
    oracle_merkle_leaves(buf, len, leaf_bytes, nodes);
    oracle_merkle_reduce(nodes, n, out);
    free(nodes);
    return 0;
}

/* Algorithm 2: a tree per tensor, then one reduction over the per-tensor roots
 * taken as ready-made nodes (they are not hashed again as leaves). */
int oracle_merkle_segments(const uint8_t *const *ptrs, const size_t *lens, size_t n_seg,
                           size_t leaf_bytes, uint8_t *seg_roots /* n_seg*32 */, uint8_t out[32])
{
    if (n_seg == 0 || leaf_bytes == 0) return -1;
    for (size_t t = 0; t < n_seg; t++) {
        int rc = oracle_merkle_root(ptrs[t], lens[t], leaf_bytes, seg_roots + 32 * t);
        if (rc) return rc;
    }
    uint8_t *nodes = (uint8_t *)malloc(32 * n_seg);
    if (!nodes) return -3;
    memcpy(nodes, seg_roots, 32 * n_seg);
    oracle_merkle_reduce(nodes, n_seg, out);
    free(nodes);
    return 0;
}

/* Algorithm 3 (in-place hashing): the blocks of all tensors, in tensor order, are the
 * leaves of ONE tree; the last block of a tensor is short rather than padded or filled
 * from the next tensor (section 4.2.1, "In-place Hashing").  A tensor of length 0 has no
 * block; if no tensor has one, the tree is the single empty leaf. */
int oracle_merkle_inplace(const uint8_t *const *ptrs, const size_t *lens, size_t n_seg,
                          size_t leaf_bytes, uint8_t out[32])
{
    if (leaf_bytes == 0) return -1;
    size_t total = 0;
    for (size_t t = 0; t < n_seg; t++) total += (lens[t] + leaf_bytes - 1) / leaf_bytes;
    if (total == 0) { oracle_sha256(NULL, 0, out); return 0; }
    uint8_t *nodes = (uint8_t *)malloc(32 * total);
    if (!nodes) return -3;
    size_t k = 0;
    for (size_t t = 0; t < n_seg; t++)
        if (lens[t]) k += oracle_merkle_leaves(ptrs[t], lens[t], leaf_bytes, nodes + 32 * k);
    oracle_merkle_reduce(nodes, total, out);
    free(nodes);
    return 0;
}

/* 0 = equal, 1 = different; every byte is looked at */
int oracle_verify(const uint8_t a[32], const uint8_t b[32])
{
    unsigned diff = 0;
    for (int i = 0; i < 32; i++) diff |= (unsigned)(a[i] ^ b[i]);
    return diff ? 1 : 0;
}

/* ------------------------------------------------------------------------ */
/* BLAKE2b (RFC 7693) with an explicit 64-byte parameter block, unkeyed     */
/* ------------------------------------------------------------------------ */

static const uint64_t blake2b_IV[8] = {   /* frac(sqrt(prime_i)) * 2^64, pinned by a test */
    0x6a09e667f3bcc908ULL, 0xbb67ae8584caa73bULL, 0x3c6ef372fe94f82bULL, 0xa54ff53a5f1d36f1ULL,
    0x510e527fade682d1ULL, 0x9b05688c2b3e6c1fULL, 0x1f83d9abfb41bd6bULL, 0x5be0cd19137e2179ULL
};

static const uint8_t blake2b_sigma[10][16] = {
    { 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15 },
    { 14, 10, 4, 8, 9, 15, 13, 6, 1, 12, 0, 2, 11, 7, 5, 3 },
    { 11, 8, 12, 0, 5, 2, 15, 13, 10, 14, 3, 6, 7, 1, 9, 4 },
    { 7, 9, 3, 1, 13, 12, 11, 14, 2, 6, 5, 10, 4, 0, 15, 8 },
    { 9, 0, 5, 7, 2, 4, 10, 15, 14, 1, 11, 12, 6, 8, 3, 13 },
    { 2, 12, 6, 10, 0, 11, 8, 3, 4, 13, 7, 5, 15, 14, 1, 9 },
    { 12, 5, 1, 15, 14, 13, 4, 10, 0, 7, 6, 3, 9, 2, 8, 11 },
    { 13, 11, 7, 14, 12, 1, 3, 9, 5, 0, 15, 4, 8, 6, 2, 10 },
    { 6, 15, 14, 9, 11, 3, 0, 8, 12, 2, 13, 7, 1, 4, 10, 5 },
    { 10, 2, 8, 4, 7, 6, 1, 5, 15, 11, 9, 14, 3, 12, 13, 0 }
};

void oracle_blake2b_constants(uint64_t iv_out[8], uint8_t sigma_out[160])
{
    memcpy(iv_out, blake2b_IV, sizeof blake2b_IV);
    memcpy(sigma_out, blake2b_sigma, 160);
}

static uint64_t rotr64(uint64_t x, int n) { return (x >> n) | (x << (64 - n)); }

static uint64_t load_le64(const uint8_t *p)
{
    uint64_t v = 0;
    for (int i = 7; i >= 0; i--) v = (v << 8) | p[i];
    return v;
}

static void blake2b_G(uint64_t v[16], int a, int b, int c, int d, uint64_t x, uint64_t y)
{
    v[a] = v[a] + v[b] + x; v[d] = rotr64(v[d] ^ v[a], 32);
    v[c] = v[c] + v[d];     v[b] = rotr64(v[b] ^ v[c], 24);
    v[a] = v[a] + v[b] + y; v[d] = rotr64(v[d] ^ v[a], 16);
    v[c] = v[c] + v[d];     v[b] = rotr64(v[b] ^ v[c], 63);
}

/* t = number of message bytes fed so far, this block included */
static void blake2b_compress(uint64_t h[8], const uint8_t block[128], uint64_t t, int last)
{
    uint64_t m[16], v[16];
    for (int i = 0; i < 16; i++) m[i] = load_le64(block + 8 * i);
    for (int i = 0; i < 8; i++) { v[i] = h[i]; v[i + 8] = blake2b_IV[i]; }
    v[12] ^= t;            /* low word of the 128-bit counter; the high word stays 0 */
    if (last) v[14] = ~v[14];
    for (int r = 0; r < 12; r++) {
        const uint8_t *s = blake2b_sigma[r % 10];
        blake2b_G(v, 0, 4, 8, 12, m[s[0]], m[s[1]]);
        blake2b_G(v, 1, 5, 9, 13, m[s[2]], m[s[3]]);
        blake2b_G(v, 2, 6, 10, 14, m[s[4]], m[s[5]]);
        blake2b_G(v, 3, 7, 11, 15, m[s[6]], m[s[7]]);
        blake2b_G(v, 0, 5, 10, 15, m[s[8]], m[s[9]]);
        blake2b_G(v, 1, 6, 11, 12, m[s[10]], m[s[11]]);
        blake2b_G(v, 2, 7, 8, 13, m[s[12]], m[s[13]]);
        blake2b_G(v, 3, 4, 9, 14, m[s[14]], m[s[15]]);
    }
    for (int i = 0; i < 8; i++) h[i] ^= v[i] ^ v[i + 8];
}

/* Unkeyed BLAKE2b of msg under the given parameter block; writes out_len
 * (<= 64) bytes, the first out_len bytes of the little-endian state. */
void oracle_blake2b_param(const uint8_t param[64], const uint8_t *msg, size_t len,
                          uint8_t *out, size_t out_len)
{
    uint64_t h[8];
    for (int i = 0; i < 8; i++) h[i] = blake2b_IV[i] ^ load_le64(param + 8 * i);
    /* every block but the last is a full one; the last holds 1..128 bytes
     * (0 only for the empty message) and is zero-padded */
    size_t done = 0;
    while (len - done > 128) {
        done += 128;
        blake2b_compress(h, msg + done - 128, (uint64_t)done, 0);
    }
    uint8_t last[128];
    memset(last, 0, sizeof last);
    if (len - done) memcpy(last, msg + done, len - done);
    blake2b_compress(h, last, (uint64_t)len, 1);
    uint8_t full[64];
    for (int i = 0; i < 8; i++)
        for (int j = 0; j < 8; j++) full[8 * i + j] = (uint8_t)(h[i] >> (8 * j));
    memcpy(out, full, out_len);
}

/* Parameter block layout used by BLAKE2Xb: byte 0 digest length, 1 key length,
 * 2 fanout, 3 depth, 4..7 leaf length (LE32), 8..11 node offset (LE32),
 * 12..15 XOF digest length (LE32), 16 node depth, 17 inner length, rest zero. */
static void blake2xb_param(uint8_t p[64], uint8_t digest_len, uint8_t fanout, uint8_t depth,
                           uint32_t leaf_len, uint32_t node_offset, uint32_t xof_len,
                           uint8_t inner_len)
{
    memset(p, 0, 64);
    p[0] = digest_len; p[1] = 0; p[2] = fanout; p[3] = depth;
    for (int i = 0; i < 4; i++) {
        p[4 + i] = (uint8_t)(leaf_len >> (8 * i));
        p[8 + i] = (uint8_t)(node_offset >> (8 * i));
        p[12 + i] = (uint8_t)(xof_len >> (8 * i));
    }
    p[16] = 0; p[17] = inner_len;
}

/* The root hash H0 of BLAKE2Xb: an ordinary sequential BLAKE2b-512 whose
 * parameter block also carries the requested XOF length. */
void oracle_blake2xb_root(const uint8_t *msg, size_t len, uint32_t xof_len, uint8_t h0[64])
{
    uint8_t p[64];
    blake2xb_param(p, 64, 1, 1, 0, 0, xof_len, 0);
    oracle_blake2b_param(p, msg, len, h0, 64);
}

/* BLAKE2Xb: out = B_0 || B_1 || ..., B_j = BLAKE2b(H0) under the expansion-node
 * parameters with node offset j; the last B_j is cut to the bytes still needed. */
void oracle_blake2xb(const uint8_t *msg, size_t len, uint8_t *out, uint32_t xof_len)
{
    uint8_t h0[64];
    oracle_blake2xb_root(msg, len, xof_len, h0);
    uint32_t produced = 0, j = 0;
    while (produced < xof_len) {
        uint32_t want = xof_len - produced;
        if (want > 64) want = 64;
        uint8_t p[64];
        blake2xb_param(p, (uint8_t)want, 0, 0, 64, j, xof_len, 64);
        oracle_blake2b_param(p, h0, 64, out + produced, want);
        produced += want; j++;
    }
}

/* ------------------------------------------------------------------------ */
/* SHA3-256 (FIPS 202) and Merkle trees over other leaf functions           */
/* ------------------------------------------------------------------------ */

static uint64_t keccak_RC[24];
static int keccak_rho[5][5];     /* rotation offset of lane (x, y) */
static int keccak_ready = 0;

/* Round constants from the degree-8 LFSR and rotation offsets from the (x, y) walk, both as
 * FIPS 202 section 3.2 defines them. */
static void keccak_make_tables(void)
{
    uint8_t R = 1;   /* LFSR state, x^8 + x^6 + x^5 + x^4 + 1 */
    for (int round = 0; round < 24; round++) {
        uint64_t rc = 0;
        for (int j = 0; j <= 6; j++) {
            if (R & 1) rc |= (uint64_t)1 << ((1 << j) - 1);
            uint8_t hi = R & 0x80;
            R = (uint8_t)(R << 1);
            if (hi) R ^= 0x71;
        }
        keccak_RC[round] = rc;
    }
    int x = 1, y = 0;
    keccak_rho[0][0] = 0;
    for (int t = 0; t < 24; t++) {
        keccak_rho[x][y] = ((t + 1) * (t + 2) / 2) % 64;
        int nx = y, ny = (2 * x + 3 * y) % 5;
        x = nx; y = ny;
    }
    keccak_ready = 1;
}

static uint64_t rotl64(uint64_t v, int n) { return n ? (v << n) | (v >> (64 - n)) : v; }

/* A[x][y] is lane x + 5y of the 1600-bit state */
static void keccak_f1600(uint64_t A[25])
{
    for (int round = 0; round < 24; round++) {
        uint64_t C[5], D[5], B[25];
        for (int x = 0; x < 5; x++) C[x] = A[x] ^ A[x + 5] ^ A[x + 10] ^ A[x + 15] ^ A[x + 20];
        for (int x = 0; x < 5; x++) D[x] = C[(x + 4) % 5] ^ rotl64(C[(x + 1) % 5], 1);
        for (int i = 0; i < 25; i++) A[i] ^= D[i % 5];                               /* theta */
        for (int x = 0; x < 5; x++)
            for (int y = 0; y < 5; y++)
                B[y + 5 * ((2 * x + 3 * y) % 5)] = rotl64(A[x + 5 * y], keccak_rho[x][y]);   /* rho, pi */
        for (int y = 0; y < 5; y++)
            for (int x = 0; x < 5; x++)
                A[x + 5 * y] = B[x + 5 * y] ^ (~B[(x + 1) % 5 + 5 * y] & B[(x + 2) % 5 + 5 * y]);   /* chi */
        A[0] ^= keccak_RC[round];                                                   /* iota */
    }
}

void oracle_keccak_constants(uint64_t rc_out[24], int32_t rho_out[25])
{
    if (!keccak_ready) keccak_make_tables();
    memcpy(rc_out, keccak_RC, sizeof keccak_RC);
    for (int x = 0; x < 5; x++)
        for (int y = 0; y < 5; y++) rho_out[x + 5 * y] = keccak_rho[x][y];
}

/* SHA3-256: rate 136 bytes, domain bits 01 then pad10*1 (first pad byte 0x06, last 0x80) */
void oracle_sha3_256(const uint8_t *msg, size_t len, uint8_t out[32])
{
    if (!keccak_ready) keccak_make_tables();
    uint64_t A[25];
    memset(A, 0, sizeof A);
    const size_t rate = 136;
    while (len >= rate) {
        for (size_t i = 0; i < rate / 8; i++) A[i] ^= load_le64(msg + 8 * i);
        keccak_f1600(A);
        msg += rate; len -= rate;
    }
    uint8_t last[136];
    memset(last, 0, sizeof last);
    if (len) memcpy(last, msg, len);
    last[len] ^= 0x06;
    last[rate - 1] ^= 0x80;
    for (size_t i = 0; i < rate / 8; i++) A[i] ^= load_le64(last + 8 * i);
    keccak_f1600(A);
    for (int i = 0; i < 4; i++)
        for (int j = 0; j < 8; j++) out[8 * i + j] = (uint8_t)(A[i] >> (8 * j));
}

/* The Merkle tree of section 4.2.1 over any of the paper's three leaf functions:
 * hash 0 = SHA-256 (32-byte nodes), 1 = BLAKE2b-512 (64-byte nodes), 2 = SHA3-256 (32-byte
 * nodes).  Same rules as oracle_merkle_root: node = H(left || right) with the full hash, a lone
 * last node moves up unchanged, short last leaf, len 0 = one empty leaf.  Returns the digest
 * length, or a negative error. */
static void hash_any(int hash, const uint8_t *msg, size_t len, uint8_t *out)
{
    if (hash == 0) {
        oracle_sha256(msg, len, out);
    } else if (hash == 1) {
        uint8_t param[64];
        memset(param, 0, sizeof param);
        param[0] = 64; param[2] = 1; param[3] = 1;
        oracle_blake2b_param(param, msg, len, out, 64);
    } else {
        oracle_sha3_256(msg, len, out);
    }
}

static size_t digest_len(int hash) { return hash == 1 ? 64 : 32; }

/* leaf digests of one buffer under hash h: max(1, ceil(len/L)) of them; returns the count */
static size_t leaves_h(int hash, const uint8_t *buf, size_t len, size_t leaf_bytes, uint8_t *digests)
{
    const size_t dl = digest_len(hash);
    size_t n = (len + leaf_bytes - 1) / leaf_bytes;
    if (n == 0) n = 1;
    for (size_t i = 0; i < n; i++) {
        size_t start = i * leaf_bytes, stop = start + leaf_bytes;
        if (stop > len) stop = len;
        hash_any(hash, buf + start, stop - start, digests + dl * i);
    }
    return n;
}

/* n >= 1 ready-made nodes to one, in place: neighbours hashed pairwise, a lone last node
 * moves up unchanged */
static void reduce_h(int hash, uint8_t *nodes, size_t n, uint8_t *out)
{
    const size_t dl = digest_len(hash);
    while (n > 1) {
        size_t pairs = n / 2;
        for (size_t i = 0; i < pairs; i++) {
            uint8_t cat[128], dig[64];
            memcpy(cat, nodes + 2 * dl * i, 2 * dl);
            hash_any(hash, cat, 2 * dl, dig);
            memcpy(nodes + dl * i, dig, dl);
        }
        if (n & 1) memmove(nodes + dl * pairs, nodes + dl * (n - 1), dl);
        n = pairs + (n & 1);
    }
    memcpy(out, nodes, dl);
}

int oracle_merkle_root_h(int hash, const uint8_t *buf, size_t len, size_t leaf_bytes, uint8_t *out)
{
    if (leaf_bytes == 0 || hash < 0 || hash > 2) return -1;
    const size_t dl = digest_len(hash);
    size_t n = (len + leaf_bytes - 1) / leaf_bytes;
    if (n == 0) n = 1;
    uint8_t *nodes = (uint8_t *)malloc(dl * n);
    if (!nodes) return -3;
    leaves_h(hash, buf, len, leaf_bytes, nodes);
    reduce_h(hash, nodes, n, out);
    free(nodes);
    return (int)dl;
}

/* Algorithm 2 under hash h: a tree per tensor, then the tree over the per-tensor roots taken as
 * ready-made nodes.  seg_roots: n_seg digests.  Returns the digest length. */
int oracle_merkle_segments_h(int hash, const uint8_t *const *ptrs, const size_t *lens, size_t n_seg,
                             size_t leaf_bytes, uint8_t *seg_roots, uint8_t *out)
{
    if (n_seg == 0 || leaf_bytes == 0 || hash < 0 || hash > 2) return -1;
    const size_t dl = digest_len(hash);
    for (size_t t = 0; t < n_seg; t++) {
        int rc = oracle_merkle_root_h(hash, ptrs[t], lens[t], leaf_bytes, seg_roots + dl * t);
        if (rc < 0) return rc;
    }
    uint8_t *nodes = (uint8_t *)malloc(dl * n_seg);
    if (!nodes) return -3;
    memcpy(nodes, seg_roots, dl * n_seg);
    reduce_h(hash, nodes, n_seg, out);
    free(nodes);
    return (int)dl;
}

/* Algorithm 3 under hash h: the blocks of all tensors, in tensor order, are the leaves of one
 * tree; a tensor of length 0 has no block; no block at all = the single empty leaf. */
int oracle_merkle_inplace_h(int hash, const uint8_t *const *ptrs, const size_t *lens, size_t n_seg,
                            size_t leaf_bytes, uint8_t *out)
{
    if (leaf_bytes == 0 || hash < 0 || hash > 2) return -1;
    const size_t dl = digest_len(hash);
    size_t total = 0;
    for (size_t t = 0; t < n_seg; t++) total += (lens[t] + leaf_bytes - 1) / leaf_bytes;
    if (total == 0) { hash_any(hash, NULL, 0, out); return (int)dl; }
    uint8_t *nodes = (uint8_t *)malloc(dl * total);
    if (!nodes) return -3;
    size_t k = 0;
    for (size_t t = 0; t < n_seg; t++)
        if (lens[t]) k += leaves_h(hash, ptrs[t], lens[t], leaf_bytes, nodes + dl * k);
    reduce_h(hash, nodes, total, out);
    free(nodes);
    return (int)dl;
}

/* Algorithm 1 (coalesced hashing) under hash h: the tensors are copied one behind the other
 * into one buffer; the buffer's size is the total rounded up to a whole number of blocks and
 * the bytes after the last tensor are filled (section 4.2.1, "Coalesced Hashing"; the fill value
 * is not given there: zero bytes here); then the Merkle tree over that buffer.  No byte at all
 * = the single empty leaf, as everywhere else. */
int oracle_merkle_coalesced_h(int hash, const uint8_t *const *ptrs, const size_t *lens, size_t n_seg,
                              size_t leaf_bytes, uint8_t *out)
{
    if (leaf_bytes == 0 || hash < 0 || hash > 2) return -1;
    size_t total = 0;
    for (size_t t = 0; t < n_seg; t++) total += lens[t];
    const size_t padded = (total + leaf_bytes - 1) / leaf_bytes * leaf_bytes;
    uint8_t *buffer = (uint8_t *)malloc(padded ? padded : 1);
    if (!buffer) return -3;
    size_t at = 0;
    for (size_t t = 0; t < n_seg; t++) {
        if (lens[t]) memcpy(buffer + at, ptrs[t], lens[t]);
        at += lens[t];
    }
    memset(buffer + at, 0, padded - at);
    int rc = oracle_merkle_root_h(hash, buffer, padded, leaf_bytes, out);
    free(buffer);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Lattice hash, 1024 lanes of 16 bits (section 2.2 Eq. (1), section 4.2.2) */
/* ------------------------------------------------------------------------ */

#define ORACLE_LANES 1024

/* lanes of one record: the 2048 XOF bytes read as little-endian uint16 */
void oracle_lthash_one(const uint8_t *rec, size_t len, uint16_t lanes[ORACLE_LANES])
{
    uint8_t x[2 * ORACLE_LANES];
    oracle_blake2xb(rec, len, x, 2 * ORACLE_LANES);
    for (int l = 0; l < ORACLE_LANES; l++)
        lanes[l] = (uint16_t)(x[2 * l] | ((uint16_t)x[2 * l + 1] << 8));
}

/* record i = bytes [offsets[i], offsets[i+1]) of records; acc = sum mod 2^16 */
void oracle_lthash(const uint8_t *records, const uint64_t *offsets, size_t n,
                   uint16_t acc[ORACLE_LANES])
{
    memset(acc, 0, ORACLE_LANES * sizeof(uint16_t));
    for (size_t i = 0; i < n; i++) {
        uint16_t lanes[ORACLE_LANES];
        oracle_lthash_one(records + offsets[i], (size_t)(offsets[i + 1] - offsets[i]), lanes);
        for (int l = 0; l < ORACLE_LANES; l++)
            acc[l] = (uint16_t)((acc[l] + lanes[l]) & 0xFFFFu);
    }
}

/* The digests of Eq. (1) one by one: row i of out = the 1024 lanes of record i. */
void oracle_lthash_digests(const uint8_t *records, const uint64_t *offsets, size_t n, uint16_t *out)
{
    for (size_t i = 0; i < n; i++)
        oracle_lthash_one(records + offsets[i], (size_t)(offsets[i + 1] - offsets[i]), out + i * ORACLE_LANES);
}

/* Eq. (1) over digests that are already there: acc[l] = sum over rows of digests[row][l] mod 2^16 */
void oracle_lthash_sum(const uint16_t *digests, size_t n, uint16_t acc[ORACLE_LANES])
{
    memset(acc, 0, ORACLE_LANES * sizeof(uint16_t));
    for (size_t i = 0; i < n; i++)
        for (int l = 0; l < ORACLE_LANES; l++)
            acc[l] = (uint16_t)((acc[l] + digests[i * ORACLE_LANES + l]) & 0xFFFFu);
}

/* Mixed-source batch (section 4.1.2, section 4.3): record i belongs to data source src[i];
 * every source keeps a running sum, acc[s] += sum of the digests of its records in this
 * batch.  acc holds n_sources rows of 1024 lanes and is updated in place.  Records whose
 * source id is not below n_sources are left out. */
void oracle_lthash_sources(const uint8_t *records, const uint64_t *offsets, const uint32_t *src,
                           size_t n, size_t n_sources, uint16_t *acc)
{
    for (size_t i = 0; i < n; i++) {
        if (src[i] >= n_sources) continue;
        uint16_t lanes[ORACLE_LANES];
        oracle_lthash_one(records + offsets[i], (size_t)(offsets[i + 1] - offsets[i]), lanes);
        uint16_t *row = acc + (size_t)src[i] * ORACLE_LANES;
        for (int l = 0; l < ORACLE_LANES; l++) row[l] = (uint16_t)((row[l] + lanes[l]) & 0xFFFFu);
    }
}

/* Model lattice hash (section 4.2.2, Algorithm 4).  The blocks of all tensors, in tensor
 * order, are numbered 0, 1, 2, ... across the model; block k of block_bytes bytes (the last
 * block of a tensor may be short) has the digest BLAKE2b-512(LE64(k) || block), read as 32
 * little-endian uint16 partitions (the 64-byte, 4 x 16 bits per 64-bit word layout of
 * section 4.2.2).  layer_lanes[t] = sum of the digests of tensor t's blocks, lanes = sum over
 * all blocks = sum of the layer digests, every partition mod 2^16.
 * Reading: the text says the block is concatenated with "the block index" against
 * reordering, Algorithm 4 prints the layer index; the block index is taken, since a layer
 * index would not tell two blocks of one layer apart.  Width, position and byte order of
 * the index (8 bytes, little endian, in front) are this build's choice. */
#define ORACLE_MODEL_LANES 32
/* first_index: the model-wide index of the first block of ptrs[0] (0 for a whole model; a
 * slice of a model can be hashed on its own and added to the other slices). */
void oracle_lthash_model_from(const uint8_t *const *ptrs, const size_t *lens, size_t n_seg, size_t block_bytes,
                              uint64_t first_index, uint16_t *layer_lanes /* n_seg * 32, may be NULL */,
                              uint16_t lanes[ORACLE_MODEL_LANES]);

void oracle_lthash_model(const uint8_t *const *ptrs, const size_t *lens, size_t n_seg, size_t block_bytes,
                         uint16_t *layer_lanes /* n_seg * 32, may be NULL */, uint16_t lanes[ORACLE_MODEL_LANES])
{
    oracle_lthash_model_from(ptrs, lens, n_seg, block_bytes, 0, layer_lanes, lanes);
}

/* acc[l] = (acc[l] + x[l]) mod 2^16 for n partitions */
void oracle_lanes_add(uint16_t *acc, const uint16_t *x, size_t n)
{
    for (size_t l = 0; l < n; l++) acc[l] = (uint16_t)((acc[l] + x[l]) & 0xFFFFu);
}

void oracle_lthash_model_from(const uint8_t *const *ptrs, const size_t *lens, size_t n_seg, size_t block_bytes,
                              uint64_t first_index, uint16_t *layer_lanes, uint16_t lanes[ORACLE_MODEL_LANES])
{
    uint8_t param[64];
    memset(param, 0, sizeof param);
    param[0] = 64; param[2] = 1; param[3] = 1;      /* plain BLAKE2b-512: digest 64, fanout 1, depth 1 */
    uint8_t *msg = (uint8_t *)malloc(block_bytes + 8);
    memset(lanes, 0, ORACLE_MODEL_LANES * sizeof(uint16_t));
    uint64_t k = first_index;
    for (size_t t = 0; t < n_seg; t++) {
        uint16_t layer[ORACLE_MODEL_LANES];
        memset(layer, 0, sizeof layer);
        for (size_t start = 0; start < lens[t]; start += block_bytes, k++) {
            size_t n = lens[t] - start < block_bytes ? lens[t] - start : block_bytes;
            for (int i = 0; i < 8; i++) msg[i] = (uint8_t)(k >> (8 * i));
            memcpy(msg + 8, ptrs[t] + start, n);
            uint8_t dig[64];
            oracle_blake2b_param(param, msg, n + 8, dig, 64);
            for (int l = 0; l < ORACLE_MODEL_LANES; l++) {
                uint16_t v = (uint16_t)(dig[2 * l] | ((uint16_t)dig[2 * l + 1] << 8));
                layer[l] = (uint16_t)((layer[l] + v) & 0xFFFFu);
            }
        }
        for (int l = 0; l < ORACLE_MODEL_LANES; l++) {
            if (layer_lanes) layer_lanes[t * ORACLE_MODEL_LANES + l] = layer[l];
            lanes[l] = (uint16_t)((lanes[l] + layer[l]) & 0xFFFFu);
        }
    }
    free(msg);
}

/* The dataset lattice hash at the paper's own digest width (section 4.2.2: a 64-byte BLAKE2b
 * digest per item, its 64-bit words split into four 16-bit partitions): h(M) = the plain,
 * unkeyed BLAKE2b-512 of the sample (digest 64, fanout 1, depth 1, nothing else set), read as
 * 32 little-endian uint16; acc[l] = sum over the records of h(record)[l] mod 2^16.  No index
 * is mixed in (samples are a multiset, section 4.1.2). */
void oracle_lthash32(const uint8_t *records, const uint64_t *offsets, size_t n, uint16_t acc[ORACLE_MODEL_LANES])
{
    uint8_t param[64];
    memset(param, 0, sizeof param);
    param[0] = 64; param[2] = 1; param[3] = 1;
    memset(acc, 0, ORACLE_MODEL_LANES * sizeof(uint16_t));
    for (size_t i = 0; i < n; i++) {
        uint8_t dig[64];
        oracle_blake2b_param(param, records + offsets[i], (size_t)(offsets[i + 1] - offsets[i]), dig, 64);
        for (int l = 0; l < ORACLE_MODEL_LANES; l++) {
            uint16_t v = (uint16_t)(dig[2 * l] | ((uint16_t)dig[2 * l + 1] << 8));
            acc[l] = (uint16_t)((acc[l] + v) & 0xFFFFu);
        }
    }
}

/* Mixed-source batch at the 32-partition width (section 4.1.2, section 4.3 with the digest of
 * section 4.2.2): acc holds n_sources rows of 32 partitions; the digest of record i is added to
 * row src[i]; records whose source id is not below n_sources are left out. */
void oracle_lthash32_sources(const uint8_t *records, const uint64_t *offsets, const uint32_t *src,
                             size_t n, size_t n_sources, uint16_t *acc)
{
    uint8_t param[64];
    memset(param, 0, sizeof param);
    param[0] = 64; param[2] = 1; param[3] = 1;
    for (size_t i = 0; i < n; i++) {
        if (src[i] >= n_sources) continue;
        uint8_t dig[64];
        oracle_blake2b_param(param, records + offsets[i], (size_t)(offsets[i + 1] - offsets[i]), dig, 64);
        uint16_t *mine = acc + (size_t)src[i] * ORACLE_MODEL_LANES;
        for (int l = 0; l < ORACLE_MODEL_LANES; l++) {
            uint16_t v = (uint16_t)(dig[2 * l] | ((uint16_t)dig[2 * l + 1] << 8));
            mine[l] = (uint16_t)((mine[l] + v) & 0xFFFFu);
        }
    }
}

/* acc[l] = (acc[l] - x[l]) mod 2^16 for n partitions */
void oracle_lanes_sub(uint16_t *acc, const uint16_t *x, size_t n)
{
    for (size_t l = 0; l < n; l++) acc[l] = (uint16_t)((acc[l] + 0x10000u - x[l]) & 0xFFFFu);
}

void oracle_lthash_combine(uint16_t acc[ORACLE_LANES], const uint16_t x[ORACLE_LANES])
{
    for (int l = 0; l < ORACLE_LANES; l++) acc[l] = (uint16_t)((acc[l] + x[l]) & 0xFFFFu);
}

void oracle_lthash_remove(uint16_t acc[ORACLE_LANES], const uint16_t x[ORACLE_LANES])
{
    for (int l = 0; l < ORACLE_LANES; l++)
        acc[l] = (uint16_t)((acc[l] + 0x10000u - x[l]) & 0xFFFFu);
}

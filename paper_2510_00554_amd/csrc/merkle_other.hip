// Merkle trees over the paper's other two leaf functions, BLAKE2b-512 and SHA3-256 (section
// 4.2.1: "supports SHA256, BLAKE2B, and SHA3 as compression functions for Merkle tree
// hashing").  Same tree rules as the SHA-256 path: one leaf per lane, node = H(left || right)
// with the full hash, a lone last node moves up unchanged, a short last leaf is hashed at its
// true length.  These kernels are the plain version of the scheme (leaf digests to memory,
// then 512 nodes folded per workgroup in LDS); the tuned path is the SHA-256 one.
#include "blake2b_device.h"
#include "sentry_internal.h"

namespace {

constexpr int OTHER_WG = 256;
constexpr int OTHER_WG_SMALL = 64;
constexpr int OTHER_RED_IN = 2 * OTHER_WG;

// data word w (8 bytes at offset 8w) of an n-byte message at p (8-byte aligned), zero beyond n
__device__ __forceinline__ uint64_t word_or_zero(const uint8_t *p, uint64_t n, uint64_t w)
{
    const uint64_t o = 8 * w;
    if (o + 8 <= n) return *reinterpret_cast<const uint64_t *>(p + o);
    uint64_t v = 0;
    for (uint32_t i = 0; i < 8; i++)
        if (o + i < n) v |= (uint64_t)p[o + i] << (8 * i);
    return v;
}

// ---------------------------------------------------------------------------
// BLAKE2b-512, default parameter block
// ---------------------------------------------------------------------------
struct Blake2bTree {
    static constexpr int WORDS = 16;   // 32-bit words per digest

    __device__ static void leaf(const uint8_t *p, uint64_t n, uint32_t (&out)[WORDS])
    {
        uint64_t h[8];
#pragma unroll
        for (int i = 0; i < 8; i++) h[i] = b2_iv(i);
        h[0] ^= 0x0000000001010040ull;
        const uint64_t ncomp = n ? (n + 127) >> 7 : 1;
        const uint4 *q = reinterpret_cast<const uint4 *>(p);
        for (uint64_t j = 0; j + 1 < ncomp; j++) {      // full blocks that are not the last
            uint64_t m[16];
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const uint4 c = q[8 * j + i];
                m[2 * i] = pack64(c.x, c.y);
                m[2 * i + 1] = pack64(c.z, c.w);
            }
            blake2b_compress(h, m, 128 * (j + 1), false);
        }
        uint64_t m[16];
#pragma unroll
        for (int i = 0; i < 16; i++) m[i] = word_or_zero(p, n, 16 * (ncomp - 1) + i);
        blake2b_compress(h, m, n, true);
#pragma unroll
        for (int i = 0; i < 8; i++) { out[2 * i] = (uint32_t)h[i]; out[2 * i + 1] = (uint32_t)(h[i] >> 32); }
    }

    // H(l || r): one 128-byte block
    __device__ static void pair(const uint32_t (&l)[WORDS], const uint32_t (&r)[WORDS], uint32_t (&out)[WORDS])
    {
        uint64_t h[8], m[16];
#pragma unroll
        for (int i = 0; i < 8; i++) {
            h[i] = b2_iv(i);
            m[i] = pack64(l[2 * i], l[2 * i + 1]);
            m[8 + i] = pack64(r[2 * i], r[2 * i + 1]);
        }
        h[0] ^= 0x0000000001010040ull;
        blake2b_compress(h, m, 128, true);
#pragma unroll
        for (int i = 0; i < 8; i++) { out[2 * i] = (uint32_t)h[i]; out[2 * i + 1] = (uint32_t)(h[i] >> 32); }
    }
};

// ---------------------------------------------------------------------------
// SHA3-256 (FIPS 202): Keccak-f[1600], rate 136 bytes
// ---------------------------------------------------------------------------

// round constants from the LFSR of FIPS 202 section 3.2.5, evaluated at compile time
constexpr uint64_t keccak_rc(int round)
{
    uint32_t R = 1;
    uint64_t rc = 0;
    for (int r = 0; r <= round; r++) {
        rc = 0;
        for (int j = 0; j <= 6; j++) {
            if (R & 1) rc |= (uint64_t)1 << ((1 << j) - 1);
            const uint32_t hi = R & 0x80;
            R = (R << 1) & 0xff;
            if (hi) R ^= 0x71;
        }
    }
    return rc;
}
struct KeccakRC {
    uint64_t v[24];
};
constexpr KeccakRC make_keccak_rc()
{
    KeccakRC t = {};
    for (int r = 0; r < 24; r++) t.v[r] = keccak_rc(r);
    return t;
}
__device__ const KeccakRC KECCAK_RC = make_keccak_rc();

// rotation offset of lane (x, y): the (t+1)(t+2)/2 walk of FIPS 202 section 3.2.2
constexpr int keccak_rho(int x, int y)
{
    if (x == 0 && y == 0) return 0;
    int cx = 1, cy = 0;
    for (int t = 0; t < 24; t++) {
        if (cx == x && cy == y) return ((t + 1) * (t + 2) / 2) % 64;
        const int nx = cy, ny = (2 * cx + 3 * cy) % 5;
        cx = nx; cy = ny;
    }
    return 0;
}

template <int N>
__device__ __forceinline__ uint64_t rotl64c(uint64_t x)
{
    if (N == 0) return x;
    const uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
    if (N == 32) return pack64(hi, lo);
    if (N < 32) return pack64(__builtin_amdgcn_alignbit(lo, hi, 32 - N), __builtin_amdgcn_alignbit(hi, lo, 32 - N));
    return pack64(__builtin_amdgcn_alignbit(hi, lo, 64 - N), __builtin_amdgcn_alignbit(lo, hi, 64 - N));
}

__device__ __forceinline__ uint64_t xor3_64(uint64_t a, uint64_t b, uint64_t c)
{
    return pack64(__builtin_amdgcn_bitop3_b32((uint32_t)a, (uint32_t)b, (uint32_t)c, 0x96),
                  __builtin_amdgcn_bitop3_b32((uint32_t)(a >> 32), (uint32_t)(b >> 32), (uint32_t)(c >> 32), 0x96));
}
__device__ __forceinline__ uint64_t chi64(uint64_t a, uint64_t b, uint64_t c)   // a ^ (~b & c)
{
    return pack64(__builtin_amdgcn_bitop3_b32((uint32_t)a, (uint32_t)b, (uint32_t)c, 0xD2),
                  __builtin_amdgcn_bitop3_b32((uint32_t)(a >> 32), (uint32_t)(b >> 32), (uint32_t)(c >> 32), 0xD2));
}

template <int X, int Y>
__device__ __forceinline__ void rho_pi(const uint64_t (&A)[25], uint64_t (&B)[25])
{
    B[Y + 5 * ((2 * X + 3 * Y) % 5)] = rotl64c<keccak_rho(X, Y)>(A[X + 5 * Y]);
}

__device__ __forceinline__ void keccak_f1600(uint64_t (&A)[25])
{
#pragma unroll 1
    for (int round = 0; round < 24; round++) {
        uint64_t C[5], D[5], B[25];
#pragma unroll
        for (int x = 0; x < 5; x++) C[x] = xor3_64(xor3_64(A[x], A[x + 5], A[x + 10]), A[x + 15], A[x + 20]);
#pragma unroll
        for (int x = 0; x < 5; x++) D[x] = C[(x + 4) % 5] ^ rotl64c<1>(C[(x + 1) % 5]);
#pragma unroll
        for (int i = 0; i < 25; i++) A[i] ^= D[i % 5];
        rho_pi<0, 0>(A, B); rho_pi<1, 0>(A, B); rho_pi<2, 0>(A, B); rho_pi<3, 0>(A, B); rho_pi<4, 0>(A, B);
        rho_pi<0, 1>(A, B); rho_pi<1, 1>(A, B); rho_pi<2, 1>(A, B); rho_pi<3, 1>(A, B); rho_pi<4, 1>(A, B);
        rho_pi<0, 2>(A, B); rho_pi<1, 2>(A, B); rho_pi<2, 2>(A, B); rho_pi<3, 2>(A, B); rho_pi<4, 2>(A, B);
        rho_pi<0, 3>(A, B); rho_pi<1, 3>(A, B); rho_pi<2, 3>(A, B); rho_pi<3, 3>(A, B); rho_pi<4, 3>(A, B);
        rho_pi<0, 4>(A, B); rho_pi<1, 4>(A, B); rho_pi<2, 4>(A, B); rho_pi<3, 4>(A, B); rho_pi<4, 4>(A, B);
#pragma unroll
        for (int y = 0; y < 5; y++)
#pragma unroll
            for (int x = 0; x < 5; x++) A[x + 5 * y] = chi64(B[x + 5 * y], B[(x + 1) % 5 + 5 * y], B[(x + 2) % 5 + 5 * y]);
        A[0] ^= KECCAK_RC.v[round];
    }
}

struct Sha3Tree {
    static constexpr int WORDS = 8;
    static constexpr int RATE_WORDS = 17;   // 136 bytes

    __device__ static void squeeze(const uint64_t (&A)[25], uint32_t (&out)[WORDS])
    {
#pragma unroll
        for (int i = 0; i < 4; i++) { out[2 * i] = (uint32_t)A[i]; out[2 * i + 1] = (uint32_t)(A[i] >> 32); }
    }

    __device__ static void leaf(const uint8_t *p, uint64_t n, uint32_t (&out)[WORDS])
    {
        uint64_t A[25];
#pragma unroll
        for (int i = 0; i < 25; i++) A[i] = 0;
        const uint64_t nfull = n / 136;
        const uint64_t *q = reinterpret_cast<const uint64_t *>(p);   // leaf starts are 16-byte aligned, 136 = 17 * 8
        for (uint64_t j = 0; j < nfull; j++) {
#pragma unroll
            for (int i = 0; i < RATE_WORDS; i++) A[i] ^= q[RATE_WORDS * j + i];
            keccak_f1600(A);
        }
        // last block: the remaining bytes, 0x06 after them, 0x80 in the last byte of the rate
        const uint32_t rem = (uint32_t)(n - 136 * nfull);
#pragma unroll
        for (int i = 0; i < RATE_WORDS; i++) {
            uint64_t w = word_or_zero(p, n, RATE_WORDS * nfull + i);
            if ((uint32_t)i == rem / 8) w ^= (uint64_t)0x06 << (8 * (rem % 8));
            A[i] ^= w;
        }
        A[16] ^= 0x8000000000000000ull;
        keccak_f1600(A);
        squeeze(A, out);
    }

    // H(l || r): 64 bytes, one block
    __device__ static void pair(const uint32_t (&l)[WORDS], const uint32_t (&r)[WORDS], uint32_t (&out)[WORDS])
    {
        uint64_t A[25];
#pragma unroll
        for (int i = 0; i < 25; i++) A[i] = 0;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            A[i] = pack64(l[2 * i], l[2 * i + 1]);
            A[4 + i] = pack64(r[2 * i], r[2 * i + 1]);
        }
        A[8] = 0x06;
        A[16] = 0x8000000000000000ull;
        keccak_f1600(A);
        squeeze(A, out);
    }
};

// ---------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------

template <class H, int WG>
__global__ void __launch_bounds__(WG)
other_leaf_kernel(const uint8_t *base, uint64_t len, uint64_t n_leaves, uint64_t leaf_bytes, uint32_t *out)
{
    const uint64_t leaf = (uint64_t)blockIdx.x * WG + threadIdx.x;
    if (leaf >= n_leaves) return;
    const uint64_t start = leaf * leaf_bytes;
    const uint64_t left = len - start;
    uint32_t d[H::WORDS];
    H::leaf(base + start, left < leaf_bytes ? left : leaf_bytes, d);
#pragma unroll
    for (int i = 0; i < H::WORDS; i += 4)
        *reinterpret_cast<uint4 *>(out + leaf * H::WORDS + i) = make_uint4(d[i], d[i + 1], d[i + 2], d[i + 3]);
}

// 512 consecutive nodes per workgroup -> one node (first level from memory, the rest in LDS)
template <class H>
__global__ void __launch_bounds__(OTHER_WG)
other_reduce_kernel(const uint32_t *in, uint64_t n, uint8_t *out)
{
    constexpr int W = H::WORDS;
    __shared__ uint32_t lds[2][W][OTHER_WG];
    const uint32_t tid = threadIdx.x;
    const uint64_t first = (uint64_t)blockIdx.x * OTHER_RED_IN;
    const uint64_t rem = n - first;
    const uint32_t count = rem < (uint64_t)OTHER_RED_IN ? (uint32_t)rem : (uint32_t)OTHER_RED_IN;
    const uint32_t pairs = count >> 1;
    if (tid < pairs) {
        uint32_t l[W], r[W], d[W];
#pragma unroll
        for (int i = 0; i < W; i++) { l[i] = in[(first + 2 * tid) * W + i]; r[i] = in[(first + 2 * tid + 1) * W + i]; }
        H::pair(l, r, d);
#pragma unroll
        for (int i = 0; i < W; i++) lds[0][i][tid] = d[i];
    } else if (tid == pairs && (count & 1)) {
#pragma unroll
        for (int i = 0; i < W; i++) lds[0][i][tid] = in[(first + count - 1) * W + i];
    }
    __syncthreads();
    uint32_t cnt = pairs + (count & 1);
    int cur = 0;
    while (cnt > 1) {
        const uint32_t pr = cnt >> 1;
        if (tid < pr) {
            uint32_t l[W], r[W], d[W];
#pragma unroll
            for (int i = 0; i < W; i++) { l[i] = lds[cur][i][2 * tid]; r[i] = lds[cur][i][2 * tid + 1]; }
            H::pair(l, r, d);
#pragma unroll
            for (int i = 0; i < W; i++) lds[cur ^ 1][i][tid] = d[i];
        } else if (tid == pr && (cnt & 1)) {
#pragma unroll
            for (int i = 0; i < W; i++) lds[cur ^ 1][i][pr] = lds[cur][i][cnt - 1];
        }
        __syncthreads();
        cnt = pr + (cnt & 1);
        cur ^= 1;
    }
    if (tid == 0) {
        uint8_t *o = out + (uint64_t)blockIdx.x * 4 * W;
        if ((reinterpret_cast<uintptr_t>(o) & 3) == 0) {
            for (int i = 0; i < W; i++) reinterpret_cast<uint32_t *>(o)[i] = lds[cur][i][0];
        } else {
            for (int i = 0; i < W; i++)
                for (int j = 0; j < 4; j++) o[4 * i + j] = (uint8_t)(lds[cur][i][0] >> (8 * j));
        }
    }
}

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

template <class H>
int tree_root(const void *dev_buf, size_t len, size_t leaf_bytes, uint8_t *out_digest, hipStream_t s)
{
    constexpr size_t DL = 4 * H::WORDS;
    uint64_t n = ceil_div(len, leaf_bytes);
    if (n == 0) n = 1;
    SENTRY_REQUIRE(n <= 0xffffffffull - OTHER_WG, "sentry_merkle_root_h: too many leaves");
    void *a, *b;
    int rc = sentry::scratch_get(s, sentry::R_NODES_A, DL * n, &a);
    if (rc) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_NODES_B, DL * ceil_div(n, OTHER_RED_IN), &b))) return rc;
    const uint8_t *base = static_cast<const uint8_t *>(dev_buf);
    if (ceil_div(n, 64) <= 2048)   // few leaves: single-wave workgroups spread over all SIMDs
        hipLaunchKernelGGL((other_leaf_kernel<H, OTHER_WG_SMALL>), dim3((uint32_t)ceil_div(n, OTHER_WG_SMALL)),
                           dim3(OTHER_WG_SMALL), 0, s, base, (uint64_t)len, n, (uint64_t)leaf_bytes, static_cast<uint32_t *>(a));
    else
        hipLaunchKernelGGL((other_leaf_kernel<H, OTHER_WG>), dim3((uint32_t)ceil_div(n, OTHER_WG)), dim3(OTHER_WG), 0, s,
                           base, (uint64_t)len, n, (uint64_t)leaf_bytes, static_cast<uint32_t *>(a));
    SENTRY_HIP_CHECK(hipGetLastError());
    uint8_t *bufs[2] = {static_cast<uint8_t *>(b), static_cast<uint8_t *>(a)};
    const uint32_t *src = static_cast<const uint32_t *>(a);
    uint64_t m = n;
    int turn = 0;
    do {   // at least one pass, so that the result lands in out_digest
        const uint64_t g = ceil_div(m, OTHER_RED_IN);
        uint8_t *dst = g == 1 ? out_digest : bufs[turn];
        hipLaunchKernelGGL(other_reduce_kernel<H>, dim3((uint32_t)g), dim3(OTHER_WG), 0, s, src, m, dst);
        SENTRY_HIP_CHECK(hipGetLastError());
        src = reinterpret_cast<const uint32_t *>(dst);
        m = g;
        turn ^= 1;
    } while (m > 1);
    return SENTRY_OK;
}

}  // namespace

extern "C" {

int sentry_merkle_root_h(int hash, const void *dev_buf, size_t len, size_t leaf_bytes, uint8_t *out_digest,
                         void *stream)
{
    sentry::clear_error();
    if (hash == SENTRY_HASH_SHA256) return sentry_merkle_root(dev_buf, len, leaf_bytes, out_digest, stream);
    SENTRY_REQUIRE(hash == SENTRY_HASH_BLAKE2B || hash == SENTRY_HASH_SHA3_256, "sentry_merkle_root_h: unknown hash %d", hash);
    SENTRY_REQUIRE(leaf_bytes > 0 && leaf_bytes % 64 == 0,
                   "sentry_merkle_root_h: leaf_bytes must be a positive multiple of 64 (got %zu)", leaf_bytes);
    SENTRY_REQUIRE(dev_buf != nullptr || len == 0, "sentry_merkle_root_h: NULL buffer with len %zu", len);
    SENTRY_REQUIRE((reinterpret_cast<uintptr_t>(dev_buf) & 15) == 0, "sentry_merkle_root_h: buffer %p is not 16-byte aligned",
                   dev_buf);
    SENTRY_REQUIRE(out_digest != nullptr, "sentry_merkle_root_h: NULL out_digest");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hash == SENTRY_HASH_BLAKE2B) return tree_root<Blake2bTree>(dev_buf, len, leaf_bytes, out_digest, s);
    return tree_root<Sha3Tree>(dev_buf, len, leaf_bytes, out_digest, s);
}

}  // extern "C"

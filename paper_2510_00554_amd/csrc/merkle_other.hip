// Merkle trees over the paper's other two leaf functions, BLAKE2b-512 and SHA3-256 (section
// 4.2.1 names three hash functions for the tree: SHA-256, BLAKE2b and SHA-3).  Same tree rules
// as the SHA-256 path: one leaf per lane, node = H(left || right)
// with the full hash, a lone last node moves up unchanged, a short last leaf is hashed at its
// true length.  These kernels are the plain version of the scheme (leaf digests to memory,
// then 512 nodes folded per workgroup in LDS); the tuned path is the SHA-256 one.
//
// Fragmented tensors (per-tensor trees of Algorithm 2, the flat in-place tree of Algorithm 3)
// are driven by small tables instead of one launch per tensor: the prefix sums of the
// tensors' leaf counts, and of their node counts on every later level.  A lane (leaf kernel)
// or a workgroup (reduce kernel) finds its tensor by binary search in the prefix sums, which
// is a dozen steps next to a hash of thousands of instructions.
#include <cstring>
#include <vector>

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

template <class H>
__device__ __forceinline__ void store_leaf_digest(uint32_t *out, uint64_t leaf, const uint32_t (&d)[H::WORDS])
{
#pragma unroll
    for (int i = 0; i < H::WORDS; i += 4)
        *reinterpret_cast<uint4 *>(out + leaf * H::WORDS + i) = make_uint4(d[i], d[i + 1], d[i + 2], d[i + 3]);
}

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
    store_leaf_digest<H>(out, leaf, d);
}

struct SegDesc {
    const uint8_t *base;
    uint64_t len;
};

// the last t < n with start[t] <= i, for a non-decreasing start[0..n] with start[0] <= i < start[n]
__device__ __forceinline__ uint32_t find_segment(const uint64_t *start, uint32_t n, uint64_t i)
{
    uint32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (start[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
}

// Leaf kernel over fragmented tensors: leaf_start[t] = number of leaves before tensor t
// (n_seg + 1 entries); leaf i of the launch is leaf i - leaf_start[t] of its tensor and its
// digest goes to position i, so the digests of a tensor are adjacent and in order.
template <class H, int WG>
__global__ void __launch_bounds__(WG)
other_leaf_table_kernel(const SegDesc *segs, const uint64_t *leaf_start, uint32_t n_seg, uint64_t leaf_bytes,
                        uint32_t *out)
{
    const uint64_t leaf = (uint64_t)blockIdx.x * WG + threadIdx.x;
    if (leaf >= leaf_start[n_seg]) return;
    const uint32_t t = find_segment(leaf_start, n_seg, leaf);
    const SegDesc sd = segs[t];
    const uint64_t start = (leaf - leaf_start[t]) * leaf_bytes;   // 0 for the empty leaf of an empty tensor
    const uint64_t left = sd.len - start;
    uint32_t d[H::WORDS];
    H::leaf(sd.base + start, left < leaf_bytes ? left : leaf_bytes, d);
    store_leaf_digest<H>(out, leaf, d);
}

// count (1..512) consecutive nodes at in + first -> one node at o (first level from memory,
// the rest in LDS); all lanes of the workgroup call this
template <class H>
__device__ __forceinline__ void reduce_group(const uint32_t *in, uint64_t first, uint32_t count, uint8_t *o)
{
    constexpr int W = H::WORDS;
    __shared__ uint32_t lds[2][W][OTHER_WG];
    const uint32_t tid = threadIdx.x;
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
        if ((reinterpret_cast<uintptr_t>(o) & 3) == 0) {
            for (int i = 0; i < W; i++) reinterpret_cast<uint32_t *>(o)[i] = lds[cur][i][0];
        } else {
            for (int i = 0; i < W; i++)
                for (int j = 0; j < 4; j++) o[4 * i + j] = (uint8_t)(lds[cur][i][0] >> (8 * j));
        }
    }
}

// 512 consecutive nodes per workgroup -> one node
template <class H>
__global__ void __launch_bounds__(OTHER_WG)
other_reduce_kernel(const uint32_t *in, uint64_t n, uint8_t *out)
{
    const uint64_t first = (uint64_t)blockIdx.x * OTHER_RED_IN;
    const uint64_t rem = n - first;
    reduce_group<H>(in, first, rem < (uint64_t)OTHER_RED_IN ? (uint32_t)rem : (uint32_t)OTHER_RED_IN,
                    out + (uint64_t)blockIdx.x * 4 * H::WORDS);
}

// One level of all per-tensor trees: node_start[t] = nodes before tensor t on this level,
// group_start[t] = workgroups (= nodes of the next level) before tensor t; a tensor with m
// nodes has ceil(m / 512) workgroups, the last one short.  Every tensor has at least one node.
template <class H>
__global__ void __launch_bounds__(OTHER_WG)
other_reduce_table_kernel(const uint32_t *in, const uint64_t *node_start, const uint64_t *group_start, uint32_t n_seg,
                          uint8_t *out)
{
    const uint64_t g = blockIdx.x;
    const uint32_t t = find_segment(group_start, n_seg, g);
    const uint64_t local = g - group_start[t];
    const uint64_t m = node_start[t + 1] - node_start[t];
    const uint64_t rem = m - local * OTHER_RED_IN;
    reduce_group<H>(in, node_start[t] + local * OTHER_RED_IN,
                    rem < (uint64_t)OTHER_RED_IN ? (uint32_t)rem : (uint32_t)OTHER_RED_IN, out + g * 4 * H::WORDS);
}

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// few leaves: single-wave workgroups spread over all SIMDs
inline bool few_leaves(uint64_t n) { return ceil_div(n, 64) <= 2048; }

// Reduce m nodes at src to one digest at out_digest.  buf0 and buf1 hold ceil(m / 512) nodes
// each; src may be buf1 (it is no longer read when the second pass writes there), not buf0.
template <class H>
int reduce_flat(const uint32_t *src, uint64_t m, uint8_t *buf0, uint8_t *buf1, uint8_t *out_digest, hipStream_t s)
{
    uint8_t *bufs[2] = {buf0, buf1};
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
    if (few_leaves(n))
        hipLaunchKernelGGL((other_leaf_kernel<H, OTHER_WG_SMALL>), dim3((uint32_t)ceil_div(n, OTHER_WG_SMALL)),
                           dim3(OTHER_WG_SMALL), 0, s, base, (uint64_t)len, n, (uint64_t)leaf_bytes, static_cast<uint32_t *>(a));
    else
        hipLaunchKernelGGL((other_leaf_kernel<H, OTHER_WG>), dim3((uint32_t)ceil_div(n, OTHER_WG)), dim3(OTHER_WG), 0, s,
                           base, (uint64_t)len, n, (uint64_t)leaf_bytes, static_cast<uint32_t *>(a));
    SENTRY_HIP_CHECK(hipGetLastError());
    return reduce_flat<H>(static_cast<const uint32_t *>(a), n, static_cast<uint8_t *>(b), static_cast<uint8_t *>(a),
                          out_digest, s);
}

// Tables of a launch over fragmented tensors, uploaded in one copy:
//   SegDesc[n_seg] | level 0: start[n_seg + 1] | level 1: start[n_seg + 1] | ...
// level 0 holds the prefix sums of the leaf counts, level k + 1 those of ceil(count_k / 512).
struct SegTables {
    const SegDesc *segs;                       // device
    std::vector<const uint64_t *> level;       // device, one prefix-sum array per level
    std::vector<uint64_t> total;               // nodes per level
};

template <bool EMPTY_HAS_LEAF, bool ALL_LEVELS>
int upload_tables(const char *fn, const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes,
                  hipStream_t s, SegTables *out)
{
    std::vector<std::vector<uint64_t>> starts;
    {
        std::vector<uint64_t> l0(n_seg + 1);
        l0[0] = 0;
        for (size_t t = 0; t < n_seg; t++) {
            uint64_t nl = ceil_div(lens[t], leaf_bytes);
            if (EMPTY_HAS_LEAF && nl == 0) nl = 1;
            l0[t + 1] = l0[t] + nl;
        }
        starts.push_back(std::move(l0));
    }
    SENTRY_REQUIRE(starts[0][n_seg] <= 0xffffffffull - OTHER_WG, "%s: too many leaves", fn);
    while (ALL_LEVELS && starts.back()[n_seg] > n_seg) {   // some tensor still has more than one node
        const std::vector<uint64_t> &cur = starts.back();
        std::vector<uint64_t> nxt(n_seg + 1);
        nxt[0] = 0;
        for (size_t t = 0; t < n_seg; t++) nxt[t + 1] = nxt[t] + ceil_div(cur[t + 1] - cur[t], OTHER_RED_IN);
        starts.push_back(std::move(nxt));
    }
    const size_t level_bytes = 8 * (n_seg + 1);
    const size_t table_bytes = n_seg * sizeof(SegDesc) + starts.size() * level_bytes;
    void *host_tab, *dev_tab;
    int rc = sentry::table_staging_get(s, table_bytes, &host_tab);
    if (rc) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_TABLES, table_bytes, &dev_tab))) return rc;
    SegDesc *hseg = static_cast<SegDesc *>(host_tab);
    for (size_t t = 0; t < n_seg; t++) hseg[t] = SegDesc{static_cast<const uint8_t *>(dev_ptrs[t]), lens[t]};
    char *hp = static_cast<char *>(host_tab) + n_seg * sizeof(SegDesc);
    const char *dp = static_cast<const char *>(dev_tab) + n_seg * sizeof(SegDesc);
    out->segs = static_cast<const SegDesc *>(dev_tab);
    for (const std::vector<uint64_t> &lv : starts) {
        std::memcpy(hp, lv.data(), level_bytes);
        out->level.push_back(reinterpret_cast<const uint64_t *>(dp));
        out->total.push_back(lv[n_seg]);
        hp += level_bytes;
        dp += level_bytes;
    }
    SENTRY_HIP_CHECK(hipMemcpyAsync(dev_tab, host_tab, table_bytes, hipMemcpyHostToDevice, s));
    return sentry::table_staging_mark(s);
}

template <class H>
int launch_table_leaves(const SegTables &tab, size_t n_seg, size_t leaf_bytes, uint32_t *digests, hipStream_t s)
{
    const uint64_t n = tab.total[0];
    if (few_leaves(n))
        hipLaunchKernelGGL((other_leaf_table_kernel<H, OTHER_WG_SMALL>), dim3((uint32_t)ceil_div(n, OTHER_WG_SMALL)),
                           dim3(OTHER_WG_SMALL), 0, s, tab.segs, tab.level[0], (uint32_t)n_seg, (uint64_t)leaf_bytes, digests);
    else
        hipLaunchKernelGGL((other_leaf_table_kernel<H, OTHER_WG>), dim3((uint32_t)ceil_div(n, OTHER_WG)), dim3(OTHER_WG),
                           0, s, tab.segs, tab.level[0], (uint32_t)n_seg, (uint64_t)leaf_bytes, digests);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

// Algorithm 2 over hash H: per-tensor roots, then the tree over the roots.
template <class H>
int tree_segments(const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes,
                  uint8_t *out_seg_roots, uint8_t *out_root, hipStream_t s)
{
    constexpr size_t DL = 4 * H::WORDS;
    SegTables tab;
    int rc = upload_tables<true, true>("sentry_merkle_segments_h", dev_ptrs, lens, n_seg, leaf_bytes, s, &tab);
    if (rc) return rc;
    const size_t levels = tab.level.size();   // level 0 = leaves, the last level has one node per tensor
    void *a, *b = nullptr, *roots, *r0, *r1;
    if ((rc = sentry::scratch_get(s, sentry::R_SEG_ROOTS, DL * n_seg, &roots))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_RED_0, DL * ceil_div(n_seg, OTHER_RED_IN), &r0))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_RED_1, DL * ceil_div(n_seg, OTHER_RED_IN), &r1))) return rc;
    if (levels == 1) {
        a = roots;   // every tensor is a single leaf
    } else {
        if ((rc = sentry::scratch_get(s, sentry::R_NODES_A, DL * tab.total[0], &a))) return rc;
        if (levels > 2 && (rc = sentry::scratch_get(s, sentry::R_NODES_B, DL * tab.total[1], &b))) return rc;
    }
    if ((rc = launch_table_leaves<H>(tab, n_seg, leaf_bytes, static_cast<uint32_t *>(a), s))) return rc;
    const uint32_t *src = static_cast<const uint32_t *>(a);
    for (size_t k = 0; k + 1 < levels; k++) {
        // level k -> level k + 1: outputs alternate between the two node buffers, the last goes to roots
        uint8_t *dst = (k + 2 == levels) ? static_cast<uint8_t *>(roots) : static_cast<uint8_t *>((k & 1) ? a : b);
        hipLaunchKernelGGL(other_reduce_table_kernel<H>, dim3((uint32_t)tab.total[k + 1]), dim3(OTHER_WG), 0, s, src,
                           tab.level[k], tab.level[k + 1], (uint32_t)n_seg, dst);
        SENTRY_HIP_CHECK(hipGetLastError());
        src = reinterpret_cast<const uint32_t *>(dst);
    }
    if (out_seg_roots) SENTRY_HIP_CHECK(hipMemcpyAsync(out_seg_roots, roots, DL * n_seg, hipMemcpyDefault, s));
    return reduce_flat<H>(static_cast<const uint32_t *>(roots), n_seg, static_cast<uint8_t *>(r0),
                          static_cast<uint8_t *>(r1), out_root, s);
}

// Algorithm 3 over hash H: one flat tree over the blocks of all tensors.
template <class H>
int tree_inplace(const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes, uint8_t *out_root,
                 hipStream_t s)
{
    constexpr size_t DL = 4 * H::WORDS;
    uint64_t total = 0;
    for (size_t t = 0; t < n_seg; t++) total += ceil_div(lens[t], leaf_bytes);
    if (total == 0) return tree_root<H>(nullptr, 0, leaf_bytes, out_root, s);   // the single empty leaf
    SegTables tab;
    int rc = upload_tables<false, false>("sentry_merkle_inplace_h", dev_ptrs, lens, n_seg, leaf_bytes, s, &tab);
    if (rc) return rc;
    void *a, *b;
    if ((rc = sentry::scratch_get(s, sentry::R_NODES_A, DL * total, &a))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_NODES_B, DL * ceil_div(total, OTHER_RED_IN), &b))) return rc;
    if ((rc = launch_table_leaves<H>(tab, n_seg, leaf_bytes, static_cast<uint32_t *>(a), s))) return rc;
    return reduce_flat<H>(static_cast<const uint32_t *>(a), total, static_cast<uint8_t *>(b), static_cast<uint8_t *>(a),
                          out_root, s);
}

int check_segment_args(const char *fn, int hash, const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                       size_t leaf_bytes, const uint8_t *out_root)
{
    SENTRY_REQUIRE(hash == SENTRY_HASH_BLAKE2B || hash == SENTRY_HASH_SHA3_256, "%s: unknown hash %d", fn, hash);
    SENTRY_REQUIRE(n_seg >= 1 && n_seg <= 0xfffffffeull, "%s: n_seg must be 1 .. 2^32 - 2", fn);
    SENTRY_REQUIRE(dev_ptrs && lens && out_root, "%s: NULL argument", fn);
    SENTRY_REQUIRE(leaf_bytes > 0 && leaf_bytes % 64 == 0, "%s: leaf_bytes must be a positive multiple of 64 (got %zu)", fn,
                   leaf_bytes);
    for (size_t t = 0; t < n_seg; t++) {
        SENTRY_REQUIRE(dev_ptrs[t] != nullptr || lens[t] == 0, "%s: segment %zu is NULL", fn, t);
        SENTRY_REQUIRE((reinterpret_cast<uintptr_t>(dev_ptrs[t]) & 15) == 0, "%s: segment %zu is not 16-byte aligned", fn, t);
    }
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

int sentry_merkle_segments_h(int hash, const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes,
                             uint8_t *out_seg_roots, uint8_t *out_root, void *stream)
{
    sentry::clear_error();
    if (hash == SENTRY_HASH_SHA256)
        return sentry_merkle_segments(dev_ptrs, lens, n_seg, leaf_bytes, out_seg_roots, out_root, stream);
    int rc = check_segment_args("sentry_merkle_segments_h", hash, dev_ptrs, lens, n_seg, leaf_bytes, out_root);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hash == SENTRY_HASH_BLAKE2B)
        return tree_segments<Blake2bTree>(dev_ptrs, lens, n_seg, leaf_bytes, out_seg_roots, out_root, s);
    return tree_segments<Sha3Tree>(dev_ptrs, lens, n_seg, leaf_bytes, out_seg_roots, out_root, s);
}

int sentry_merkle_inplace_h(int hash, const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes,
                            uint8_t *out_root, void *stream)
{
    sentry::clear_error();
    if (hash == SENTRY_HASH_SHA256) return sentry_merkle_inplace(dev_ptrs, lens, n_seg, leaf_bytes, out_root, stream);
    int rc = check_segment_args("sentry_merkle_inplace_h", hash, dev_ptrs, lens, n_seg, leaf_bytes, out_root);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hash == SENTRY_HASH_BLAKE2B) return tree_inplace<Blake2bTree>(dev_ptrs, lens, n_seg, leaf_bytes, out_root, s);
    return tree_inplace<Sha3Tree>(dev_ptrs, lens, n_seg, leaf_bytes, out_root, s);
}

}  // extern "C"

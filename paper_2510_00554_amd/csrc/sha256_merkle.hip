// SHA-256 Merkle tree on gfx950: block hashing kernel and reduction kernel of
// section 4.2.1, the table-driven launch over fragmented tensors of section
// 4.2.1 "In-place Hashing", and the per-tensor digests of Algorithm 2.
//
// Mapping: one leaf per lane (SHA-256 is serial inside a leaf), 256 leaves per
// workgroup (64 when a launch has few leaves).  The workgroup folds its leaf
// digests through eight (six) tree levels in LDS, so the leaf kernel emits one
// node per 256 (64) leaves; later stages fold 512 nodes per workgroup.
// Power-of-two-aligned groups reduce to the same subtrees as the level-by-level
// rule, and only the last group of a buffer can be partial, so the promoted odd
// node lands where the plain rule puts it.
#include <cstring>
#include <mutex>
#include <vector>

#include "sentry_internal.h"

// Scratch of sentry_merkle_root_noalloc (the entry point that allocates nothing).
// Largest input: 2^22 leaves, that is at most 65,536 workgroup nodes whichever kernel is chosen.
constexpr uint64_t NOALLOC_MAX_LEAVES = 1ull << 22;
constexpr uint64_t NOALLOC_MAX_GROUPS = NOALLOC_MAX_LEAVES / 64;
constexpr size_t NOALLOC_NODES_BYTES = 32 * NOALLOC_MAX_GROUPS;                         // 2 MiB
constexpr size_t NOALLOC_RED_BYTES = 32 * ((NOALLOC_MAX_GROUPS + 511) / 512);   // 4 KiB, twice
constexpr size_t NOALLOC_TICKET_AT = NOALLOC_NODES_BYTES + 2 * NOALLOC_RED_BYTES;
constexpr size_t NOALLOC_BYTES = NOALLOC_TICKET_AT + 256;

// Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress: kernels get the
// address that call returns, never the name.
static __device__ __align__(256) unsigned char scratch[NOALLOC_BYTES];

namespace {

constexpr int LEAF_WG = 256;          // lanes = leaves per workgroup of the leaf kernel ...
constexpr int LEAF_WG_SMALL = 64;     // ... and when there are too few leaves to fill the chip
constexpr uint64_t SMALL_LAUNCH_WAVES = 2048;   // two waves per SIMD on 256 CUs x 4 SIMDs
constexpr uint64_t LONG_LEAF_BYTES = 32768;     // leaves this long: single-wave workgroups whatever the launch size
constexpr uint64_t SPLIT_LAUNCH_WAVES = 512;    // groups of 64 leaves the two-wave split kernel takes: two per CU
constexpr uint64_t SPLIT_SINGLE_GROUPS = 256;   // up to one group per CU: one pair per workgroup
constexpr int RED_WG = 256;           // lanes per workgroup of the reduce kernel
constexpr int RED_IN = 2 * RED_WG;    // nodes folded by one reduce workgroup
static_assert(LEAF_WG_SMALL == 64 && RED_IN == 512, "the fixed scratch array is sized for these");

struct SegDesc {
    const uint8_t *base;
    uint64_t len;
    uint64_t first_leaf;   // leaves of all segments before this one (used by the packed leaf stage)
};

// Packed leaf stage: lane L of the launch takes leaf L of the concatenated leaf list of all
// segments, whatever segment it belongs to, instead of every segment starting a workgroup of
// its own.  With few leaves per segment that halves the waves of a launch (291 tensors of a 7B
// checkpoint in 1 MiB leaves: 394 groups of at most 64 leaves become 202 full ones).  The
// segment is found by bisection over first_leaf (the last segment whose first_leaf is <= L,
// which skips segments without leaves).
struct PackedLeaf {
    const uint8_t *p;
    uint64_t len;
};
__device__ __forceinline__ PackedLeaf find_packed_leaf(const SegDesc *segs, uint32_t n_seg, uint64_t leaf, uint64_t leaf_bytes)
{
    uint32_t lo = 0, hi = n_seg;
    while (hi - lo > 1) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if (segs[mid].first_leaf <= leaf) lo = mid; else hi = mid;
    }
    const SegDesc sd = segs[lo];
    const uint64_t start = (leaf - sd.first_leaf) * leaf_bytes;
    const uint64_t left = sd.len - start;                // 0 only for an empty segment's single leaf
    return PackedLeaf{sd.base + start, left < leaf_bytes ? left : leaf_bytes};
}

// One workgroup's share of a stage: `count` consecutive items starting at `first`
// (leaf index inside segment `seg` for the leaf kernel, node index in the input
// array for the reduce kernel).  `out` is where the leaf kernel puts its result in the
// output array: the node index of the group when it folds its leaves, the index of the
// group's first leaf digest when it stores them all.
struct Group {
    uint64_t first;
    uint64_t out;
    uint32_t count;
    uint32_t seg;
};

// ---------------------------------------------------------------------------
// SHA-256 (FIPS 180-4) on 32-bit lanes
// ---------------------------------------------------------------------------

constexpr uint32_t k256(int t)
{
    constexpr uint32_t K[64] = {
        0x428a2f98u, 0x71374491u, 0xb5c0fbcfu, 0xe9b5dba5u, 0x3956c25bu, 0x59f111f1u, 0x923f82a4u, 0xab1c5ed5u,
        0xd807aa98u, 0x12835b01u, 0x243185beu, 0x550c7dc3u, 0x72be5d74u, 0x80deb1feu, 0x9bdc06a7u, 0xc19bf174u,
        0xe49b69c1u, 0xefbe4786u, 0x0fc19dc6u, 0x240ca1ccu, 0x2de92c6fu, 0x4a7484aau, 0x5cb0a9dcu, 0x76f988dau,
        0x983e5152u, 0xa831c66du, 0xb00327c8u, 0xbf597fc7u, 0xc6e00bf3u, 0xd5a79147u, 0x06ca6351u, 0x14292967u,
        0x27b70a85u, 0x2e1b2138u, 0x4d2c6dfcu, 0x53380d13u, 0x650a7354u, 0x766a0abbu, 0x81c2c92eu, 0x92722c85u,
        0xa2bfe8a1u, 0xa81a664bu, 0xc24b8b70u, 0xc76c51a3u, 0xd192e819u, 0xd6990624u, 0xf40e3585u, 0x106aa070u,
        0x19a4c116u, 0x1e376c08u, 0x2748774cu, 0x34b0bcb5u, 0x391c0cb3u, 0x4ed8aa4au, 0x5b9cca4fu, 0x682e6ff3u,
        0x748f82eeu, 0x78a5636fu, 0x84c87814u, 0x8cc70208u, 0x90befffau, 0xa4506cebu, 0xbef9a3f7u, 0xc67178f2u};
    return K[t];
}

constexpr uint32_t crotr(uint32_t x, int n) { return (x >> n) | (x << (32 - n)); }

// K[t] + W[t] of the second block of a 64-byte message: 0x80, zeros, bit length 512.
// The block is the same for every inner node, so its message schedule is a constant.
struct KW64 {
    uint32_t v[64];
};
constexpr KW64 make_pad64()
{
    uint32_t w[64] = {};
    w[0] = 0x80000000u;
    w[15] = 512u;
    for (int t = 16; t < 64; t++) {
        uint32_t s0 = crotr(w[t - 15], 7) ^ crotr(w[t - 15], 18) ^ (w[t - 15] >> 3);
        uint32_t s1 = crotr(w[t - 2], 17) ^ crotr(w[t - 2], 19) ^ (w[t - 2] >> 10);
        w[t] = s1 + w[t - 7] + s0 + w[t - 16];
    }
    KW64 r = {};
    for (int t = 0; t < 64; t++) r.v[t] = k256(t) + w[t];
    return r;
}

// gfx950 has a three-input boolean instruction (v_bitop3_b32); the immediate is the truth
// table of the function evaluated on a = 0xF0, b = 0xCC, c = 0xAA.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) { return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96); }
__device__ __forceinline__ uint32_t ch(uint32_t e, uint32_t f, uint32_t g) { return __builtin_amdgcn_bitop3_b32(e, f, g, 0xCA); }
__device__ __forceinline__ uint32_t maj(uint32_t a, uint32_t b, uint32_t c) { return __builtin_amdgcn_bitop3_b32(a, b, c, 0xE8); }
__device__ __forceinline__ uint32_t rotr(uint32_t x, uint32_t n) { return __builtin_amdgcn_alignbit(x, x, n); }
__device__ __forceinline__ uint32_t bsig0(uint32_t x) { return xor3(rotr(x, 2), rotr(x, 13), rotr(x, 22)); }
__device__ __forceinline__ uint32_t bsig1(uint32_t x) { return xor3(rotr(x, 6), rotr(x, 11), rotr(x, 25)); }
__device__ __forceinline__ uint32_t ssig0(uint32_t x) { return xor3(rotr(x, 7), rotr(x, 18), x >> 3); }
__device__ __forceinline__ uint32_t ssig1(uint32_t x) { return xor3(rotr(x, 17), rotr(x, 19), x >> 10); }

#define SENTRY_H0 {0x6a09e667u, 0xbb67ae85u, 0x3c6ef372u, 0xa54ff53au, 0x510e527fu, 0x9b05688cu, 0x1f83d9abu, 0x5be0cd19u}

// One compression: st <- st + rounds(st, block).  w holds the 16 big-endian words of
// the block and is overwritten by the rolling message schedule.  The eight working
// variables stay in fixed registers; the role of each register rotates with t.
__device__ __forceinline__ void sha256_compress(uint32_t (&st)[8], uint32_t (&w)[16])
{
    uint32_t v[8];
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = st[i];
#pragma unroll
    for (int t = 0; t < 64; t++) {
        // the word of round t is ready; the word of round t + 16 is made here, off this
        // round's critical path, and takes the place of the one just used
        const uint32_t wt = w[t & 15];
        if (t + 16 < 64)
            w[t & 15] = wt + ssig0(w[(t + 1) & 15]) + w[(t + 9) & 15] + ssig1(w[(t + 14) & 15]);
#define V(i) v[((i) - t) & 7]
        uint32_t t1 = V(7) + bsig1(V(4)) + ch(V(4), V(5), V(6)) + k256(t) + wt;
        V(3) += t1;
        V(7) = t1 + bsig0(V(0)) + maj(V(0), V(1), V(2));
#undef V
    }
#pragma unroll
    for (int i = 0; i < 8; i++) st[i] += v[i];
}

// The compression of the constant padding block that ends every 64-byte message.
__device__ __forceinline__ void sha256_compress_pad64(uint32_t (&st)[8])
{
    constexpr KW64 kw = make_pad64();
    uint32_t v[8];
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = st[i];
#pragma unroll
    for (int t = 0; t < 64; t++) {
#define V(i) v[((i) - t) & 7]
        uint32_t t1 = V(7) + bsig1(V(4)) + ch(V(4), V(5), V(6)) + kw.v[t];
        V(3) += t1;
        V(7) = t1 + bsig0(V(0)) + maj(V(0), V(1), V(2));
#undef V
    }
#pragma unroll
    for (int i = 0; i < 8; i++) st[i] += v[i];
}

// node = SHA-256(left || right); words are the big-endian words of the digests
__device__ __forceinline__ void node_hash(const uint32_t (&l)[8], const uint32_t (&r)[8], uint32_t (&out)[8])
{
    uint32_t st[8] = SENTRY_H0;
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 8; i++) { w[i] = l[i]; w[8 + i] = r[i]; }
    sha256_compress(st, w);
    sha256_compress_pad64(st);
#pragma unroll
    for (int i = 0; i < 8; i++) out[i] = st[i];
}

// Padding blocks of a leaf of llen bytes whose last r = llen % 64 bytes start at tail:
// k = 0 is the block holding those bytes and 0x80, k = 1 the extra block needed when
// r >= 56.  Only whole 4-byte words inside the leaf and single bytes are read.
__device__ __forceinline__ void build_tail(uint32_t (&w)[16], const uint8_t *tail, uint32_t r,
                                           uint64_t llen, uint32_t k)
{
#pragma unroll
    for (int i = 0; i < 16; i++) w[i] = 0;
    if (k == 0) {
        const uint32_t *tw = reinterpret_cast<const uint32_t *>(tail);   // leaf starts are 16-byte aligned
        const uint32_t rw = r >> 2, rb = r & 3;
        uint32_t part = 0x80u << (24 - 8 * rb);
        for (uint32_t j = 0; j < rb; j++) part |= (uint32_t)tail[4 * rw + j] << (24 - 8 * j);
#pragma unroll
        for (int i = 0; i < 16; i++) {
            if ((uint32_t)(4 * i + 4) <= r) w[i] = __builtin_bswap32(tw[i]);
            if ((uint32_t)i == rw) w[i] = part;
        }
    }
    if (k == 1 || r < 56) {
        const uint64_t bits = llen * 8;
        w[14] = (uint32_t)(bits >> 32);
        w[15] = (uint32_t)bits;
    }
}

__device__ __forceinline__ void bswap_block(uint32_t (&w)[16], const uint4 &a, const uint4 &b, const uint4 &c,
                                            const uint4 &d)
{
    w[0] = __builtin_bswap32(a.x); w[1] = __builtin_bswap32(a.y); w[2] = __builtin_bswap32(a.z); w[3] = __builtin_bswap32(a.w);
    w[4] = __builtin_bswap32(b.x); w[5] = __builtin_bswap32(b.y); w[6] = __builtin_bswap32(b.z); w[7] = __builtin_bswap32(b.w);
    w[8] = __builtin_bswap32(c.x); w[9] = __builtin_bswap32(c.y); w[10] = __builtin_bswap32(c.z); w[11] = __builtin_bswap32(c.w);
    w[12] = __builtin_bswap32(d.x); w[13] = __builtin_bswap32(d.y); w[14] = __builtin_bswap32(d.z); w[15] = __builtin_bswap32(d.w);
}

// SHA-256 of llen bytes at p (16-byte aligned).  A lane walks its leaf in pairs of blocks:
// the eight 16-byte loads of a pair cover one whole 128-byte cache line, so every line is
// fetched by one burst of one lane and never has to survive in L2 between two visits.  The
// loads of the next pair are issued before the second compression of the current pair.
__device__ __forceinline__ void hash_leaf(uint32_t (&st)[8], const uint8_t *p, uint64_t llen)
{
    const uint64_t nblk = llen >> 6;
    const uint32_t r = (uint32_t)(llen & 63);
    const uint64_t total = nblk + 1 + (r >= 56 ? 1 : 0);
    const uint4 *q = reinterpret_cast<const uint4 *>(p);
    uint4 c[8] = {};
    if (nblk >= 1) { c[0] = q[0]; c[1] = q[1]; c[2] = q[2]; c[3] = q[3]; }
    if (nblk >= 2) { c[4] = q[4]; c[5] = q[5]; c[6] = q[6]; c[7] = q[7]; }
    for (uint64_t b = 0; b < total; b++) {
        uint32_t w[16];
        if (b < nblk) {
            if ((b & 1) == 0) {
                bswap_block(w, c[0], c[1], c[2], c[3]);
            } else {
                bswap_block(w, c[4], c[5], c[6], c[7]);
                q += 8;                                  // blocks b+1 and b+2
                if (b + 1 < nblk) { c[0] = q[0]; c[1] = q[1]; c[2] = q[2]; c[3] = q[3]; }
                if (b + 2 < nblk) { c[4] = q[4]; c[5] = q[5]; c[6] = q[6]; c[7] = q[7]; }
            }
        } else {
            build_tail(w, p + (nblk << 6), r, llen, (uint32_t)(b - nblk));
        }
        sha256_compress(st, w);
    }
}

// Store a digest (big-endian words) as its 32 canonical bytes.
__device__ __forceinline__ void store_digest(uint8_t *out, const uint32_t (&d)[8])
{
    if ((reinterpret_cast<uintptr_t>(out) & 15) == 0) {
        uint4 *o = reinterpret_cast<uint4 *>(out);
        o[0] = make_uint4(__builtin_bswap32(d[0]), __builtin_bswap32(d[1]), __builtin_bswap32(d[2]), __builtin_bswap32(d[3]));
        o[1] = make_uint4(__builtin_bswap32(d[4]), __builtin_bswap32(d[5]), __builtin_bswap32(d[6]), __builtin_bswap32(d[7]));
    } else {
        for (int i = 0; i < 8; i++)
            for (int j = 0; j < 4; j++) out[4 * i + j] = (uint8_t)(d[i] >> (24 - 8 * j));
    }
}

__device__ __forceinline__ void load_digest(const uint8_t *in, uint32_t (&d)[8])   // 16-byte aligned
{
    const uint4 *p = reinterpret_cast<const uint4 *>(in);
    uint4 a = p[0], b = p[1];
    d[0] = __builtin_bswap32(a.x); d[1] = __builtin_bswap32(a.y);
    d[2] = __builtin_bswap32(a.z); d[3] = __builtin_bswap32(a.w);
    d[4] = __builtin_bswap32(b.x); d[5] = __builtin_bswap32(b.y);
    d[6] = __builtin_bswap32(b.z); d[7] = __builtin_bswap32(b.w);
}

// Fold cnt (<= WG) nodes held in lds[0] (word-major: lds[buf][word][node]) to one node by
// the pairwise rule; a lone last node moves up unchanged.  All lanes of the workgroup
// call this; on return lane 0 holds the result in out.
template <int WG>
__device__ __forceinline__ void wg_tree_fold(uint32_t (&lds)[2][8][WG], uint32_t cnt, uint32_t tid,
                                             uint32_t (&out)[8])
{
    int cur = 0;
    while (cnt > 1) {
        const uint32_t pairs = cnt >> 1;
        if (tid < pairs) {
            uint32_t l[8], r[8], d[8];
#pragma unroll
            for (int i = 0; i < 8; i++) { l[i] = lds[cur][i][2 * tid]; r[i] = lds[cur][i][2 * tid + 1]; }
            node_hash(l, r, d);
#pragma unroll
            for (int i = 0; i < 8; i++) lds[cur ^ 1][i][tid] = d[i];
        } else if (tid == pairs && (cnt & 1)) {
#pragma unroll
            for (int i = 0; i < 8; i++) lds[cur ^ 1][i][pairs] = lds[cur][i][cnt - 1];
        }
        __syncthreads();
        cnt = pairs + (cnt & 1);
        cur ^= 1;
    }
    if (tid == 0) {
#pragma unroll
        for (int i = 0; i < 8; i++) out[i] = lds[cur][i][0];
    }
}

// One-launch tree for launches of at most 512 workgroups (TAIL): every workgroup stores its node,
// makes it visible to the device and takes a ticket; the workgroup that draws the last ticket
// folds all the nodes itself, so that no second launch is needed (the launch gap and the start of
// a kernel are a twentieth of a 16 MiB call).  The ticket counter is zero before the launch and
// the last workgroup puts it back to zero.
//
// tail_ticket: called by all lanes of the workgroup after its node is stored (by lane 0, before
// the call); true in all lanes of the workgroup that finishes last.
__device__ __forceinline__ bool tail_ticket(uint32_t *ticket, uint32_t tid, uint32_t *flag)
{
    __syncthreads();          // every node store of this workgroup precedes the ticket
    if (tid == 0) {
        __threadfence();      // release: the node is visible to the whole device first
        *flag = atomicAdd(ticket, 1u) == gridDim.x - 1;
    }
    __syncthreads();
    if (!*flag) return false;
    __threadfence();          // acquire: nothing read below comes from a stale cache line
    return true;
}

// Fold cnt (2 .. 512) nodes at `nodes` (device memory, written by other workgroups) to one digest
// at `out` by the pairwise rule; all NT lanes of the workgroup call this.  t = LDS, 2 x 8 x 512 words.
template <int NT>
__device__ __forceinline__ void tail_fold(const uint8_t *nodes, uint32_t cnt, uint8_t *out, uint32_t *ticket,
                                          uint32_t tid, uint32_t (*t)[8][RED_IN])
{
    for (uint32_t i = tid; i < cnt; i += NT) {
        uint32_t d[8];
        load_digest(nodes + 32 * (uint64_t)i, d);
#pragma unroll
        for (int k = 0; k < 8; k++) t[0][k][i] = d[k];
    }
    __syncthreads();
    int cur = 0;
#pragma unroll 1
    while (cnt > 1) {
        const uint32_t pairs = cnt >> 1;
#pragma unroll 1
        for (uint32_t i = tid; i < pairs; i += NT) {
            uint32_t l[8], r[8], d[8];
#pragma unroll
            for (int k = 0; k < 8; k++) { l[k] = t[cur][k][2 * i]; r[k] = t[cur][k][2 * i + 1]; }
            node_hash(l, r, d);
#pragma unroll
            for (int k = 0; k < 8; k++) t[cur ^ 1][k][i] = d[k];
        }
        if (tid == 0 && (cnt & 1)) {
#pragma unroll
            for (int k = 0; k < 8; k++) t[cur ^ 1][k][pairs] = t[cur][k][cnt - 1];
        }
        __syncthreads();
        cnt = pairs + (cnt & 1);
        cur ^= 1;
    }
    if (tid == 0) {
        uint32_t root[8];
#pragma unroll
        for (int k = 0; k < 8; k++) root[k] = t[cur][k][0];
        store_digest(out, root);
        *ticket = 0;          // ready for the next launch
    }
}

// Block hashing kernel.  FUSE: fold the workgroup's leaves in LDS and store one node per
// workgroup at out + 32*blockIdx; otherwise store every leaf digest at out + 32*leaf.
// WG = leaves per workgroup: 256, or 64 (one wave per workgroup).  A lone wave on a SIMD issues
// faster than two that share it, so a launch that cannot give every SIMD two waves is cut into
// single-wave workgroups, which the dispatcher spreads over all SIMDs of the chip.  Long leaves
// get single-wave workgroups as well: a workgroup then lives for milliseconds, and when other
// kernels share the chip a single wave fits any free wave slot, where a workgroup of four
// waves needs one on every SIMD of a CU at once (70B stream beside two chain-bound launches:
// 103.8 -> 99.4 ms); with the chip to itself the launch takes the same time either way, and
// with short leaves the deeper fold of 256 digests in LDS is worth 2-3 %.
__host__ inline bool single_wave_groups(uint64_t waves, uint64_t leaf_bytes)
{
    return waves <= SMALL_LAUNCH_WAVES || leaf_bytes >= LONG_LEAF_BYTES;
}

// PACKED (with SEGMENTED, without FUSE): nleaves0 = leaves of all segments, n_seg = segments;
// digest L goes to out + 32 L.
// TAIL (with FUSE, one buffer): the one-launch tree; `out` holds gridDim.x nodes, root to final_out.
template <int WG, bool FUSE, bool SEGMENTED, bool PACKED = false, bool TAIL = false>
__global__ void __launch_bounds__(WG)
merkle_leaf_kernel(const uint8_t *base0, uint64_t len0, uint64_t nleaves0, const SegDesc *segs, uint32_t n_seg,
                   const Group *groups, uint64_t leaf_bytes, uint8_t *out, uint32_t *ticket = nullptr,
                   uint8_t *final_out = nullptr)
{
    static_assert(!TAIL || (FUSE && !SEGMENTED && !PACKED), "the one-launch tree is for one buffer");
    const uint32_t g = blockIdx.x, tid = threadIdx.x;
    if (PACKED) {
        static_assert(!PACKED || (SEGMENTED && !FUSE), "the packed leaf stage writes leaf digests");
        const uint64_t leaf = (uint64_t)g * WG + tid;
        if (leaf >= nleaves0) return;
        const PackedLeaf pl = find_packed_leaf(segs, n_seg, leaf, leaf_bytes);
        uint32_t st[8] = SENTRY_H0;
        hash_leaf(st, pl.p, pl.len);
        store_digest(out + 32 * leaf, st);
        return;
    }
    const uint8_t *base;
    uint64_t seglen, first, out_at;
    uint32_t count;
    if (SEGMENTED) {
        const Group gr = groups[g];
        const SegDesc sd = segs[gr.seg];
        base = sd.base; seglen = sd.len; first = gr.first; count = gr.count; out_at = gr.out;
    } else {
        base = base0; seglen = len0; first = (uint64_t)g * WG;
        const uint64_t rem = nleaves0 - first;
        count = rem < (uint64_t)WG ? (uint32_t)rem : (uint32_t)WG;
        out_at = FUSE ? (uint64_t)g : first;
    }
    uint32_t st[8] = SENTRY_H0;
    if (tid < count) {
        const uint64_t start = (first + tid) * leaf_bytes;
        const uint64_t left = seglen - start;            // 0 only for the empty buffer's single leaf
        hash_leaf(st, base + start, left < leaf_bytes ? left : leaf_bytes);
    }
    if (!FUSE) {
        if (tid < count) store_digest(out + 32 * (out_at + tid), st);
        return;
    }
    __shared__ uint32_t lds[2][8][WG];
#pragma unroll
    for (int i = 0; i < 8; i++) lds[0][i][tid] = st[i];
    __syncthreads();
    uint32_t root[8];
    wg_tree_fold<WG>(lds, count, tid, root);
    if (tid == 0) store_digest(out + 32 * out_at, root);
    if constexpr (TAIL) {
        __shared__ uint32_t last;
        __shared__ uint32_t tail_lds[2][8][RED_IN];
        if (tail_ticket(ticket, tid, &last)) tail_fold<WG>(out, gridDim.x, final_out, ticket, tid, tail_lds);
    }
}

// Block hashing kernel for launches with very few leaves, where the run time is one lane's
// serial chain and most SIMDs idle.  A lone wave issues an instruction every five cycles or
// so whatever it does, so the only way to shorten the chain is to give it fewer instructions:
// two waves share each group of 64 leaves.  The producer wave loads the blocks, swaps bytes
// and expands the message schedule W[0..63] (which does not depend on the chaining value) into
// LDS; the consumer wave runs only the 64 rounds.  One barrier per block, two LDS slots:
// when the producer passes the barrier of block b+1 the consumer has finished block b, whose
// slot is the one the producer fills next.
constexpr int SPLIT_LEAVES = 64;
constexpr int SPLIT_PAIR_LANES = 128;                         // one producer wave + one consumer wave
constexpr uint64_t SPLIT_MIN_LEAF = 512;                      // below this the per-block barrier does not pay
constexpr int SPLIT_LANE_WORDS = 68;                          // 64 schedule words + 4 of padding:
constexpr int SPLIT_SLOT_WORDS = SPLIT_LEAVES * SPLIT_LANE_WORDS;   // 16-byte accesses stay conflict-free

// producer: schedule of one block into dst[0..63]; w is consumed
__device__ __forceinline__ void sha256_schedule_to_lds(uint32_t (&w)[16], uint32_t *dst)
{
    uint4 *d4 = reinterpret_cast<uint4 *>(dst);
#pragma unroll
    for (int g = 0; g < 4; g++) d4[g] = make_uint4(w[4 * g], w[4 * g + 1], w[4 * g + 2], w[4 * g + 3]);
#pragma unroll
    for (int t = 16; t < 64; t++) {
        w[t & 15] = w[t & 15] + ssig0(w[(t + 1) & 15]) + w[(t + 9) & 15] + ssig1(w[(t + 14) & 15]);
        if ((t & 3) == 3)
            d4[t >> 2] = make_uint4(w[(t - 3) & 15], w[(t - 2) & 15], w[(t - 1) & 15], w[t & 15]);
    }
}

// The consumer is alone on its SIMD, so nothing hides the latency of an LDS read that is
// issued right before its use, which is where the compiler puts them (eight stalls of a
// hundred cycles per block).  The reads are therefore spelled out and pinned: the words of
// rounds 8g+8 .. 8g+15 are requested before the arithmetic of rounds 8g .. 8g+7 and waited
// for after it.  `pin` passes through unchanged and ties the request to that place.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// `array` is not used by the instructions: naming the pointer tells the compiler that the
// statement reads the memory behind it, so that the stores that fill it stay.
__device__ __forceinline__ void lds_request_8_words(uint32_t lds_addr, const uint32_t *array, u32x4 &x0, u32x4 &x1,
                                                    uint32_t &pin)
{
    asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %3 offset:16"
                 : "=&v"(x0), "=&v"(x1), "+v"(pin)
                 : "v"(lds_addr), "v"(array)
                 : "memory");
}
__device__ __forceinline__ void lds_wait_8_words(u32x4 &x0, u32x4 &x1)
{
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x0), "+v"(x1));
}

// consumer: the 64 rounds over a schedule held in LDS; st is updated only where apply is set
__device__ __forceinline__ void sha256_rounds_from_lds(uint32_t (&st)[8], const uint32_t *src, bool apply)
{
    // LDS byte address of this lane's schedule: the low half of the flat address
    const uint32_t base = (uint32_t)reinterpret_cast<uintptr_t>(src);
    uint32_t v[8];
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = st[i];
    u32x4 c0, c1, n0 = {}, n1 = {};
    lds_request_8_words(base, src, c0, c1, v[0]);
#pragma unroll
    for (int g = 0; g < 8; g++) {
        lds_wait_8_words(c0, c1);
        if (g < 7) lds_request_8_words(base + 32u * (uint32_t)(g + 1), src, n0, n1, v[0]);
        const uint32_t w8[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const int t = 8 * g + k;
#define V(i) v[((i) - t) & 7]
            uint32_t t1 = V(7) + bsig1(V(4)) + ch(V(4), V(5), V(6)) + k256(t) + w8[k];
            V(3) += t1;
            V(7) = t1 + bsig0(V(0)) + maj(V(0), V(1), V(2));
#undef V
        }
        c0 = n0;
        c1 = n1;
    }
    if (apply) {
#pragma unroll
        for (int i = 0; i < 8; i++) st[i] += v[i];
    }
}

// A tree level of a launch that has more SIMDs than nodes is one node hash on a lone wave:
// two compressions, 2304 instructions, one after the other.  The message schedule of the first
// compression (480 of them) does not depend on the chaining value, so a second wave can expand it
// while the first runs the rounds, as for the leaves: the producer writes W[16..63] to LDS in six
// chunks of eight words, one barrier after each; the consumer starts with the sixteen words it holds
// (the two child digests), passes barrier k before the eight rounds that precede the use of chunk
// k, and requests chunk k right behind the barrier, so that the read's latency hides behind those
// rounds.  The producer needs 80 instructions per chunk, the consumer 112 per eight rounds, so the
// consumer never waits.  Its chain per node: 64 + 64 rounds and the reads, about 1850 instructions.
constexpr int TREE_LANE_WORDS = 52;                         // 48 schedule words + 4: 16-byte accesses stay conflict-free
constexpr int TREE_SLOT_WORDS = 64 * TREE_LANE_WORDS;       // one pair of waves
enum TreeRole { TREE_PRODUCER = 0, TREE_CONSUMER = 1, TREE_BYSTANDER = 2 };

__device__ __forceinline__ void sha256_eight_rounds(uint32_t (&v)[8], const uint32_t (&w8)[8], int t0)
{
#pragma unroll
    for (int k = 0; k < 8; k++) {
        const int t = t0 + k;
#define V(i) v[((i) - t) & 7]
        uint32_t t1 = V(7) + bsig1(V(4)) + ch(V(4), V(5), V(6)) + k256(t) + w8[k];
        V(3) += t1;
        V(7) = t1 + bsig0(V(0)) + maj(V(0), V(1), V(2));
#undef V
    }
}

// out = SHA-256(l || r), computed by the consumer wave with the producer wave's help.  Every wave of
// the workgroup calls this at the same point; the six barriers stand outside the role-dependent
// parts, so that every wave executes exactly six whatever its role.  The lanes of producer and
// consumer with the same lane number hold the same l, r and the same slot (LDS, TREE_LANE_WORDS
// words).  Only the consumer's out is defined.
__device__ __forceinline__ void node_hash_split(int role, const uint32_t (&l)[8], const uint32_t (&r)[8], uint32_t *slot,
                                                uint32_t (&out)[8])
{
    const bool producer = role == TREE_PRODUCER, consumer = role == TREE_CONSUMER;
    const uint32_t base = (uint32_t)reinterpret_cast<uintptr_t>(slot);   // LDS byte address of this lane's slot
    uint4 *s4 = reinterpret_cast<uint4 *>(slot);
    uint32_t w[16] = {};
    uint32_t v[8] = SENTRY_H0;
    u32x4 c0 = {}, c1 = {}, n0 = {}, n1 = {};
    // producer: chunk g = W[16 + 8g .. 23 + 8g] into the slot
    auto chunk = [&](int g) {
#pragma unroll
        for (int t = 16 + 8 * g; t < 24 + 8 * g; t++)
            w[t & 15] = w[t & 15] + ssig0(w[(t + 1) & 15]) + w[(t + 9) & 15] + ssig1(w[(t + 14) & 15]);
        const int b = (8 * g) & 15;                     // W[16 + 8g + k] sits in w[(8g + k) & 15]
        s4[2 * g] = make_uint4(w[b], w[b + 1], w[b + 2], w[b + 3]);
        s4[2 * g + 1] = make_uint4(w[b + 4], w[b + 5], w[b + 6], w[b + 7]);
    };
    if (producer) {
#pragma unroll
        for (int i = 0; i < 8; i++) { w[i] = l[i]; w[8 + i] = r[i]; }
        chunk(0);
    }
    if (consumer) sha256_eight_rounds(v, l, 0);
    __syncthreads();                                    // chunk 0 is in LDS
    if (producer) chunk(1);
    if (consumer) {
        lds_request_8_words(base, slot, c0, c1, v[0]);
        sha256_eight_rounds(v, r, 8);
        lds_wait_8_words(c0, c1);
    }
    __syncthreads();                                    // chunk 1
#pragma unroll
    for (int g = 1; g < 5; g++) {
        if (producer) chunk(g + 1);
        if (consumer) {
            lds_request_8_words(base + 32u * (uint32_t)g, slot, n0, n1, v[0]);
            const uint32_t w8[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
            sha256_eight_rounds(v, w8, 8 + 8 * g);
            lds_wait_8_words(n0, n1);
            c0 = n0;
            c1 = n1;
        }
        __syncthreads();                                // chunk g + 1
    }
    if (consumer) {
        lds_request_8_words(base + 32u * 5u, slot, n0, n1, v[0]);
        const uint32_t w8[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        sha256_eight_rounds(v, w8, 48);
        lds_wait_8_words(n0, n1);
        const uint32_t x8[8] = {n0.x, n0.y, n0.z, n0.w, n1.x, n1.y, n1.z, n1.w};
        sha256_eight_rounds(v, x8, 56);
        uint32_t st[8] = SENTRY_H0;
#pragma unroll
        for (int i = 0; i < 8; i++) st[i] += v[i];
        sha256_compress_pad64(st);
#pragma unroll
        for (int i = 0; i < 8; i++) out[i] = st[i];
    }
}

// tail_fold for workgroups of two or four waves: wave 0 is the producer and wave 1 the consumer of
// every node hash, 64 nodes of a level per trip.  t = LDS, 2 x 8 x 512 words; slots = LDS,
// TREE_SLOT_WORDS words.
template <int NT>
__device__ __forceinline__ void tail_fold_split(const uint8_t *nodes, uint32_t cnt, uint8_t *out, uint32_t *ticket,
                                                uint32_t tid, uint32_t (*t)[8][RED_IN], uint32_t *slots)
{
    for (uint32_t i = tid; i < cnt; i += NT) {
        uint32_t d[8];
        load_digest(nodes + 32 * (uint64_t)i, d);
#pragma unroll
        for (int k = 0; k < 8; k++) t[0][k][i] = d[k];
    }
    __syncthreads();
    const uint32_t lane = tid & 63, wave = tid >> 6;
    const int role = wave == 0 ? TREE_PRODUCER : wave == 1 ? TREE_CONSUMER : TREE_BYSTANDER;
    uint32_t *slot = slots + lane * TREE_LANE_WORDS;
    int cur = 0;
#pragma unroll 1
    while (cnt > 1) {
        const uint32_t pairs = cnt >> 1;
#pragma unroll 1
        for (uint32_t first = 0; first < pairs; first += 64) {
            const uint32_t i = first + lane;
            const bool act = i < pairs;
            const uint32_t at = act ? i : 0;
            uint32_t l[8], r[8], d[8];
            if (role != TREE_BYSTANDER) {
#pragma unroll
                for (int k = 0; k < 8; k++) { l[k] = t[cur][k][2 * at]; r[k] = t[cur][k][2 * at + 1]; }
            }
            node_hash_split(role, l, r, slot, d);
            if (role == TREE_CONSUMER && act) {
#pragma unroll
                for (int k = 0; k < 8; k++) t[cur ^ 1][k][i] = d[k];
            }
        }
        if (tid == 0 && (cnt & 1)) {
#pragma unroll
            for (int k = 0; k < 8; k++) t[cur ^ 1][k][pairs] = t[cur][k][cnt - 1];
        }
        __syncthreads();
        cnt = pairs + (cnt & 1);
        cur ^= 1;
    }
    if (tid == 0) {
        uint32_t root[8];
#pragma unroll
        for (int k = 0; k < 8; k++) root[k] = t[cur][k][0];
        store_digest(out, root);
        *ticket = 0;          // ready for the next launch
    }
}

// Workgroup = 256 lanes = two producer/consumer pairs (waves P0, C0, P1, C1), each pair with
// its own group of 64 leaves.  Four waves of one workgroup land on the four SIMDs of a CU,
// one each, which single- or two-wave workgroups do not guarantee once a CU holds two of
// them; with at most one workgroup per CU every wave of the launch has a SIMD to itself.
// All barriers are workgroup-wide, so both pairs run the trip count of the longer group.
// PAIRS = 1 (128 lanes) is used while there is at most one group per CU: two busy SIMDs per
// CU run a little faster than four.
// TAIL (with FUSE, one buffer): the one-launch tree; `out` holds n_groups nodes, root to final_out.
template <int PAIRS, bool FUSE, bool SEGMENTED, bool PACKED = false, bool TAIL = false>
__global__ void __launch_bounds__(SPLIT_PAIR_LANES * PAIRS)
merkle_leaf_split_kernel(const uint8_t *base0, uint64_t len0, uint64_t nleaves0, uint32_t n_groups,
                         const SegDesc *segs, uint32_t n_seg, const Group *groups, uint64_t leaf_bytes, uint8_t *out,
                         uint32_t *ticket = nullptr, uint8_t *final_out = nullptr)
{
    static_assert(!PACKED || (SEGMENTED && !FUSE), "the packed leaf stage writes leaf digests");
    static_assert(!TAIL || (FUSE && !SEGMENTED && !PACKED), "the one-launch tree is for one buffer");
    static_assert(2 * SPLIT_SLOT_WORDS >= TREE_SLOT_WORDS, "the tree levels use the schedule slots of their pair");
    __shared__ __attribute__((aligned(16))) uint32_t sched[PAIRS][2 * SPLIT_SLOT_WORDS];
    __shared__ uint32_t lds[PAIRS][2][8][SPLIT_LEAVES];
    __shared__ unsigned long long trip_share[2 * PAIRS];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t pr = wave >> 1;
    const bool consumer = wave & 1;
    const uint32_t g = PAIRS * blockIdx.x + pr;
    const uint8_t *base = nullptr;
    uint64_t seglen = 0, first = 0, out_at = 0;
    uint32_t count = 0;
    if (g < n_groups) {
        if (PACKED || !SEGMENTED) {
            base = base0; seglen = len0; first = (uint64_t)g * SPLIT_LEAVES;
            const uint64_t rem = nleaves0 - first;
            count = rem < (uint64_t)SPLIT_LEAVES ? (uint32_t)rem : (uint32_t)SPLIT_LEAVES;
            out_at = FUSE ? (uint64_t)g : first;
        } else {
            const Group gr = groups[g];
            const SegDesc sd = segs[gr.seg];
            base = sd.base; seglen = sd.len; first = gr.first; count = gr.count; out_at = gr.out;
        }
    }
    const bool have = lane < count;
    uint64_t llen = 0;
    const uint8_t *p = base;
    if (have) {
        if (PACKED) {
            const PackedLeaf pl = find_packed_leaf(segs, n_seg, first + lane, leaf_bytes);
            p = pl.p; llen = pl.len;
        } else {
            const uint64_t start = (first + lane) * leaf_bytes;
            const uint64_t left = seglen - start;
            llen = left < leaf_bytes ? left : leaf_bytes;
            p = base + start;
        }
    }
    const uint64_t nblk = llen >> 6;
    const uint32_t r = (uint32_t)(llen & 63);
    const uint64_t total = have ? nblk + 1 + (r >= 56 ? 1 : 0) : 0;
    // the longest leaf of the group (lane 0 holds it unless the group is packed from several
    // segments); the larger of the two groups' block counts is the trip count of all four waves
    uint64_t longest = total;
    if (PACKED) {
#pragma unroll
        for (int d = 32; d; d >>= 1) {
            const uint64_t o = __shfl_xor(longest, d, 64);
            longest = o > longest ? o : longest;
        }
    }
    if (lane == 0) trip_share[wave] = longest;
    __syncthreads();
    uint64_t trips = trip_share[0];
    if (PAIRS == 2 && trip_share[2] > trips) trips = trip_share[2];
    uint32_t *my = &sched[pr][lane * SPLIT_LANE_WORDS];
    uint32_t st[8] = SENTRY_H0;

    if (!consumer) {
        // two pairs of blocks (two 128-byte lines) are in flight per lane: the producer is short
        // of work, not of registers
        const uint4 *q = reinterpret_cast<const uint4 *>(p);
        uint4 c[16] = {};
#pragma unroll
        for (int k = 0; k < 4; k++) {
            if (nblk >= (uint64_t)(k + 1)) {
                c[4 * k] = q[4 * k]; c[4 * k + 1] = q[4 * k + 1]; c[4 * k + 2] = q[4 * k + 2]; c[4 * k + 3] = q[4 * k + 3];
            }
        }
        for (uint64_t b = 0; b < trips; b++) {
            uint32_t w[16];
            if (b < nblk) {
                const uint32_t slot = (uint32_t)b & 3;
                if (slot == 0) bswap_block(w, c[0], c[1], c[2], c[3]);
                else if (slot == 1) bswap_block(w, c[4], c[5], c[6], c[7]);
                else if (slot == 2) bswap_block(w, c[8], c[9], c[10], c[11]);
                else bswap_block(w, c[12], c[13], c[14], c[15]);
                if (slot & 1) {   // a pair is used up: refill it with blocks b+3 and b+4
                    const uint4 *n = q + 4 * (b + 3);
                    if (slot == 1) {
                        if (b + 3 < nblk) { c[0] = n[0]; c[1] = n[1]; c[2] = n[2]; c[3] = n[3]; }
                        if (b + 4 < nblk) { c[4] = n[4]; c[5] = n[5]; c[6] = n[6]; c[7] = n[7]; }
                    } else {
                        if (b + 3 < nblk) { c[8] = n[0]; c[9] = n[1]; c[10] = n[2]; c[11] = n[3]; }
                        if (b + 4 < nblk) { c[12] = n[4]; c[13] = n[5]; c[14] = n[6]; c[15] = n[7]; }
                    }
                }
            } else if (b < total) {
                build_tail(w, p + (nblk << 6), r, llen, (uint32_t)(b - nblk));
            } else {
#pragma unroll
                for (int i = 0; i < 16; i++) w[i] = 0;   // this lane's leaf is done; the slot is not used
            }
            sha256_schedule_to_lds(w, my + (b & 1) * SPLIT_SLOT_WORDS);
            __syncthreads();
        }
    } else {
        for (uint64_t b = 0; b < trips; b++) {
            __syncthreads();
            sha256_rounds_from_lds(st, my + (b & 1) * SPLIT_SLOT_WORDS, b < total);
        }
    }
    if (!FUSE) {
        if (consumer && have) store_digest(out + 32 * (out_at + lane), st);
        return;
    }
    // each consumer wave folds its 64 leaf digests; six levels for everybody keeps the
    // barriers of the two pairs in step
    if (consumer) {
#pragma unroll
        for (int i = 0; i < 8; i++) lds[pr][0][i][lane] = st[i];
    }
    __syncthreads();
    // the schedule slots are free now: the producer wave of each pair expands the message schedules of
    // the node hashes there while the consumer wave runs their rounds (node_hash_split)
    uint32_t *tree_slot = &sched[pr][lane * TREE_LANE_WORDS];
    uint32_t cnt = count;
    int cur = 0;
#pragma unroll 1
    for (int level = 0; level < 6; level++) {
        const uint32_t pairs = cnt >> 1;
        const bool work = cnt > 1;                       // the same for both waves of a pair
        const bool act = work && lane < pairs;
        const uint32_t at = act ? lane : 0;
        uint32_t l[8], rr[8], d[8];
        if (work) {
#pragma unroll
            for (int i = 0; i < 8; i++) { l[i] = lds[pr][cur][i][2 * at]; rr[i] = lds[pr][cur][i][2 * at + 1]; }
        }
        node_hash_split(work ? (consumer ? TREE_CONSUMER : TREE_PRODUCER) : TREE_BYSTANDER, l, rr, tree_slot, d);
        if (consumer && work) {
            if (act) {
#pragma unroll
                for (int i = 0; i < 8; i++) lds[pr][cur ^ 1][i][lane] = d[i];
            } else if (lane == pairs && (cnt & 1)) {
#pragma unroll
                for (int i = 0; i < 8; i++) lds[pr][cur ^ 1][i][pairs] = lds[pr][cur][i][cnt - 1];
            }
        }
        __syncthreads();
        if (cnt > 1) { cnt = pairs + (cnt & 1); cur ^= 1; }
    }
    if (consumer && lane == 0 && g < n_groups) {
        uint32_t root[8];
#pragma unroll
        for (int i = 0; i < 8; i++) root[i] = lds[pr][cur][i][0];
        store_digest(out + 32 * out_at, root);
        if constexpr (TAIL) __threadfence();   // released by the lane that stored it
    }
    if constexpr (TAIL) {
        // the schedule slots of pair 0 are free now (tail_ticket starts with a barrier)
        __shared__ uint32_t last;
        __shared__ uint32_t tail_nodes[2][8][RED_IN];
        if (tail_ticket(ticket, threadIdx.x, &last))
            tail_fold_split<SPLIT_PAIR_LANES * PAIRS>(out, n_groups, final_out, ticket, threadIdx.x, tail_nodes, &sched[0][0]);
    }
}

// Reduction kernel: each workgroup folds up to 512 consecutive nodes of one segment into one.
template <bool SEGMENTED>
__global__ void __launch_bounds__(RED_WG)
merkle_reduce_kernel(const uint8_t *in, uint64_t n0, const Group *groups, uint8_t *out)
{
    const uint32_t g = blockIdx.x, tid = threadIdx.x;
    uint64_t first;
    uint32_t count;
    if (SEGMENTED) {
        const Group gr = groups[g];
        first = gr.first; count = gr.count;
    } else {
        first = (uint64_t)g * RED_IN;
        const uint64_t rem = n0 - first;
        count = rem < (uint64_t)RED_IN ? (uint32_t)rem : (uint32_t)RED_IN;
    }
    __shared__ uint32_t lds[2][8][RED_WG];
    const uint32_t pairs = count >> 1;
    if (tid < pairs) {
        uint32_t l[8], r[8], d[8];
        load_digest(in + 32 * (first + 2 * tid), l);
        load_digest(in + 32 * (first + 2 * tid + 1), r);
        node_hash(l, r, d);
#pragma unroll
        for (int i = 0; i < 8; i++) lds[0][i][tid] = d[i];
    } else if (tid == pairs && (count & 1)) {
        uint32_t d[8];
        load_digest(in + 32 * (first + count - 1), d);
#pragma unroll
        for (int i = 0; i < 8; i++) lds[0][i][tid] = d[i];
    }
    __syncthreads();
    uint32_t root[8];
    wg_tree_fold<RED_WG>(lds, pairs + (count & 1), tid, root);
    if (tid == 0) store_digest(out + 32 * (uint64_t)g, root);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// the two-wave split kernel over n_groups groups of 64 leaves
template <bool FUSE, bool SEGMENTED, bool PACKED = false, bool TAIL = false>
void launch_split(uint32_t n_groups, hipStream_t s, const uint8_t *base0, uint64_t len0, uint64_t nleaves0,
                  const SegDesc *segs, uint32_t n_seg, const Group *groups, uint64_t leaf_bytes, uint8_t *out,
                  uint32_t *ticket = nullptr, uint8_t *final_out = nullptr)
{
    if (n_groups <= SPLIT_SINGLE_GROUPS)
        hipLaunchKernelGGL((merkle_leaf_split_kernel<1, FUSE, SEGMENTED, PACKED, TAIL>), dim3(n_groups),
                           dim3(SPLIT_PAIR_LANES), 0, s, base0, len0, nleaves0, n_groups, segs, n_seg, groups, leaf_bytes,
                           out, ticket, final_out);
    else
        hipLaunchKernelGGL((merkle_leaf_split_kernel<2, FUSE, SEGMENTED, PACKED, TAIL>), dim3((n_groups + 1) / 2),
                           dim3(2 * SPLIT_PAIR_LANES), 0, s, base0, len0, nleaves0, n_groups, segs, n_seg, groups,
                           leaf_bytes, out, ticket, final_out);
}

// The packed leaf stage pays where per-segment groups would leave at least a ninth of the
// waves' lanes without a leaf (waves = groups of 64 when every segment starts its own).
inline bool packed_leaf_stage(uint64_t waves, uint64_t total_leaves)
{
    const uint64_t full = ceil_div(total_leaves, 64);
    return waves - full >= ceil_div(full, 8);
}

inline uint64_t leaf_count(uint64_t len, uint64_t leaf_bytes)
{
    uint64_t n = ceil_div(len, leaf_bytes);
    return n ? n : 1;
}

// a launch holds fewer than 2^32 work-items in all (grid x workgroup size)
constexpr uint64_t MAX_GRID = 0xffffffffull / 256;

int check_leaf_args(const char *fn, const void *buf, size_t len, size_t leaf_bytes)
{
    SENTRY_REQUIRE(leaf_bytes > 0 && leaf_bytes % 64 == 0,
                   "%s: leaf_bytes must be a positive multiple of 64 (got %zu)", fn, leaf_bytes);
    SENTRY_REQUIRE(buf != nullptr || len == 0, "%s: NULL buffer with len %zu", fn, len);
    SENTRY_REQUIRE((reinterpret_cast<uintptr_t>(buf) & 15) == 0, "%s: buffer %p is not 16-byte aligned", fn, buf);
    const uint64_t n_leaves = leaf_count(len, leaf_bytes);
    SENTRY_REQUIRE(ceil_div(n_leaves, single_wave_groups(ceil_div(n_leaves, 64), leaf_bytes) ? LEAF_WG_SMALL : LEAF_WG) <= MAX_GRID,
                   "%s: too many leaves", fn);
    return SENTRY_OK;
}

// Reduce n nodes at `in` (device, 16-byte aligned) to one digest at out_digest; intermediate
// levels ping-pong between red0 and red1 (device, 16-byte aligned, 32 * ceil(n / 512) bytes each,
// distinct from `in`; not touched when n <= 512).
int reduce_nodes_in(const uint8_t *in, uint64_t n, uint8_t *out_digest, hipStream_t s, uint8_t *red0, uint8_t *red1)
{
    const uint8_t *src = in;
    uint8_t *bufs[2] = {red0, red1};
    uint64_t m = n;
    int turn = 0;
    do {   // at least one pass so that the result lands in out_digest
        const uint64_t g = ceil_div(m, RED_IN);
        uint8_t *dst = g == 1 ? out_digest : bufs[turn];
        hipLaunchKernelGGL(merkle_reduce_kernel<false>, dim3((uint32_t)g), dim3(RED_WG), 0, s, src, m,
                           (const Group *)nullptr, dst);
        SENTRY_HIP_CHECK(hipGetLastError());
        src = dst;
        m = g;
        turn ^= 1;
    } while (m > 1);
    return SENTRY_OK;
}

// The same with the level buffers taken from the two R_RED regions of the stream's scratch
// (`in` is not one of them).
int reduce_nodes(const uint8_t *in, uint64_t n, uint8_t *out_digest, hipStream_t s)
{
    void *a = nullptr, *b = nullptr;
    if (n > RED_IN) {   // the first pass is the largest
        const uint64_t g = ceil_div(n, RED_IN);
        int rc = sentry::scratch_get(s, sentry::R_RED_0, 32 * g, &a);
        if (rc) return rc;
        if ((rc = sentry::scratch_get(s, sentry::R_RED_1, 32 * g, &b))) return rc;
    }
    return reduce_nodes_in(in, n, out_digest, s, static_cast<uint8_t *>(a), static_cast<uint8_t *>(b));
}

// How sentry_merkle_root cuts a buffer into workgroups, and the scratch that needs.
struct RootPlan {
    uint64_t leaves, groups;   // groups = workgroups of the leaf kernel = nodes it writes
    bool small;                // single-wave workgroups of 64 leaves (else 256)
    bool split;                // the two-wave producer/consumer kernel
    bool tail;                 // 2 .. 512 groups: the last workgroup folds the nodes, one launch in all
};

RootPlan plan_root(uint64_t len, uint64_t leaf_bytes)
{
    RootPlan p;
    p.leaves = leaf_count(len, leaf_bytes);
    p.small = single_wave_groups(ceil_div(p.leaves, 64), leaf_bytes);
    p.groups = ceil_div(p.leaves, p.small ? LEAF_WG_SMALL : LEAF_WG);
    p.split = p.small && p.groups <= SPLIT_LAUNCH_WAVES && leaf_bytes >= SPLIT_MIN_LEAF;
    p.tail = p.small && p.groups > 1 && p.groups <= RED_IN;
    return p;
}

// nodes: 32 * groups bytes (not used for one group); ticket: one zeroed word (tail plans only);
// red0, red1: 32 * ceil(groups / 512) bytes each (plans with more than 512 groups only)
struct RootScratch {
    uint8_t *nodes;
    uint32_t *ticket;
    uint8_t *red0, *red1;
};

__global__ void zero_words_kernel(uint32_t *p, uint32_t n)
{
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

int merkle_root_launch(const RootPlan &plan, const void *dev_buf, uint64_t len, uint64_t leaf_bytes, uint8_t *out_digest,
                       hipStream_t s, const RootScratch &sc)
{
    const uint8_t *buf = static_cast<const uint8_t *>(dev_buf);
    const uint32_t g = (uint32_t)plan.groups;
    uint8_t *dst = g > 1 ? sc.nodes : out_digest;
    if (plan.tail) {
        if (plan.split)
            launch_split<true, false, false, true>(g, s, buf, len, plan.leaves, nullptr, 0, nullptr, leaf_bytes, dst,
                                                   sc.ticket, out_digest);
        else
            hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG_SMALL, true, false, false, true>), dim3(g), dim3(LEAF_WG_SMALL),
                               0, s, buf, len, plan.leaves, (const SegDesc *)nullptr, 0u, (const Group *)nullptr,
                               leaf_bytes, dst, sc.ticket, out_digest);
        SENTRY_HIP_CHECK(hipGetLastError());
        return SENTRY_OK;
    }
    if (plan.split)
        launch_split<true, false>(g, s, buf, len, plan.leaves, nullptr, 0, nullptr, leaf_bytes, dst);
    else if (plan.small)
        hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG_SMALL, true, false>), dim3(g), dim3(LEAF_WG_SMALL), 0, s, buf, len,
                           plan.leaves, (const SegDesc *)nullptr, 0u, (const Group *)nullptr, leaf_bytes, dst);
    else
        hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG, true, false>), dim3(g), dim3(LEAF_WG), 0, s, buf, len,
                           plan.leaves, (const SegDesc *)nullptr, 0u, (const Group *)nullptr, leaf_bytes, dst);
    SENTRY_HIP_CHECK(hipGetLastError());
    if (g > 1) return reduce_nodes_in(dst, g, out_digest, s, sc.red0, sc.red1);
    return SENTRY_OK;
}

// ---------------------------------------------------------------------------
// sentry_merkle_root_noalloc: the same launches with their scratch in a fixed device array
// ---------------------------------------------------------------------------

constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex g_noalloc_mu;
unsigned char *g_noalloc_ptr[NOALLOC_MAX_DEVICES] = {};

// Device address of `scratch` on the current device, looked up once per device.
int noalloc_scratch(unsigned char **out)
{
    int dev = 0;
    SENTRY_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) {
        sentry::set_error("sentry_merkle_root_noalloc: device %d is beyond the %d devices supported", dev, NOALLOC_MAX_DEVICES);
        return SENTRY_ERR_INVALID_ARG;
    }
    std::lock_guard<std::mutex> lock(g_noalloc_mu);
    if (!g_noalloc_ptr[dev]) {
        unsigned char *ptr = nullptr;
        SENTRY_HIP_CHECK(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) {
            sentry::set_error("sentry_merkle_root_noalloc: no device address for the scratch array on device %d", dev);
            return SENTRY_ERR_HIP;
        }
        g_noalloc_ptr[dev] = ptr;
    }
    *out = g_noalloc_ptr[dev];
    return SENTRY_OK;
}

}  // namespace

namespace sentry {

// Leaf digests of a device chunk into dst (32 bytes per leaf), used by the streaming paths.
// Scratch for every sentry_merkle_root, sentry_merkle_leaves and sentry_merkle_reduce call on s whose
// input has at most max_len bytes in leaves of leaf_bytes: the node buffer for the smallest
// workgroups any such input gets (64 leaves), the level buffers of the reduction over that many
// nodes, and the ticket counter of the one-launch tree, cleared.
int merkle_reserve(uint64_t max_len, uint64_t leaf_bytes, hipStream_t s)
{
    const uint64_t leaves = leaf_count(max_len, leaf_bytes);
    const uint64_t groups = ceil_div(leaves, LEAF_WG_SMALL);
    void *p;
    int rc;
    bool fresh;
    if ((rc = scratch_get(s, R_NODES_A, 32 * groups, &p))) return rc;
    // sentry_merkle_reduce may be given all the leaf digests: its first level has leaves / 512 nodes
    if ((rc = scratch_get(s, R_RED_0, 32 * ceil_div(leaves, RED_IN), &p))) return rc;
    if ((rc = scratch_get(s, R_RED_1, 32 * ceil_div(leaves, RED_IN), &p))) return rc;
    if ((rc = scratch_get_fresh(s, R_TICKET, 256, &p, &fresh))) return rc;
    if (fresh) {
        hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, s, static_cast<uint32_t *>(p), 64u);
        SENTRY_HIP_CHECK(hipGetLastError());
    }
    return SENTRY_OK;
}

int merkle_leaves_into(const void *dev_buf, size_t len, size_t leaf_bytes, uint8_t *dst, hipStream_t s)
{
    const uint64_t n = leaf_count(len, leaf_bytes);
    if (ceil_div(n, 64) <= SPLIT_LAUNCH_WAVES && leaf_bytes >= SPLIT_MIN_LEAF)
        launch_split<false, false>((uint32_t)ceil_div(n, SPLIT_LEAVES), s, static_cast<const uint8_t *>(dev_buf),
                                   (uint64_t)len, n, nullptr, 0, nullptr, (uint64_t)leaf_bytes, dst);
    else if (single_wave_groups(ceil_div(n, 64), leaf_bytes))
        hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG_SMALL, false, false>), dim3((uint32_t)ceil_div(n, LEAF_WG_SMALL)),
                           dim3(LEAF_WG_SMALL), 0, s, static_cast<const uint8_t *>(dev_buf), (uint64_t)len, n,
                           (const SegDesc *)nullptr, 0u, (const Group *)nullptr, (uint64_t)leaf_bytes, dst);
    else
        hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG, false, false>), dim3((uint32_t)ceil_div(n, LEAF_WG)),
                           dim3(LEAF_WG), 0, s, static_cast<const uint8_t *>(dev_buf), (uint64_t)len, n,
                           (const SegDesc *)nullptr, 0u, (const Group *)nullptr, (uint64_t)leaf_bytes, dst);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

int merkle_reduce_into(const uint8_t *dev_nodes, uint64_t n, uint8_t *out_digest, hipStream_t s)
{
    return reduce_nodes(dev_nodes, n, out_digest, s);
}

}  // namespace sentry

extern "C" {

int sentry_merkle_root(const void *dev_buf, size_t len, size_t leaf_bytes, uint8_t *out_digest, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = check_leaf_args("sentry_merkle_root", dev_buf, len, leaf_bytes);
    if (rc) return rc;
    SENTRY_REQUIRE(out_digest != nullptr, "sentry_merkle_root: NULL out_digest");
    const RootPlan plan = plan_root(len, leaf_bytes);
    RootScratch sc = {};
    if (plan.groups > 1) {
        void *p;
        if ((rc = sentry::scratch_get(s, sentry::R_NODES_A, 32 * plan.groups, &p))) return rc;
        sc.nodes = static_cast<uint8_t *>(p);
    }
    if (plan.tail) {
        void *p;
        bool fresh;
        if ((rc = sentry::scratch_get_fresh(s, sentry::R_TICKET, 256, &p, &fresh))) return rc;
        sc.ticket = static_cast<uint32_t *>(p);
        if (fresh) {   // from then on the last workgroup of every launch leaves it at zero
            hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, s, sc.ticket, 64u);
            SENTRY_HIP_CHECK(hipGetLastError());
        }
    } else if (plan.groups > RED_IN) {
        void *a, *b;
        const uint64_t g1 = ceil_div(plan.groups, RED_IN);
        if ((rc = sentry::scratch_get(s, sentry::R_RED_0, 32 * g1, &a))) return rc;
        if ((rc = sentry::scratch_get(s, sentry::R_RED_1, 32 * g1, &b))) return rc;
        sc.red0 = static_cast<uint8_t *>(a);
        sc.red1 = static_cast<uint8_t *>(b);
    }
    return merkle_root_launch(plan, dev_buf, len, leaf_bytes, out_digest, s, sc);
}

int sentry_merkle_root_noalloc(const void *dev_buf, size_t len, size_t leaf_bytes, uint8_t *out_digest, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = check_leaf_args("sentry_merkle_root_noalloc", dev_buf, len, leaf_bytes);
    if (rc) return rc;
    SENTRY_REQUIRE(out_digest != nullptr, "sentry_merkle_root_noalloc: NULL out_digest");
    const RootPlan plan = plan_root(len, leaf_bytes);
    SENTRY_REQUIRE(plan.leaves <= NOALLOC_MAX_LEAVES,
                   "sentry_merkle_root_noalloc: %llu leaves, the fixed scratch holds at most %llu (use sentry_merkle_root)",
                   (unsigned long long)plan.leaves, (unsigned long long)NOALLOC_MAX_LEAVES);
    unsigned char *ptr;
    if ((rc = noalloc_scratch(&ptr))) return rc;
    RootScratch sc;
    sc.nodes = ptr;
    sc.red0 = ptr + NOALLOC_NODES_BYTES;
    sc.red1 = sc.red0 + NOALLOC_RED_BYTES;
    sc.ticket = reinterpret_cast<uint32_t *>(ptr + NOALLOC_TICKET_AT);
    if (plan.tail) {
        // the array keeps what the last call left: the ticket must start at zero (a fill kernel, so
        // that the call can be captured into a graph)
        hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, s, sc.ticket, 64u);
        SENTRY_HIP_CHECK(hipGetLastError());
    }
    return merkle_root_launch(plan, dev_buf, len, leaf_bytes, out_digest, s, sc);
}

int sentry_merkle_leaves(const void *dev_buf, size_t len, size_t leaf_bytes, uint8_t *out_leaf_digests, void *stream)
{
    sentry::clear_error();
    int rc = check_leaf_args("sentry_merkle_leaves", dev_buf, len, leaf_bytes);
    if (rc) return rc;
    SENTRY_REQUIRE(out_leaf_digests != nullptr && (reinterpret_cast<uintptr_t>(out_leaf_digests) & 15) == 0,
                   "sentry_merkle_leaves: out_leaf_digests must be non-NULL and 16-byte aligned");
    return sentry::merkle_leaves_into(dev_buf, len, leaf_bytes, out_leaf_digests, static_cast<hipStream_t>(stream));
}

int sentry_merkle_reduce(const uint8_t *dev_nodes, size_t n, uint8_t *out_digest, void *stream)
{
    sentry::clear_error();
    SENTRY_REQUIRE(n >= 1, "sentry_merkle_reduce: n must be at least 1");
    SENTRY_REQUIRE(dev_nodes != nullptr && (reinterpret_cast<uintptr_t>(dev_nodes) & 15) == 0,
                   "sentry_merkle_reduce: dev_nodes must be non-NULL and 16-byte aligned");
    SENTRY_REQUIRE(out_digest != nullptr, "sentry_merkle_reduce: NULL out_digest");
    SENTRY_REQUIRE(ceil_div(n, RED_IN) <= MAX_GRID, "sentry_merkle_reduce: too many nodes");
    return reduce_nodes(dev_nodes, n, out_digest, static_cast<hipStream_t>(stream));
}

int sentry_merkle_segments(const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes,
                           uint8_t *out_seg_roots, uint8_t *out_root, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(n_seg >= 1, "sentry_merkle_segments: n_seg must be at least 1");
    SENTRY_REQUIRE(dev_ptrs && lens && out_root, "sentry_merkle_segments: NULL argument");
    SENTRY_REQUIRE(leaf_bytes > 0 && leaf_bytes % 64 == 0,
                   "sentry_merkle_segments: leaf_bytes must be a positive multiple of 64 (got %zu)", leaf_bytes);
    for (size_t t = 0; t < n_seg; t++) {
        SENTRY_REQUIRE(dev_ptrs[t] != nullptr || lens[t] == 0, "sentry_merkle_segments: segment %zu is NULL", t);
        SENTRY_REQUIRE((reinterpret_cast<uintptr_t>(dev_ptrs[t]) & 15) == 0,
                       "sentry_merkle_segments: segment %zu is not 16-byte aligned", t);
    }
    SENTRY_REQUIRE(n_seg <= 0xffffffffull, "sentry_merkle_segments: too many segments");

    // Stage tables, built on the host: stage 0 splits every segment's leaves into groups of 256
    // (or 64), each folded to one node by its workgroup; or, where that would leave many groups
    // part-filled, stage 0 is packed (one leaf per lane across segments, leaf digests written out).
    // Each later stage splits every segment's nodes into groups of 512, until every segment is
    // down to one node.
    std::vector<std::vector<Group>> stages;
    std::vector<uint64_t> m(n_seg);   // nodes per segment after the current stage
    uint64_t waves = 0, total_leaves = 0;
    for (size_t t = 0; t < n_seg; t++) {
        const uint64_t nl = leaf_count(lens[t], leaf_bytes);
        waves += ceil_div(nl, 64);
        total_leaves += nl;
    }
    const bool packed = packed_leaf_stage(waves, total_leaves);
    if (packed) waves = ceil_div(total_leaves, 64);
    const bool small = single_wave_groups(waves, leaf_bytes);
    const uint64_t wg0 = small ? LEAF_WG_SMALL : LEAF_WG;
    {
        std::vector<Group> g0;
        for (size_t t = 0; t < n_seg; t++) {
            const uint64_t nl = leaf_count(lens[t], leaf_bytes);
            if (packed) {
                m[t] = nl;
                continue;
            }
            for (uint64_t f = 0; f < nl; f += wg0)
                g0.push_back(Group{f, (uint64_t)g0.size(), (uint32_t)(nl - f < wg0 ? nl - f : wg0), (uint32_t)t});
            m[t] = ceil_div(nl, wg0);
        }
        stages.push_back(std::move(g0));
    }
    const uint64_t grid0 = packed ? ceil_div(total_leaves, wg0) : stages[0].size();
    const uint64_t nodes0 = packed ? total_leaves : stages[0].size();   // digests stage 0 writes
    SENTRY_REQUIRE(grid0 <= MAX_GRID, "sentry_merkle_segments: too many leaves");
    for (;;) {
        bool more = false;
        for (size_t t = 0; t < n_seg; t++) more |= m[t] > 1;
        if (!more) break;
        std::vector<Group> gs;
        uint64_t node0 = 0;
        for (size_t t = 0; t < n_seg; t++) {
            for (uint64_t f = 0; f < m[t]; f += RED_IN)
                gs.push_back(Group{node0 + f, (uint64_t)gs.size(), (uint32_t)(m[t] - f < RED_IN ? m[t] - f : RED_IN), (uint32_t)t});
            node0 += m[t];
            m[t] = ceil_div(m[t], RED_IN);
        }
        stages.push_back(std::move(gs));
    }
    size_t table_bytes = n_seg * sizeof(SegDesc);
    for (auto &st : stages) {
        SENTRY_REQUIRE(st.size() <= MAX_GRID, "sentry_merkle_segments: too many leaves");
        table_bytes += st.size() * sizeof(Group);
    }

    void *host_tab, *dev_tab;
    int rc = sentry::table_staging_get(s, table_bytes, &host_tab);
    if (rc) return rc;
    rc = sentry::scratch_get(s, sentry::R_TABLES, table_bytes, &dev_tab);
    if (rc) return rc;
    SegDesc *hseg = static_cast<SegDesc *>(host_tab);
    {
        uint64_t leaf0 = 0;
        for (size_t t = 0; t < n_seg; t++) {
            hseg[t] = SegDesc{static_cast<const uint8_t *>(dev_ptrs[t]), lens[t], leaf0};
            leaf0 += leaf_count(lens[t], leaf_bytes);
        }
    }
    std::vector<const Group *> dev_groups;
    {
        char *hp = static_cast<char *>(host_tab) + n_seg * sizeof(SegDesc);
        char *dp = static_cast<char *>(dev_tab) + n_seg * sizeof(SegDesc);
        for (auto &st : stages) {
            std::memcpy(hp, st.data(), st.size() * sizeof(Group));
            dev_groups.push_back(reinterpret_cast<const Group *>(dp));
            hp += st.size() * sizeof(Group);
            dp += st.size() * sizeof(Group);
        }
    }
    SENTRY_HIP_CHECK(hipMemcpyAsync(dev_tab, host_tab, table_bytes, hipMemcpyHostToDevice, s));
    rc = sentry::table_staging_mark(s);
    if (rc) return rc;

    // where the per-segment roots end up
    uint8_t *roots = out_seg_roots;
    if (!roots || (reinterpret_cast<uintptr_t>(roots) & 15)) {
        void *p;
        rc = sentry::scratch_get(s, sentry::R_SEG_ROOTS, 32 * n_seg, &p);
        if (rc) return rc;
        roots = static_cast<uint8_t *>(p);
    }
    uint8_t *bufs[2] = {nullptr, nullptr};
    if (stages.size() > 1) {
        void *a, *b;
        rc = sentry::scratch_get(s, sentry::R_NODES_A, 32 * nodes0, &a);
        if (rc) return rc;
        rc = sentry::scratch_get(s, sentry::R_NODES_B, 32 * stages[1].size(), &b);
        if (rc) return rc;
        bufs[0] = static_cast<uint8_t *>(a);
        bufs[1] = static_cast<uint8_t *>(b);
    }
    const SegDesc *dseg = static_cast<const SegDesc *>(dev_tab);
    const uint8_t *src = nullptr;
    for (size_t k = 0; k < stages.size(); k++) {
        uint8_t *dst = (k + 1 == stages.size()) ? roots : bufs[k & 1];
        const uint32_t grid = (uint32_t)(k == 0 ? grid0 : stages[k].size());
        const bool split = small && waves <= SPLIT_LAUNCH_WAVES && leaf_bytes >= SPLIT_MIN_LEAF;
        if (k == 0 && packed) {
            if (split)
                launch_split<false, true, true>((uint32_t)waves, s, nullptr, 0, total_leaves, dseg, (uint32_t)n_seg, nullptr,
                                                (uint64_t)leaf_bytes, dst);
            else if (small)
                hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG_SMALL, false, true, true>), dim3(grid), dim3(LEAF_WG_SMALL), 0, s,
                                   (const uint8_t *)nullptr, (uint64_t)0, total_leaves, dseg, (uint32_t)n_seg,
                                   (const Group *)nullptr, (uint64_t)leaf_bytes, dst);
            else
                hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG, false, true, true>), dim3(grid), dim3(LEAF_WG), 0, s,
                                   (const uint8_t *)nullptr, (uint64_t)0, total_leaves, dseg, (uint32_t)n_seg,
                                   (const Group *)nullptr, (uint64_t)leaf_bytes, dst);
        } else if (k == 0) {
            if (split)
                launch_split<true, true>(grid, s, nullptr, 0, 0, dseg, (uint32_t)n_seg, dev_groups[0], (uint64_t)leaf_bytes, dst);
            else if (small)
                hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG_SMALL, true, true>), dim3(grid), dim3(LEAF_WG_SMALL), 0, s,
                                   (const uint8_t *)nullptr, (uint64_t)0, (uint64_t)0, dseg, (uint32_t)n_seg, dev_groups[0],
                                   (uint64_t)leaf_bytes, dst);
            else
                hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG, true, true>), dim3(grid), dim3(LEAF_WG), 0, s,
                                   (const uint8_t *)nullptr, (uint64_t)0, (uint64_t)0, dseg, (uint32_t)n_seg, dev_groups[0],
                                   (uint64_t)leaf_bytes, dst);
        } else {
            hipLaunchKernelGGL(merkle_reduce_kernel<true>, dim3(grid), dim3(RED_WG), 0, s, src, (uint64_t)0,
                               dev_groups[k], dst);
        }
        SENTRY_HIP_CHECK(hipGetLastError());
        src = dst;
    }
    if (out_seg_roots && roots != out_seg_roots)
        SENTRY_HIP_CHECK(hipMemcpyAsync(out_seg_roots, roots, 32 * n_seg, hipMemcpyDefault, s));
    return reduce_nodes(roots, n_seg, out_root, s);
}

int sentry_merkle_inplace(const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes,
                          uint8_t *out_root, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(n_seg >= 1, "sentry_merkle_inplace: n_seg must be at least 1");
    SENTRY_REQUIRE(dev_ptrs && lens && out_root, "sentry_merkle_inplace: NULL argument");
    SENTRY_REQUIRE(leaf_bytes > 0 && leaf_bytes % 64 == 0,
                   "sentry_merkle_inplace: leaf_bytes must be a positive multiple of 64 (got %zu)", leaf_bytes);
    SENTRY_REQUIRE(n_seg <= 0xffffffffull, "sentry_merkle_inplace: too many segments");
    uint64_t total = 0, waves = 0;
    for (size_t t = 0; t < n_seg; t++) {
        SENTRY_REQUIRE(dev_ptrs[t] != nullptr || lens[t] == 0, "sentry_merkle_inplace: segment %zu is NULL", t);
        SENTRY_REQUIRE((reinterpret_cast<uintptr_t>(dev_ptrs[t]) & 15) == 0,
                       "sentry_merkle_inplace: segment %zu is not 16-byte aligned", t);
        const uint64_t nl = ceil_div(lens[t], leaf_bytes);     // an empty tensor has no block
        total += nl;
        waves += ceil_div(nl, 64);
    }
    if (total == 0) return sentry_merkle_root(nullptr, 0, leaf_bytes, out_root, stream);   // the empty leaf

    // the lookup table of section 4.2.1: one row per workgroup (tensor, first block, blocks,
    // position of the first digest in the flat digest array); or, where many workgroups would be
    // part-filled, one row per tensor (its first block's index) and a bisection per lane
    const bool packed = packed_leaf_stage(waves, total);
    if (packed) waves = ceil_div(total, 64);
    const bool small = single_wave_groups(waves, leaf_bytes);
    const bool split = small && waves <= SPLIT_LAUNCH_WAVES && leaf_bytes >= SPLIT_MIN_LEAF;
    const uint64_t wg0 = small ? LEAF_WG_SMALL : LEAF_WG;
    std::vector<Group> g0;
    if (!packed) {
        uint64_t leaf0 = 0;
        for (size_t t = 0; t < n_seg; t++) {
            const uint64_t nl = ceil_div(lens[t], leaf_bytes);
            for (uint64_t f = 0; f < nl; f += wg0)
                g0.push_back(Group{f, leaf0 + f, (uint32_t)(nl - f < wg0 ? nl - f : wg0), (uint32_t)t});
            leaf0 += nl;
        }
    }
    const uint64_t grid0 = packed ? ceil_div(total, wg0) : g0.size();
    SENTRY_REQUIRE(grid0 <= MAX_GRID, "sentry_merkle_inplace: too many leaves");
    const size_t table_bytes = n_seg * sizeof(SegDesc) + g0.size() * sizeof(Group);
    void *host_tab, *dev_tab, *digests;
    int rc = sentry::table_staging_get(s, table_bytes, &host_tab);
    if (rc) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_TABLES, table_bytes, &dev_tab))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_NODES_A, 32 * total, &digests))) return rc;
    SegDesc *hseg = static_cast<SegDesc *>(host_tab);
    {
        uint64_t leaf0 = 0;
        for (size_t t = 0; t < n_seg; t++) {
            hseg[t] = SegDesc{static_cast<const uint8_t *>(dev_ptrs[t]), lens[t], leaf0};
            leaf0 += ceil_div(lens[t], leaf_bytes);
        }
    }
    if (!g0.empty())
        std::memcpy(static_cast<char *>(host_tab) + n_seg * sizeof(SegDesc), g0.data(), g0.size() * sizeof(Group));
    SENTRY_HIP_CHECK(hipMemcpyAsync(dev_tab, host_tab, table_bytes, hipMemcpyHostToDevice, s));
    if ((rc = sentry::table_staging_mark(s))) return rc;
    const SegDesc *dseg = static_cast<const SegDesc *>(dev_tab);
    const Group *dgroups = reinterpret_cast<const Group *>(static_cast<char *>(dev_tab) + n_seg * sizeof(SegDesc));
    const uint32_t grid = (uint32_t)grid0;
    uint8_t *dst = static_cast<uint8_t *>(digests);
    if (packed) {
        if (split)
            launch_split<false, true, true>((uint32_t)waves, s, nullptr, 0, total, dseg, (uint32_t)n_seg, nullptr,
                                            (uint64_t)leaf_bytes, dst);
        else if (small)
            hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG_SMALL, false, true, true>), dim3(grid), dim3(LEAF_WG_SMALL), 0, s,
                               (const uint8_t *)nullptr, (uint64_t)0, total, dseg, (uint32_t)n_seg, (const Group *)nullptr,
                               (uint64_t)leaf_bytes, dst);
        else
            hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG, false, true, true>), dim3(grid), dim3(LEAF_WG), 0, s,
                               (const uint8_t *)nullptr, (uint64_t)0, total, dseg, (uint32_t)n_seg, (const Group *)nullptr,
                               (uint64_t)leaf_bytes, dst);
    } else if (split)
        launch_split<false, true>(grid, s, nullptr, 0, 0, dseg, (uint32_t)n_seg, dgroups, (uint64_t)leaf_bytes, dst);
    else if (small)
        hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG_SMALL, false, true>), dim3(grid), dim3(LEAF_WG_SMALL), 0, s,
                           (const uint8_t *)nullptr, (uint64_t)0, (uint64_t)0, dseg, (uint32_t)n_seg, dgroups,
                           (uint64_t)leaf_bytes, dst);
    else
        hipLaunchKernelGGL((merkle_leaf_kernel<LEAF_WG, false, true>), dim3(grid), dim3(LEAF_WG), 0, s,
                           (const uint8_t *)nullptr, (uint64_t)0, (uint64_t)0, dseg, (uint32_t)n_seg, dgroups,
                           (uint64_t)leaf_bytes, dst);
    SENTRY_HIP_CHECK(hipGetLastError());
    return reduce_nodes(dst, total, out_root, s);
}

}  // extern "C"

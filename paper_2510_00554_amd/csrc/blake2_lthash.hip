// Lattice hash over dataset samples on gfx950 (section 2.2 Eq. (1), section 4.2.2,
// section 4.3): per-record digest h(M) = BLAKE2Xb(M) with 2048 output bytes read as
// 1024 little-endian uint16 lanes, summed lane-wise mod 2^16.
//
// The kernels:
//   lthash_root1_kernel,  the sequential BLAKE2b-512 root hash H0 of every record (the only
//   lthash_root4_kernel   serial part), one lane per record or four lanes per record (with
//                         lthash_order_count/scan/place_kernel, which order the records by
//                         length for the latter), 64 bytes per record to scratch;
//   lthash_expand_kernel  one (record, output block) pair per lane: the 32 expansion
//                         compressions of a record are independent, so they are spread
//                         over all lanes of the chip; each lane keeps the 16 packed words
//                         of "its" output block in registers and adds every record's
//                         block to them (v_pk_add_u16), so the 2048-byte digests never
//                         exist in memory; per-workgroup partial sums go to scratch;
//   lthash_fold_kernel    adds the partial sums column-wise into the 1024 lanes;
//   lthash_digests_kernel, lthash_sum_kernel   the digests written out one by one, and the
//                         lane sum over digests that are in memory;
//   src_count/scatter_kernel, lthash_expand_units_kernel, lthash_fold_sources_kernel   one
//                         running sum per data source (section 4.3); lthash_root4_rider_kernel
//                         for small batches: root hashes and the sort by source in one launch;
//                         lthash_root1_count_kernel, lthash_root4_scatter_kernel for large ones:
//                         the two steps of the sort at the front of the two root-hash launches.
// The root kernels take the first two words of the parameter block as arguments: with those of
// the plain BLAKE2b-512 they also serve the 32-partition hash of blake2_lthash32.hip.
#include "blake2b_device.h"
#include "lthash_internal.h"

namespace {

constexpr int EXP_WG = 256;
constexpr int EXP_WAVES = EXP_WG / 64;
constexpr int LANE_WORDS = SENTRY_LANES / 2;   // 512 packed 32-bit words = 2048 bytes
constexpr int FOLD_WG = 256;
constexpr int FOLD_COLS = 32;                  // packed words per fold workgroup
constexpr uint32_t XOF_BYTES = 2 * SENTRY_LANES;

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// BLAKE2Xb parameter blocks (byte 0 digest length, 1 key length, 2 fanout, 3 depth,
// 4..7 leaf length, 8..11 node offset, 12..15 XOF length, 16 node depth, 17 inner length).
// Root hash: digest 64, fanout 1, depth 1, XOF length 2048: LT_ROOT_P0, LT_ROOT_P1 (in the header
// shared with the file of the 32-partition hash, whose per-record hash has another parameter block).
static_assert(sentry::LT_ROOT_P0 == 0x0000000001010040ull && sentry::LT_ROOT_P1 == ((uint64_t)XOF_BYTES << 32),
              "root hash parameters");
// Expansion node j: digest 64, fanout 0, depth 0, leaf length 64, node offset j, XOF
// length 2048, inner length 64.
constexpr uint64_t EXP_P0 = 0x0000004000000040ull;
constexpr uint64_t EXP_P1_HI = (uint64_t)XOF_BYTES << 32;
constexpr uint64_t EXP_P2 = 0x0000000000004000ull;

// ---------------------------------------------------------------------------
// root hash kernel
// ---------------------------------------------------------------------------

// 32-bit word k of a 128-byte block that starts `sh`/8 bytes into the aligned word d[0]
#define M32(k) __builtin_amdgcn_alignbit(d[(k) + 1], d[k], sh)

// Where record i lies: bytes [offsets[i], offsets[i + 1]) less offset_base, or, for records of one
// size laid back to back (offsets == nullptr), i times that size, which offset_base then holds.
__device__ __forceinline__ void record_span(const uint64_t *offsets, uint64_t offset_base, uint64_t i, uint64_t &beg,
                                            uint64_t &len)
{
    if (offsets) {
        beg = offsets[i] - offset_base;
        len = offsets[i + 1] - offsets[i];
    } else {
        beg = i * offset_base;
        len = offset_base;
    }
}

// One record per lane: record i of n.
// p0, p1: the first two words of the parameter block (the others are zero for both hashes used).
__device__ __forceinline__ void root_one_lane(const uint8_t *records, const uint64_t *offsets, uint64_t offset_base,
                                              uint64_t n, uint64_t *h0_out, uint64_t i, uint64_t p0, uint64_t p1)
{
    if (i >= n) return;
    uint64_t beg, len;
    record_span(offsets, offset_base, i, beg, len);
    const uint32_t a = (uint32_t)((reinterpret_cast<uintptr_t>(records) + beg) & 3);
    const uint32_t sh = 8 * a;
    const uint32_t *q = reinterpret_cast<const uint32_t *>(records + beg - a);

    uint64_t h[8];
#pragma unroll
    for (int k = 0; k < 8; k++) h[k] = b2_iv(k);
    h[0] ^= p0;
    h[1] ^= p1;

    uint32_t d[33];
    uint64_t done = 0;
    // every block but the last is full; a full block that is not the last is followed by at
    // least one more byte of the record, so all 33 aligned words it touches hold record bytes
    if (len > 128) {
#pragma unroll
        for (int k = 0; k < 33; k++) d[k] = q[k];
    }
    while (len - done > 128) {
        uint64_t m[16];
#pragma unroll
        for (int k = 0; k < 16; k++) m[k] = pack64(M32(2 * k), M32(2 * k + 1));
        done += 128;
        q += 32;
        if (len - done > 128) {   // fetch the next full block while this one is compressed
            d[0] = d[32];
#pragma unroll
            for (int k = 1; k < 33; k++) d[k] = q[k];
        }
        blake2b_compress(h, m, done, false);
    }
    // last block: 1..128 bytes (0 only for the empty record), zero padded; words that hold
    // no byte of the record are not read
    {
        const uint32_t rem = (uint32_t)(len - done);
        const uint32_t span = rem ? a + rem : 0u;   // bytes from the aligned base to the record's end
#pragma unroll
        for (int k = 0; k < 33; k++) d[k] = ((uint32_t)(4 * k) < span) ? q[k] : 0u;
        uint32_t w[32];
#pragma unroll
        for (int k = 0; k < 32; k++) {
            const uint32_t lo = (uint32_t)(4 * k);
            uint32_t x = M32(k);
            if (rem < lo + 4) x = (rem <= lo) ? 0u : (x & ((1u << (8 * (rem - lo))) - 1u));
            w[k] = x;
        }
        uint64_t m[16];
#pragma unroll
        for (int k = 0; k < 16; k++) m[k] = pack64(w[2 * k], w[2 * k + 1]);
        blake2b_compress(h, m, len, true);
    }
#pragma unroll
    for (int k = 0; k < 8; k++) h0_out[8 * i + k] = h[k];
}
#undef M32

// ---------------------------------------------------------------------------
// root hash kernel, four lanes per record
// ---------------------------------------------------------------------------
//
// BLAKE2b's state is a 4x4 matrix of 64-bit words; a round applies G to the four columns,
// then to the four diagonals, and the four G calls of a step are independent.  Here lane j
// of a quad holds column j (a = v[j], b = v[4+j], c = v[8+j], d = v[12+j]); the column step
// runs in all four lanes at once, the diagonal step after rotating a, c, d inside the quad
// (DPP quad_perm) so that lane j holds the diagonal that contains its own b: b is the value
// a step produces last and needs first, so it is the one that stays where it is.  This cuts
// the serial chain of a long record to about a third, which is what bounds a launch with
// fewer records than lanes.
//
// Each lane needs different message words in every step (the sigma permutation), which
// static register indexing cannot give; the quad therefore stages the 128-byte block in LDS
// (lane j loads bytes [32j, 32j+32) from global memory) and every lane reads its four words
// per round from per-lane addresses that are computed once per kernel (16-bit addresses,
// two per register, ten rounds of sigma; rounds 10 and 11 reuse rows 0 and 1).

constexpr int ROOT4_WG = 64;               // one wave per workgroup, 16 records per wave
constexpr int ROOT4_RECORDS = ROOT4_WG / 4;
// One lane per record: workgroups of four waves, which land on the four SIMDs of a CU, one each.
// With single-wave workgroups the dispatcher now and then put two waves on one SIMD of a CU
// whose other SIMDs were idle, and a launch with fewer waves than SIMDs (50,000 images) then
// took 176 us instead of 101 us, in about every second launch.
constexpr int ROOT1_WG = 256;

__device__ const unsigned char B2_SIGMA_TABLE[10][16] = {
    {0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15}, {14, 10, 4, 8, 9, 15, 13, 6, 1, 12, 0, 2, 11, 7, 5, 3},
    {11, 8, 12, 0, 5, 2, 15, 13, 10, 14, 3, 6, 7, 1, 9, 4}, {7, 9, 3, 1, 13, 12, 11, 14, 2, 6, 5, 10, 4, 0, 15, 8},
    {9, 0, 5, 7, 2, 4, 10, 15, 14, 1, 11, 12, 6, 8, 3, 13}, {2, 12, 6, 10, 0, 11, 8, 3, 4, 13, 7, 5, 15, 14, 1, 9},
    {12, 5, 1, 15, 14, 13, 4, 10, 0, 7, 6, 3, 9, 2, 8, 11}, {13, 11, 7, 14, 12, 1, 3, 9, 5, 0, 15, 4, 8, 6, 2, 10},
    {6, 15, 14, 9, 11, 3, 0, 8, 12, 2, 13, 7, 1, 4, 10, 5}, {10, 2, 8, 4, 7, 6, 1, 5, 15, 11, 9, 14, 3, 12, 13, 0}};

// value of x in the lane of the same quad selected by the quad_perm control word
template <int CTRL>
__device__ __forceinline__ uint64_t quad_rotate(uint64_t x)
{
    // all rows and banks enabled and every source lane inside the quad: each lane is written
    const int lo = __builtin_amdgcn_mov_dpp((int)(uint32_t)x, CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_mov_dpp((int)(uint32_t)(x >> 32), CTRL, 0xf, 0xf, true);
    return pack64((uint32_t)lo, (uint32_t)hi);
}
constexpr int QP_FROM_NEXT1 = 1 | (2 << 2) | (3 << 4) | (0 << 6);   // lane j reads lane (j+1)&3
constexpr int QP_FROM_NEXT2 = 2 | (3 << 2) | (0 << 4) | (1 << 6);   // lane j reads lane (j+2)&3
constexpr int QP_FROM_NEXT3 = 3 | (0 << 2) | (1 << 4) | (2 << 6);   // lane j reads lane (j+3)&3

// A launch of this kernel is bound by the chain of dependent instructions of its longest
// record, so G is written for the shortest chain rather than the fewest instructions:
// a + x and a + y are formed before b, the last value of the previous step, is needed, so
// one add instead of two follows b.
__device__ __forceinline__ uint64_t add64(uint64_t a, uint64_t b) { return a + b; }
#define B2_G_CHAIN(a, b, c, d, x, y)                                  \
    do {                                                              \
        const uint64_t ax_ = add64(a, x);                             \
        a = add64(ax_, b); d = rotr64_32(d ^ a);                      \
        c = add64(c, d);   b = rotr64_lt32<24>(b ^ c);                \
        const uint64_t ay_ = add64(a, y);                             \
        a = add64(ay_, b); d = rotr64_lt32<16>(d ^ a);                \
        c = add64(c, d);   b = rotr64_63(b ^ c);                      \
    } while (0)

// Sixteen records per wave, four lanes each: the wave's records are first_rec .. first_rec + 15.
__device__ __forceinline__ void root_four_lanes(const uint8_t *records, const uint64_t *offsets, uint64_t offset_base,
                                                uint64_t n, const uint32_t *order, uint64_t *h0_out, uint64_t first_rec,
                                                unsigned char *stage, uint64_t p0, uint64_t p1)
{
    const uint32_t lane = threadIdx.x, quad = lane >> 2, j = lane & 3;
    const uint64_t slot = first_rec + quad;
    const bool active = slot < n;
    const uint64_t rec = (active && order) ? order[slot] : slot;   // longest records first when ordered
    uint64_t beg = 0, len = 0;
    if (active) record_span(offsets, offset_base, rec, beg, len);
    // blocks of this lane's record (the empty record has one)
    const uint32_t my_blocks = (uint32_t)(((len + 127) >> 7) > 0xffffffffull ? 0xffffffffull : (len ? (len + 127) >> 7 : 1));
    uint32_t wave_blocks = active ? my_blocks : 0u;   // the longest record of the wave
#pragma unroll
    for (int sft = 32; sft >= 4; sft >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)wave_blocks, sft, 64);
        wave_blocks = o > wave_blocks ? o : wave_blocks;
    }
    wave_blocks = __builtin_amdgcn_readfirstlane(wave_blocks);
    if (!active) return;   // whole quads leave together, so quad_perm never reads a dead lane

    const uint32_t al = (uint32_t)((reinterpret_cast<uintptr_t>(records) + beg) & 3);
    const uint32_t sh = 8 * al;
    // aligned words of this lane's 32-byte slice of the first block
    const uint32_t *q = reinterpret_cast<const uint32_t *>(records + beg - al) + 8 * j;

    // per-lane LDS addresses of the message words of every round.  The sixteen quads of a wave keep
    // their blocks 128 bytes apart, which is the width of all LDS banks: unswizzled, the sixteen lanes
    // that read the same message word of their quads would all hit one pair of banks.  So quad q keeps
    // its eight 16-byte cells (two message words each) at cell number XOR (q & 7): the sixteen quads
    // then spread over eight bank groups (two per group instead of sixteen), and a lane still stores
    // its slice as two whole cells, at two addresses that are computed once.
    const uint32_t qbase = quad * 128;
    const uint32_t cell_flip = quad & 7;
    auto swizzled = [&](uint32_t word) -> uint32_t { return 16u * ((word >> 1) ^ cell_flip) + 8u * (word & 1); };
    uint32_t maddr[10][2];
#pragma unroll
    for (int r = 0; r < 10; r++) {
#pragma unroll
        for (int st = 0; st < 2; st++) {
            // column step: column j; diagonal step: the diagonal through b of column j, number j - 1
            const uint32_t g = st == 0 ? j : ((j + 3) & 3);
            const uint32_t x = qbase + swizzled(B2_SIGMA_TABLE[r][8 * st + 2 * g]);
            const uint32_t y = qbase + swizzled(B2_SIGMA_TABLE[r][8 * st + 2 * g + 1]);
            maddr[r][st] = x | (y << 16);
        }
    }
    // this lane's 32-byte slice = message words 4j .. 4j+3 = the two 16-byte cells 2j and 2j+1
    unsigned char *my_cell0 = stage + qbase + swizzled(4 * j);
    unsigned char *my_cell1 = stage + qbase + swizzled(4 * j + 2);

    // column j of the chaining value and of the IV
    const uint64_t iv_lo = j == 0 ? b2_iv(0) : j == 1 ? b2_iv(1) : j == 2 ? b2_iv(2) : b2_iv(3);
    const uint64_t iv_hi = j == 0 ? b2_iv(4) : j == 1 ? b2_iv(5) : j == 2 ? b2_iv(6) : b2_iv(7);
    uint64_t h_lo = iv_lo ^ (j == 0 ? p0 : j == 1 ? p1 : 0ull);
    uint64_t h_hi = iv_hi;

    // Four blocks of this lane's slice are in flight: a global load takes about as long as one
    // compression, longer while the bulk of a batch streams through the chip, and with one
    // block in flight the chain of the longest record waited for its data on every block
    // (one 707 KB record alone: 9.4 ms with one block in flight, 8.1 ms with four).
    constexpr int AHEAD = 4;
    uint32_t db[AHEAD][9];
    uint64_t done = 0;
    uint32_t blk = 0;
#pragma unroll
    for (int u = 0; u < AHEAD; u++) {
        if (len > 128ull * (u + 1)) {
#pragma unroll
            for (int k = 0; k < 9; k++) db[u][k] = q[32 * u + k];
        }
    }
    // one block; d is the buffer that holds it if it is full and not the last; true when done
    auto step = [&](uint32_t (&d)[9]) -> bool {
        // The launch ends when its longest chain ends, so the wave with the most blocks still to
        // go should never wait for an issue slot: every 256 blocks the wave sets its priority
        // from what is left of its longest record (all its live lanes are at the same block).
        if ((blk & 255u) == 0) {
            const uint32_t left = wave_blocks - blk;
            if (left >= 4096) __builtin_amdgcn_s_setprio(3);
            else if (left >= 2048) __builtin_amdgcn_s_setprio(2);
            else if (left >= 768) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        blk++;
        const bool last = len - done <= 128;
        uint32_t w[8];
        uint64_t t;
        if (!last) {
#pragma unroll
            for (int k = 0; k < 8; k++) w[k] = __builtin_amdgcn_alignbit(d[k + 1], d[k], sh);
            done += 128;
            q += 32;                        // q: the next block
            t = done;
            if (len - done > 128ull * AHEAD) {   // the block AHEAD blocks on is full and not the last: fetch it now
#pragma unroll
                for (int k = 0; k < 9; k++) d[k] = q[32 * (AHEAD - 1) + k];
            }
        } else {
            // 1..128 bytes (0 for the empty record), zero padded; words without a record byte are not read
            const uint32_t rem = (uint32_t)(len - done);
            const uint32_t span = rem ? al + rem : 0u;
            uint32_t e[9];
#pragma unroll
            for (int k = 0; k < 9; k++) e[k] = ((uint32_t)(4 * (8 * j + k)) < span) ? q[k] : 0u;
#pragma unroll
            for (int k = 0; k < 8; k++) {
                const uint32_t lo = 4u * (8u * j + (uint32_t)k);
                uint32_t x = __builtin_amdgcn_alignbit(e[k + 1], e[k], sh);
                if (rem < lo + 4) x = (rem <= lo) ? 0u : (x & ((1u << (8 * (rem - lo))) - 1u));
                w[k] = x;
            }
            t = len;
        }
        // stage the block: this lane's four message words
        *reinterpret_cast<uint4 *>(my_cell0) = make_uint4(w[0], w[1], w[2], w[3]);
        *reinterpret_cast<uint4 *>(my_cell1) = make_uint4(w[4], w[5], w[6], w[7]);

        uint64_t a = h_lo, b = h_hi, c = iv_lo, dd = iv_hi;
        if (j == 0) dd ^= t;
        if (last && j == 2) dd = ~dd;
#pragma unroll
        for (int r = 0; r < 12; r++) {
            const uint32_t pc = maddr[r % 10][0], pd = maddr[r % 10][1];
            const uint64_t mc0 = *reinterpret_cast<const uint64_t *>(stage + (pc & 0xffffu));
            const uint64_t mc1 = *reinterpret_cast<const uint64_t *>(stage + (pc >> 16));
            const uint64_t md0 = *reinterpret_cast<const uint64_t *>(stage + (pd & 0xffffu));
            const uint64_t md1 = *reinterpret_cast<const uint64_t *>(stage + (pd >> 16));
            B2_G_CHAIN(a, b, c, dd, mc0, mc1);
            a = quad_rotate<QP_FROM_NEXT3>(a);     // a of column j - 1
            c = quad_rotate<QP_FROM_NEXT1>(c);     // c of column j + 1
            dd = quad_rotate<QP_FROM_NEXT2>(dd);   // d of column j + 2
            B2_G_CHAIN(a, b, c, dd, md0, md1);
            a = quad_rotate<QP_FROM_NEXT1>(a);
            c = quad_rotate<QP_FROM_NEXT3>(c);
            dd = quad_rotate<QP_FROM_NEXT2>(dd);
        }
        h_lo ^= a ^ c;
        h_hi ^= b ^ dd;
        return last;
    };
    for (bool fin = false; !fin;) {
#pragma unroll
        for (int u = 0; u < AHEAD; u++) {
            if (step(db[u])) { fin = true; break; }
        }
    }
    h0_out[8 * rec + j] = h_lo;
    h0_out[8 * rec + 4 + j] = h_hi;
}

// Root hashes of n records: one lane per record, or four lanes per record, in length order or
// not.  Which, is chosen on the device from the record lengths, which a kernel can read from
// the offsets while the host cannot (the offsets are device memory and the call does not wait).
// One lane per record is the cheaper form for many records of one size (images): every lane of
// a wave ends together and the start-up per record is small.  Four lanes in length order are
// for long records (16 KiB and more on average), whose serial chains bound the launch, and for
// batches of unequal records, where one lane per record makes a wave live as long as the
// longest of its 64 records and a launch as long as its longest record hashed by a single lane
// (1 M records, log-normal around 6 KB: 25.5 ms against 8.6 ms).  Unequal means: of 256 records
// at fixed positions of the batch the longest is at least 4 KiB and at least 1.5 times the mean.
// Four lanes without the ordering are for batches of few records (up to half the lanes of the
// chip), which are bound by one record's chain whatever its length: four lanes make it a third
// as long (10,000 images: 0.075 ms against 0.128 ms).  Every workgroup of every kernel evaluates
// this for itself (two loads per lane) and gets the same answer.
constexpr uint64_t FOUR_LANE_MEAN_BYTES = 16384;
constexpr uint64_t UNEQUAL_MIN_BYTES = 4096;
constexpr uint64_t FEW_RECORDS = 32768;
constexpr uint64_t ORDER_MIN_RECORDS = 16384;   // batches up to this size are not ordered (host side: see lthash_roots)

__device__ __forceinline__ bool ordered_mode(const uint64_t *offsets, uint64_t n)
{
    const uint64_t total = offsets[n] - offsets[0];
    if (total >= FOUR_LANE_MEAN_BYTES * n) return true;
    const uint32_t lane = threadIdx.x & 63;
    uint64_t longest = 0;
#pragma unroll
    for (int k = 0; k < 4; k++) {
        const uint64_t i = ((uint64_t)(64 * k + lane) * n) >> 8;     // n < 2^32 (checked by the host)
        const uint64_t len = offsets[i + 1] - offsets[i];
        longest = len > longest ? len : longest;
    }
#pragma unroll
    for (int d = 32; d; d >>= 1) {
        const uint64_t o = __shfl_xor(longest, d, 64);
        longest = o > longest ? o : longest;
    }
    return longest >= UNEQUAL_MIN_BYTES && 2 * longest >= 3 * (total / n);   // 1.5 x the (whole-byte) mean
}

__device__ __forceinline__ bool four_lane_mode(const uint64_t *offsets, uint64_t n)
{
    return n <= FEW_RECORDS || ordered_mode(offsets, n);
}

// Two kernels, so that each path gets its own register budget and code footprint (the
// four-lane path keeps four blocks in flight and unrolls its loop four times; inside one
// kernel that slowed the one-lane path down by a third).  Both are launched when the choice
// launched; the one whose mode is not taken returns at once.
__global__ void __launch_bounds__(ROOT1_WG)
lthash_root1_kernel(const uint8_t *records, const uint64_t *offsets, uint64_t offset_base, uint64_t n, uint64_t *h0_out,
                    uint64_t p0, uint64_t p1)
{
    if (offsets && four_lane_mode(offsets, n)) return;    // without offsets the host launches the one kernel it wants
    root_one_lane(records, offsets, offset_base, n, h0_out, (uint64_t)blockIdx.x * ROOT1_WG + threadIdx.x, p0, p1);
}

__global__ void __launch_bounds__(ROOT4_WG)
lthash_root4_kernel(const uint8_t *records, const uint64_t *offsets, uint64_t offset_base, uint64_t n,
                    const uint32_t *order, uint64_t *h0_out, uint64_t p0, uint64_t p1)
{
    __shared__ __attribute__((aligned(16))) unsigned char stage[ROOT4_RECORDS * 128];
    if (offsets && !four_lane_mode(offsets, n)) return;
    root_four_lanes(records, offsets, offset_base, n, offsets && ordered_mode(offsets, n) ? order : nullptr, h0_out,
                    (uint64_t)blockIdx.x * ROOT4_RECORDS, stage, p0, p1);
}

// Order of the records for the four-lane path: longest first (a counting sort by length in
// units of 256 bytes; the order inside a bin is arbitrary, which the order-invariant sum does
// not see).  A wave then holds sixteen records of about the same length, so it issues no
// instructions for quads that finished long ago (in the given order a wave lives as long as the
// longest of its sixteen records: twice the instructions), and consecutive waves, which the
// dispatcher deals out over the SIMDs, carry the long chains first, one per SIMD, before the
// next tier follows.  Three kernels, as in one pass of a radix sort: every workgroup counts the
// bins of its run of records; one workgroup turns the counts into the place where each
// (workgroup, bin) starts; every workgroup puts its records there.  (One workgroup doing all of
// it took 1.7 ms for a million records.)  All return at once when the batch is not ordered.
constexpr int SORT_WG = 512;              // eight waves find room on a CU that other kernels fill
constexpr uint32_t SORT_BINS = 4096;
constexpr uint32_t SORT_MAX_GROUPS = 64;
constexpr uint32_t SORT_MIN_RUN = 4096;   // records per workgroup before a second one is worth it

__device__ __forceinline__ uint32_t length_bin(uint64_t len)   // 0 = longest
{
    const uint64_t k = len >> 8;
    return SORT_BINS - 1 - (uint32_t)(k < SORT_BINS - 1 ? k : SORT_BINS - 1);
}

// the run of records of workgroup g of `groups`
__device__ __forceinline__ void sort_run(uint64_t n, uint32_t g, uint32_t groups, uint64_t &lo, uint64_t &hi)
{
    const uint64_t per = (n + groups - 1) / groups;
    lo = per * g < n ? per * g : n;
    hi = lo + per < n ? lo + per : n;
}

// bins of records [lo, hi), eight records per lane and trip so that their offsets are in flight
// together: f(record, bin) for each
template <typename F>
__device__ __forceinline__ void for_each_bin(const uint64_t *offsets, uint64_t lo, uint64_t hi, F f)
{
    constexpr int BATCH = 8;
    for (uint64_t i0 = lo + threadIdx.x; i0 < hi; i0 += (uint64_t)BATCH * SORT_WG) {
        uint32_t b[BATCH];
#pragma unroll
        for (int k = 0; k < BATCH; k++) {
            const uint64_t i = i0 + (uint64_t)k * SORT_WG;
            b[k] = i < hi ? length_bin(offsets[i + 1] - offsets[i]) : SORT_BINS;
        }
#pragma unroll
        for (int k = 0; k < BATCH; k++)
            if (b[k] < SORT_BINS) f(i0 + (uint64_t)k * SORT_WG, b[k]);
    }
}

// counts[g][bin] = records of workgroup g's run that fall into bin
__global__ void __launch_bounds__(SORT_WG)
lthash_order_count_kernel(const uint64_t *offsets, uint64_t n, uint32_t *counts)
{
    if (!ordered_mode(offsets, n)) return;
    __shared__ uint32_t bin[SORT_BINS];
    for (uint32_t k = threadIdx.x; k < SORT_BINS; k += SORT_WG) bin[k] = 0;
    __syncthreads();
    uint64_t lo, hi;
    sort_run(n, blockIdx.x, gridDim.x, lo, hi);
    for_each_bin(offsets, lo, hi, [&](uint64_t, uint32_t b) { atomicAdd(&bin[b], 1u); });
    __syncthreads();
    for (uint32_t k = threadIdx.x; k < SORT_BINS; k += SORT_WG) counts[(uint64_t)blockIdx.x * SORT_BINS + k] = bin[k];
}

// counts[g][bin] <- first place in the order of workgroup g's records of that bin: bins in
// ascending number (longest records first), inside a bin the workgroups in ascending number.
// One workgroup; lane t owns PER consecutive bins.
__global__ void __launch_bounds__(SORT_WG)
lthash_order_scan_kernel(const uint64_t *offsets, uint64_t n, uint32_t *counts, uint32_t groups)
{
    if (!ordered_mode(offsets, n)) return;
    constexpr uint32_t PER = SORT_BINS / SORT_WG;
    __shared__ uint32_t part[SORT_WG / 64];
    const uint32_t tid = threadIdx.x;
    uint32_t c[PER], sum = 0;
#pragma unroll
    for (uint32_t k = 0; k < PER; k++) c[k] = 0;
    for (uint32_t g = 0; g < groups; g++)
#pragma unroll
        for (uint32_t k = 0; k < PER; k++) c[k] += counts[(uint64_t)g * SORT_BINS + PER * tid + k];
#pragma unroll
    for (uint32_t k = 0; k < PER; k++) sum += c[k];
    // exclusive scan of the lanes' sums: prefix inside each wave by shuffles, then the totals
    // of the waves before it
    uint32_t incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, d, 64);
        if ((tid & 63) >= (uint32_t)d) incl += o;
    }
    if ((tid & 63) == 63) part[tid >> 6] = incl;
    __syncthreads();
    uint32_t before = incl - sum;
    for (uint32_t w = 0; w < (tid >> 6); w++) before += part[w];
    uint32_t at[PER];
#pragma unroll
    for (uint32_t k = 0; k < PER; k++) { at[k] = before; before += c[k]; }
    for (uint32_t g = 0; g < groups; g++)
#pragma unroll
        for (uint32_t k = 0; k < PER; k++) {
            uint32_t *p = &counts[(uint64_t)g * SORT_BINS + PER * tid + k];
            const uint32_t v = *p;
            *p = at[k];
            at[k] += v;
        }
}

__global__ void __launch_bounds__(SORT_WG)
lthash_order_place_kernel(const uint64_t *offsets, uint64_t n, const uint32_t *places, uint32_t *order)
{
    if (!ordered_mode(offsets, n)) return;
    __shared__ uint32_t bin[SORT_BINS];
    for (uint32_t k = threadIdx.x; k < SORT_BINS; k += SORT_WG) bin[k] = places[(uint64_t)blockIdx.x * SORT_BINS + k];
    __syncthreads();
    uint64_t lo, hi;
    sort_run(n, blockIdx.x, gridDim.x, lo, hi);
    for_each_bin(offsets, lo, hi, [&](uint64_t i, uint32_t b) { order[atomicAdd(&bin[b], 1u)] = (uint32_t)i; });
}

// ---------------------------------------------------------------------------
// expansion + lane accumulation kernel
// ---------------------------------------------------------------------------

// Lane l of every wave owns output block j = l & 31 and takes records 2*slot + (l >> 5),
// slot = wave index, wave index + total waves, ...  part_out: one 2048-byte partial sum per
// workgroup.  ONLY_SOURCE0: records whose source id is not 0 are left out (the one-source case of
// the per-source sums).
template <bool ONLY_SOURCE0>
__global__ void __launch_bounds__(EXP_WG)
lthash_expand_kernel(const uint64_t *h0, uint64_t n, uint32_t *part_out, const uint32_t *source_ids)
{
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t j = lane & 31;
    const uint64_t total_waves = (uint64_t)gridDim.x * EXP_WAVES;
    u16x2 acc[16];
#pragma unroll
    for (int k = 0; k < 16; k++) acc[k] = u16x2{0, 0};

    for (uint64_t slot = (uint64_t)blockIdx.x * EXP_WAVES + wave;; slot += total_waves) {
        if (2 * slot >= n) break;                      // wave-uniform
        const uint64_t rec = 2 * slot + (lane >> 5);
        if (rec < n && (!ONLY_SOURCE0 || source_ids[rec] == 0)) {
            uint64_t m[16];
#pragma unroll
            for (int k = 0; k < 8; k++) { m[k] = h0[8 * rec + k]; m[8 + k] = 0; }
            uint64_t h[8];
#pragma unroll
            for (int k = 0; k < 8; k++) h[k] = b2_iv(k);
            h[0] ^= EXP_P0;
            h[1] ^= EXP_P1_HI | (uint64_t)j;
            h[2] ^= EXP_P2;
            blake2b_compress(h, m, 64, true);
#pragma unroll
            for (int k = 0; k < 8; k++) {
                const uint32_t lo = (uint32_t)h[k], hi = (uint32_t)(h[k] >> 32);
                acc[2 * k] += u16x2{(unsigned short)lo, (unsigned short)(lo >> 16)};
                acc[2 * k + 1] += u16x2{(unsigned short)hi, (unsigned short)(hi >> 16)};
            }
        }
    }
    // the two half-waves hold the same 32 blocks: add the upper half into the lower one
    __shared__ uint32_t lds[EXP_WAVES][LANE_WORDS];
#pragma unroll
    for (int k = 0; k < 16; k++) {
        uint32_t x = (uint32_t)acc[k].x | ((uint32_t)acc[k].y << 16);
        uint32_t y = (uint32_t)__shfl_xor((int)x, 32, 64);
        u16x2 s = acc[k] + u16x2{(unsigned short)y, (unsigned short)(y >> 16)};
        if (lane < 32) lds[wave][16 * j + k] = (uint32_t)s.x | ((uint32_t)s.y << 16);
    }
    __syncthreads();
    for (uint32_t c = tid; c < LANE_WORDS; c += EXP_WG) {
        u16x2 s = u16x2{0, 0};
#pragma unroll
        for (int w = 0; w < EXP_WAVES; w++) {
            const uint32_t x = lds[w][c];
            s += u16x2{(unsigned short)x, (unsigned short)(x >> 16)};
        }
        part_out[(uint64_t)blockIdx.x * LANE_WORDS + c] = (uint32_t)s.x | ((uint32_t)s.y << 16);
    }
}

// The digests themselves, one row of 2048 bytes per record, for callers that keep them (a
// sample can later be taken out of a sum without its bytes: sentry_lthash_remove).  Same lane
// assignment as lthash_expand_kernel; each lane writes the 64 bytes of its block.
__global__ void __launch_bounds__(EXP_WG)
lthash_digests_kernel(const uint64_t *h0, uint64_t n, uint4 *out)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t j = lane & 31;
    const uint64_t total_waves = (uint64_t)gridDim.x * EXP_WAVES;
    for (uint64_t slot = (uint64_t)blockIdx.x * EXP_WAVES + wave; 2 * slot < n; slot += total_waves) {
        const uint64_t rec = 2 * slot + (lane >> 5);
        if (rec >= n) continue;
        uint64_t m[16];
#pragma unroll
        for (int k = 0; k < 8; k++) { m[k] = h0[8 * rec + k]; m[8 + k] = 0; }
        uint64_t h[8];
#pragma unroll
        for (int k = 0; k < 8; k++) h[k] = b2_iv(k);
        h[0] ^= EXP_P0;
        h[1] ^= EXP_P1_HI | (uint64_t)j;
        h[2] ^= EXP_P2;
        blake2b_compress(h, m, 64, true);
        uint4 *dst = out + rec * (XOF_BYTES / 16) + 4 * j;
#pragma unroll
        for (int k = 0; k < 4; k++)
            dst[k] = make_uint4((uint32_t)h[2 * k], (uint32_t)(h[2 * k] >> 32), (uint32_t)h[2 * k + 1], (uint32_t)(h[2 * k + 1] >> 32));
    }
}

// Eq. (1) over digests that are in memory: part_out[workgroup] = lane-wise sum of the rows the
// workgroup takes.  2048 bytes are read per row and four packed adds are done per 16 of them,
// so this kernel is bound by HBM: lane t of a half-workgroup owns 16-byte column t & 127, the
// two halves take alternate rows, every lane has eight rows in flight, and a workgroup takes
// a contiguous run of rows (2^20 rows: 7.0 TB/s; with the rows dealt out round-robin over the
// workgroups 5.6 TB/s, with plain instead of streaming loads 5.3 TB/s).
constexpr int SUM_WG = 256;
constexpr int SUM_AHEAD = 8;
constexpr int SUM_COLS = XOF_BYTES / 16;   // 128 columns of 16 bytes
constexpr int SUM_HALVES = SUM_WG / SUM_COLS;

typedef uint32_t sum_u32x4 __attribute__((ext_vector_type(4)));

// streaming load: every digest byte is read once
__device__ __forceinline__ uint4 load_once(const uint4 *p)
{
    const sum_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const sum_u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void add_packed(u16x2 (&acc)[4], const uint4 v)
{
    acc[0] += u16x2{(unsigned short)v.x, (unsigned short)(v.x >> 16)};
    acc[1] += u16x2{(unsigned short)v.y, (unsigned short)(v.y >> 16)};
    acc[2] += u16x2{(unsigned short)v.z, (unsigned short)(v.z >> 16)};
    acc[3] += u16x2{(unsigned short)v.w, (unsigned short)(v.w >> 16)};
}

__global__ void __launch_bounds__(SUM_WG)
lthash_sum_kernel(const uint4 *rows, uint64_t n, uint4 *part_out)
{
    const uint32_t c = threadIdx.x % SUM_COLS, half = threadIdx.x / SUM_COLS;
    const uint64_t per = (n + gridDim.x - 1) / gridDim.x;
    const uint64_t lo = per * blockIdx.x < n ? per * blockIdx.x : n;
    const uint64_t hi = lo + per < n ? lo + per : n;
    u16x2 acc[4] = {u16x2{0, 0}, u16x2{0, 0}, u16x2{0, 0}, u16x2{0, 0}};
    uint64_t r = lo + half;
    for (; r + (SUM_AHEAD - 1) * SUM_HALVES < hi; r += SUM_AHEAD * SUM_HALVES) {
        uint4 v[SUM_AHEAD];
#pragma unroll
        for (int k = 0; k < SUM_AHEAD; k++) v[k] = load_once(&rows[(r + k * SUM_HALVES) * SUM_COLS + c]);
#pragma unroll
        for (int k = 0; k < SUM_AHEAD; k++) add_packed(acc, v[k]);
    }
    for (; r < hi; r += SUM_HALVES) add_packed(acc, load_once(&rows[r * SUM_COLS + c]));
    __shared__ uint4 lds[SUM_COLS];
    const uint4 mine = make_uint4((uint32_t)acc[0].x | ((uint32_t)acc[0].y << 16), (uint32_t)acc[1].x | ((uint32_t)acc[1].y << 16),
                                  (uint32_t)acc[2].x | ((uint32_t)acc[2].y << 16), (uint32_t)acc[3].x | ((uint32_t)acc[3].y << 16));
    if (half == 1) lds[c] = mine;
    __syncthreads();
    if (half == 0) {
        add_packed(acc, lds[c]);
        part_out[(uint64_t)blockIdx.x * SUM_COLS + c] =
            make_uint4((uint32_t)acc[0].x | ((uint32_t)acc[0].y << 16), (uint32_t)acc[1].x | ((uint32_t)acc[1].y << 16),
                       (uint32_t)acc[2].x | ((uint32_t)acc[2].y << 16), (uint32_t)acc[3].x | ((uint32_t)acc[3].y << 16));
    }
}

// out[g][c] = sum over the partial sums p of group g of part[p][c] (packed uint16 pairs), c < 512;
// group g = rows [g * rows_per_group, (g + 1) * rows_per_group), g = blockIdx.y.  Each workgroup
// owns FOLD_COLS columns; its lanes split the rows eight ways and keep eight loads in flight
// (one at a time, 513 rows took 21 us: a load's latency per eight rows).  add_to_out: the sums are
// added to what out holds (a running sum) instead of replacing it.
__global__ void __launch_bounds__(FOLD_WG)
lthash_fold_kernel(const uint32_t *part, uint32_t n_part, uint32_t rows_per_group, uint16_t *out, bool add_to_out)
{
    constexpr int ROWS = FOLD_WG / FOLD_COLS;
    constexpr int AHEAD = 8;
    const uint32_t col = blockIdx.x * FOLD_COLS + (threadIdx.x % FOLD_COLS);
    const uint32_t row0 = threadIdx.x / FOLD_COLS;
    const uint64_t first = (uint64_t)blockIdx.y * rows_per_group;
    const uint64_t end = first + rows_per_group < n_part ? first + rows_per_group : n_part;
    u16x2 s = u16x2{0, 0};
    for (uint64_t p = first + row0; p < end; p += ROWS * AHEAD) {
        uint32_t x[AHEAD];
#pragma unroll
        for (int k = 0; k < AHEAD; k++) {
            const uint64_t q = p + (uint64_t)k * ROWS;
            x[k] = q < end ? part[q * LANE_WORDS + col] : 0u;
        }
#pragma unroll
        for (int k = 0; k < AHEAD; k++) s += u16x2{(unsigned short)x[k], (unsigned short)(x[k] >> 16)};
    }
    __shared__ uint32_t lds[ROWS][FOLD_COLS];
    lds[row0][threadIdx.x % FOLD_COLS] = (uint32_t)s.x | ((uint32_t)s.y << 16);
    __syncthreads();
    if (row0 == 0) {
        u16x2 t = u16x2{0, 0};
#pragma unroll
        for (int r = 0; r < ROWS; r++) {
            const uint32_t x = lds[r][threadIdx.x];
            t += u16x2{(unsigned short)x, (unsigned short)(x >> 16)};
        }
        uint16_t *o = out + (uint64_t)blockIdx.y * SENTRY_LANES;
        if (add_to_out) t += u16x2{o[2 * col], o[2 * col + 1]};
        o[2 * col] = t.x;            // 16-bit stores: out needs no more than 2-byte alignment
        o[2 * col + 1] = t.y;
    }
}

// acc[l] = acc[l] +/- x[l] mod 2^16: the lattice addition of section 4.2.2, two lanes per
// thread; the 16-bit lanes cannot carry into each other.
template <bool SUB>
__global__ void __launch_bounds__(LANE_WORDS)
lthash_addsub_kernel(uint16_t *acc, const uint16_t *x)
{
    const uint32_t c = threadIdx.x;
    u16x2 a = u16x2{acc[2 * c], acc[2 * c + 1]};
    u16x2 b = u16x2{x[2 * c], x[2 * c + 1]};
    u16x2 r = SUB ? (a - b) : (a + b);
    acc[2 * c] = r.x;
    acc[2 * c + 1] = r.y;
}

// ---------------------------------------------------------------------------
// mixed-source batches: one running sum per data source (section 4.1.2, section 4.3)
// ---------------------------------------------------------------------------
//
// The paper keeps a dictionary source -> samples of the batch and spawns one reduction tree
// per source.  Here the dictionary is a counting sort by source id done on the device (the
// ids are device memory, the host never sees them): count, scan, scatter.  Each source's
// records are then cut into units of `unit` records; one wave expands and sums one unit in
// registers exactly as in lthash_expand_kernel and writes a 2 KiB partial row; the rows of a
// source are adjacent, and a last kernel adds them to that source's running sum.

constexpr int SRC_WG = 256;
constexpr uint32_t SRC_MAX_SOURCES = sentry::LT_MAX_SOURCES;

// tables (uint32), at fixed places whatever the number of sources:
//   count[4096] | cursor[4096] | ticket (+ padding) | start[4097] | unit_start[4097]
// count, cursor and ticket are zero between calls: the fill kernel clears them when the scratch is
// allocated, and every call puts back to zero what it used (the last count workgroup the ticket,
// the final fold the counts and cursors of its sources), which saves a launch per call.
constexpr uint32_t SRC_TICKET_AT = 2 * SRC_MAX_SOURCES;
constexpr uint32_t SRC_START_AT = SRC_TICKET_AT + 64;
constexpr uint32_t SRC_UNIT_START_AT = SRC_START_AT + SRC_MAX_SOURCES + 1;
constexpr uint32_t SRC_TABLE_WORDS = SRC_UNIT_START_AT + SRC_MAX_SOURCES + 1;
__device__ __forceinline__ uint32_t *tab_count(uint32_t *t, uint32_t) { return t; }
__device__ __forceinline__ uint32_t *tab_cursor(uint32_t *t, uint32_t) { return t + SRC_MAX_SOURCES; }
__device__ __forceinline__ uint32_t *tab_ticket(uint32_t *t) { return t + SRC_TICKET_AT; }
__device__ __forceinline__ uint32_t *tab_start(uint32_t *t, uint32_t) { return t + SRC_START_AT; }
__device__ __forceinline__ uint32_t *tab_unit_start(uint32_t *t, uint32_t) { return t + SRC_UNIT_START_AT; }

__global__ void __launch_bounds__(SRC_WG)
src_zero_kernel(uint32_t *tables, uint32_t n_words)
{
    for (uint32_t i = blockIdx.x * SRC_WG + threadIdx.x; i < n_words; i += gridDim.x * SRC_WG) tables[i] = 0;
}

// Counts and ranks are first taken in LDS per workgroup tile, so that a source with many
// records costs one global atomic per tile instead of one per record.
constexpr int SRC_ITEMS = 8;                      // records per lane
constexpr int SRC_TILE = SRC_WG * SRC_ITEMS;      // records per workgroup

// start[] = exclusive scan of count[], unit_start[] = exclusive scan of ceil(count/unit); both get a
// closing total.  All lanes of one workgroup.
__device__ __forceinline__ void src_plan(uint32_t S, uint32_t unit, uint32_t *tables, uint32_t *sum_c, uint32_t *sum_u)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t per = (S + SRC_WG - 1) / SRC_WG;
    const uint32_t lo = tid * per, hi = lo + per < S ? lo + per : S;
    uint32_t c = 0, u = 0;
    for (uint32_t k = lo; k < hi; k++) {
        const uint32_t x = tab_count(tables, S)[k];
        c += x;
        u += (x + unit - 1) / unit;
    }
    sum_c[tid] = c;
    sum_u[tid] = u;
    __syncthreads();
    if (tid == 0) {
        uint32_t ac = 0, au = 0;
        for (int t = 0; t < SRC_WG; t++) {
            const uint32_t xc = sum_c[t], xu = sum_u[t];
            sum_c[t] = ac; sum_u[t] = au;
            ac += xc; au += xu;
        }
        tab_start(tables, S)[S] = ac;
        tab_unit_start(tables, S)[S] = au;
    }
    __syncthreads();
    c = sum_c[tid];
    u = sum_u[tid];
    for (uint32_t k = lo; k < hi; k++) {
        const uint32_t x = tab_count(tables, S)[k];
        tab_start(tables, S)[k] = c;
        tab_unit_start(tables, S)[k] = u;
        c += x;
        u += (x + unit - 1) / unit;
    }
}

// Counts per source; the workgroup that finishes last (a ticket counter, as in the one-launch Merkle
// tree) turns them into the plan, so that no launch of its own is needed for that.  The work of
// workgroup `block` of `n_blocks` (SRC_WG lanes each); hist: LDS, max(S, 2 * SRC_WG) words.
__device__ __forceinline__ void src_count_block(const uint32_t *src, uint64_t n, uint32_t S, uint32_t unit, uint32_t *tables,
                                                uint32_t block, uint32_t n_blocks, uint32_t *hist, uint32_t *last)
{
    for (uint32_t k = threadIdx.x; k < S; k += SRC_WG) hist[k] = 0;
    __syncthreads();
    const uint64_t tile = (uint64_t)block * SRC_TILE;
#pragma unroll
    for (int q = 0; q < SRC_ITEMS; q++) {
        const uint64_t i = tile + (uint64_t)q * SRC_WG + threadIdx.x;
        if (i < n) {
            const uint32_t k = src[i];
            if (k < S) atomicAdd(&hist[k], 1u);
        }
    }
    __syncthreads();
    for (uint32_t k = threadIdx.x; k < S; k += SRC_WG)
        if (hist[k]) atomicAdd(&tab_count(tables, S)[k], hist[k]);
    __threadfence();          // this workgroup's counts are visible to the device before its ticket
    __syncthreads();
    if (threadIdx.x == 0) *last = atomicAdd(tab_ticket(tables), 1u) == n_blocks - 1;
    __syncthreads();
    if (!*last) return;
    __threadfence();          // the counts of all other workgroups are read from memory, not from a stale line
    src_plan(S, unit, tables, hist, hist + SRC_WG);
    if (threadIdx.x == 0) *tab_ticket(tables) = 0;
}

__global__ void __launch_bounds__(SRC_WG)
src_count_kernel(const uint32_t *src, uint64_t n, uint32_t S, uint32_t unit, uint32_t *tables)
{
    __shared__ uint32_t hist[SRC_MAX_SOURCES];
    __shared__ uint32_t last;
    src_count_block(src, n, S, unit, tables, blockIdx.x, gridDim.x, hist, &last);
}

// Places of the records of tile `block` (WG * SRC_ITEMS records) in the order by source; WG lanes;
// cnt: LDS, S words (records of source k in this tile, then the tile's base).
template <int WG>
__device__ __forceinline__ void src_scatter_block(const uint32_t *src, uint64_t n, uint32_t S, uint32_t *tables, uint32_t *perm,
                                                  uint32_t block, uint32_t *cnt)
{
    for (uint32_t k = threadIdx.x; k < S; k += WG) cnt[k] = 0;
    __syncthreads();
    const uint64_t tile = (uint64_t)block * (WG * SRC_ITEMS);
    uint32_t key[SRC_ITEMS], rank[SRC_ITEMS];
#pragma unroll
    for (int q = 0; q < SRC_ITEMS; q++) {
        const uint64_t i = tile + (uint64_t)q * WG + threadIdx.x;
        key[q] = 0xffffffffu;
        rank[q] = 0;
        if (i < n) {
            const uint32_t k = src[i];
            if (k < S) { key[q] = k; rank[q] = atomicAdd(&cnt[k], 1u); }
        }
    }
    __syncthreads();
    for (uint32_t k = threadIdx.x; k < S; k += WG)
        if (cnt[k]) cnt[k] = tab_start(tables, S)[k] + atomicAdd(&tab_cursor(tables, S)[k], cnt[k]);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < SRC_ITEMS; q++) {
        const uint64_t i = tile + (uint64_t)q * WG + threadIdx.x;
        if (key[q] != 0xffffffffu) perm[cnt[key[q]] + rank[q]] = (uint32_t)i;
    }
}

__global__ void __launch_bounds__(SRC_WG)
src_scatter_kernel(const uint32_t *src, uint64_t n, uint32_t S, uint32_t *tables, uint32_t *perm)
{
    __shared__ uint32_t cnt[SRC_MAX_SOURCES];
    src_scatter_block<SRC_WG>(src, n, S, tables, perm, blockIdx.x, cnt);
}

// A small batch over few sources: the whole sort is the work of one wave, and it does not depend
// on the root hashes, so it rides along in their launch as one more workgroup (the root hashes of
// such a batch are one wave per SIMD at most and last as long as one record's chain: 37 us for a
// 3 KiB sample, behind which the sort's 5 us disappear, and with them two launches of 6 us each).
constexpr uint32_t RIDER_MAX_RECORDS = 8192;          // one wave sorts them in 20 us, and their root hashes are still one wave per SIMD
constexpr uint32_t RIDER_MAX_SOURCES = ROOT4_RECORDS * 128 / 8;       // two tables of words in the root kernel's LDS
static_assert(RIDER_MAX_RECORDS <= FEW_RECORDS, "the batch of a rider always takes the four-lane path");

struct SourceSort {
    const uint32_t *src;      // source id per record
    uint32_t n, S, unit;
    uint32_t *tables;         // start[] and unit_start[] are written; count[], cursor[] and the ticket stay zero
    uint32_t *perm;
};

// All 64 lanes of a one-wave workgroup; lds holds 2 * RIDER_MAX_SOURCES words.
__device__ __forceinline__ void src_sort_one_wave(const SourceSort &j, uint32_t *lds)
{
    uint32_t *hist = lds, *cur = lds + RIDER_MAX_SOURCES;
    const uint32_t lane = threadIdx.x, S = j.S;
    constexpr int AHEAD = 32;                                       // ids in flight per lane: 8192 records are four trips in all
    for (uint32_t k = lane; k < S; k += 64) hist[k] = 0;
    __syncthreads();
    for (uint32_t i0 = lane; i0 < j.n; i0 += 64 * AHEAD) {
        uint32_t k[AHEAD];
#pragma unroll
        for (int a = 0; a < AHEAD; a++) k[a] = i0 + 64 * a < j.n ? j.src[i0 + 64 * a] : 0xffffffffu;
#pragma unroll
        for (int a = 0; a < AHEAD; a++)
            if (k[a] < S) atomicAdd(&hist[k[a]], 1u);
    }
    __syncthreads();
    // exclusive scans of the counts and of the units they make; lane l owns sources 4l .. 4l+3
    constexpr int OWN = RIDER_MAX_SOURCES / 64;
    uint32_t c[OWN], sum_c = 0, sum_u = 0;
#pragma unroll
    for (int q = 0; q < OWN; q++) {
        const uint32_t k = OWN * lane + q;
        c[q] = k < S ? hist[k] : 0;
        sum_c += c[q];
        sum_u += (c[q] + j.unit - 1) / j.unit;
    }
    uint32_t inc_c = sum_c, inc_u = sum_u;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t tc = (uint32_t)__shfl_up((int)inc_c, d, 64), tu = (uint32_t)__shfl_up((int)inc_u, d, 64);
        if (lane >= (uint32_t)d) { inc_c += tc; inc_u += tu; }
    }
    uint32_t at_c = inc_c - sum_c, at_u = inc_u - sum_u;
#pragma unroll
    for (int q = 0; q < OWN; q++) {
        const uint32_t k = OWN * lane + q;
        if (k < S) {
            tab_start(j.tables, S)[k] = at_c;
            tab_unit_start(j.tables, S)[k] = at_u;
            cur[k] = at_c;
        }
        at_c += c[q];
        at_u += (c[q] + j.unit - 1) / j.unit;
    }
    if (lane == 63) {
        tab_start(j.tables, S)[S] = inc_c;
        tab_unit_start(j.tables, S)[S] = inc_u;
    }
    __syncthreads();
    for (uint32_t i0 = lane; i0 < j.n; i0 += 64 * AHEAD) {
        uint32_t k[AHEAD];
#pragma unroll
        for (int a = 0; a < AHEAD; a++) k[a] = i0 + 64 * a < j.n ? j.src[i0 + 64 * a] : 0xffffffffu;
#pragma unroll
        for (int a = 0; a < AHEAD; a++)
            if (k[a] < S) j.perm[atomicAdd(&cur[k[a]], 1u)] = i0 + 64 * a;
    }
}

// The four-lane root hashes of a batch of at most RIDER_MAX_RECORDS records, and in the last
// workgroup the sort of the batch by source.
__global__ void __launch_bounds__(ROOT4_WG)
lthash_root4_rider_kernel(const uint8_t *records, const uint64_t *offsets, uint64_t offset_base, uint64_t n,
                          uint64_t *h0_out, uint64_t p0, uint64_t p1, SourceSort sort)
{
    __shared__ __attribute__((aligned(16))) unsigned char stage[ROOT4_RECORDS * 128];
    static_assert(ROOT4_WG == 64, "the rider is written for a workgroup of one wave");
    if (blockIdx.x == gridDim.x - 1) {
        src_sort_one_wave(sort, reinterpret_cast<uint32_t *>(stage));
        return;
    }
    root_four_lanes(records, offsets, offset_base, n, nullptr, h0_out, (uint64_t)blockIdx.x * ROOT4_RECORDS, stage, p0, p1);
}

// Larger batches over few sources, for which both root kernels are launched: the count by source
// rides at the front of the one-lane launch and the scatter at the front of the four-lane launch,
// which follows it on the stream.  Whichever of the two kernels hashes the batch, one of the
// steps hides behind it and neither needs a launch of its own (50,000 samples of 3 KiB over 16
// sources: two launches of 11 and 4 us less).
static_assert(ROOT1_WG == SRC_WG, "the count rides in workgroups of the one-lane root kernel");
static_assert(RIDER_MAX_SOURCES <= 2 * SRC_WG, "the count's LDS table doubles as the plan's two scan arrays");

__global__ void __launch_bounds__(ROOT1_WG)
lthash_root1_count_kernel(const uint8_t *records, const uint64_t *offsets, uint64_t offset_base, uint64_t n, uint64_t *h0_out,
                          uint64_t p0, uint64_t p1, SourceSort sort, uint32_t n_count)
{
    __shared__ uint32_t hist[2 * SRC_WG];
    __shared__ uint32_t last;
    if (blockIdx.x < n_count) {
        src_count_block(sort.src, sort.n, sort.S, sort.unit, sort.tables, blockIdx.x, n_count, hist, &last);
        return;
    }
    if (offsets && four_lane_mode(offsets, n)) return;
    root_one_lane(records, offsets, offset_base, n, h0_out, (uint64_t)(blockIdx.x - n_count) * ROOT1_WG + threadIdx.x, p0, p1);
}

__global__ void __launch_bounds__(ROOT4_WG)
lthash_root4_scatter_kernel(const uint8_t *records, const uint64_t *offsets, uint64_t offset_base, uint64_t n,
                            const uint32_t *order, uint64_t *h0_out, uint64_t p0, uint64_t p1, SourceSort sort, uint32_t n_scatter)
{
    __shared__ __attribute__((aligned(16))) unsigned char stage[ROOT4_RECORDS * 128];
    static_assert(RIDER_MAX_SOURCES * 4 <= ROOT4_RECORDS * 128, "the scatter's table lies in the root kernel's LDS");
    if (blockIdx.x < n_scatter) {
        src_scatter_block<ROOT4_WG>(sort.src, sort.n, sort.S, sort.tables, sort.perm, blockIdx.x, reinterpret_cast<uint32_t *>(stage));
        return;
    }
    if (offsets && !four_lane_mode(offsets, n)) return;
    root_four_lanes(records, offsets, offset_base, n, offsets && ordered_mode(offsets, n) ? order : nullptr, h0_out,
                    (uint64_t)(blockIdx.x - n_scatter) * ROOT4_RECORDS, stage, p0, p1);
}

// One wave per unit.  Lane l owns output block l & 31 and takes every second record of the
// unit; the order of the records inside a source does not matter for the sum.
__global__ void __launch_bounds__(EXP_WG)
lthash_expand_units_kernel(const uint64_t *h0, const uint32_t *perm, uint32_t S, uint32_t unit,
                           uint32_t *tables, uint32_t *part_out)
{
    const uint32_t lane = threadIdx.x & 63, j = lane & 31;
    const uint32_t u = blockIdx.x * EXP_WAVES + (threadIdx.x >> 6);
    const uint32_t *unit_start = tab_unit_start(tables, S);
    if (u >= unit_start[S]) return;                     // wave-uniform
    // the source whose unit range holds u: the last k with unit_start[k] <= u.  The whole wave looks
    // for it: every lane reads the first entry of one of 64 stretches of the table, then the lanes
    // read the stretch that holds it (two loads one behind the other where a bisection has twelve).
    const uint32_t stretch = (S + 63) / 64;
    const uint32_t at1 = lane * stretch;
    const uint32_t v1 = at1 < S ? unit_start[at1] : 0xffffffffu;
    uint32_t k = (uint32_t)__popcll(__ballot(v1 <= u)) - 1;             // unit_start[0] = 0: at least lane 0
    if (stretch > 1) {
        const uint32_t at2 = k * stretch + lane;
        const uint32_t v2 = lane < stretch && at2 < S ? unit_start[at2] : 0xffffffffu;
        k = k * stretch + (uint32_t)__popcll(__ballot(v2 <= u)) - 1;
    }
    const uint32_t *start = tab_start(tables, S);
    const uint32_t first = start[k] + (u - unit_start[k]) * unit;
    const uint32_t stop = first + unit < start[k + 1] ? first + unit : start[k + 1];
    u16x2 acc[16];
#pragma unroll
    for (int q = 0; q < 16; q++) acc[q] = u16x2{0, 0};
    for (uint32_t r = first + (lane >> 5); r < stop; r += 2) {
        const uint64_t rec = perm[r];
        uint64_t m[16];
#pragma unroll
        for (int q = 0; q < 8; q++) { m[q] = h0[8 * rec + q]; m[8 + q] = 0; }
        uint64_t h[8];
#pragma unroll
        for (int q = 0; q < 8; q++) h[q] = b2_iv(q);
        h[0] ^= EXP_P0;
        h[1] ^= EXP_P1_HI | (uint64_t)j;
        h[2] ^= EXP_P2;
        blake2b_compress(h, m, 64, true);
#pragma unroll
        for (int q = 0; q < 8; q++) {
            const uint32_t l32 = (uint32_t)h[q], h32 = (uint32_t)(h[q] >> 32);
            acc[2 * q] += u16x2{(unsigned short)l32, (unsigned short)(l32 >> 16)};
            acc[2 * q + 1] += u16x2{(unsigned short)h32, (unsigned short)(h32 >> 16)};
        }
    }
#pragma unroll
    for (int q = 0; q < 16; q++) {
        const uint32_t x = (uint32_t)acc[q].x | ((uint32_t)acc[q].y << 16);
        const uint32_t y = (uint32_t)__shfl_xor((int)x, 32, 64);
        const u16x2 t = acc[q] + u16x2{(unsigned short)y, (unsigned short)(y >> 16)};
        if (lane < 32) part_out[(uint64_t)u * LANE_WORDS + 16 * j + q] = (uint32_t)t.x | ((uint32_t)t.y << 16);
    }
}

// acc[k][c] += sum of the partial rows of source k; grid = (512 / COLS, S), WG lanes a workgroup,
// which owns COLS packed words of one source and splits that source's rows WG / COLS ways.  A
// source's rows are the work of one workgroup per column block, whatever its share of the batch,
// and the launch waits for the largest share: where the sources have many rows each the larger
// workgroup keeps four times as many loads in flight (50,000 samples, uneven shares: 16 sources
// 0.230 -> 0.219 ms for the call, four 0.249 -> 0.222 ms, two 0.287 -> 0.232 ms; column blocks a
// quarter as wide, which make four times as many workgroups of a handful of sources, added nothing).
template <int WG, int COLS>
__global__ void __launch_bounds__(WG)
lthash_fold_sources_kernel(const uint32_t *part, uint32_t S, uint32_t *tables, uint16_t *acc)
{
    constexpr int ROWS = WG / COLS;
    const uint32_t k = blockIdx.y;
    const uint32_t c = threadIdx.x % COLS;
    const uint32_t col = blockIdx.x * COLS + c;
    const uint32_t row0 = threadIdx.x / COLS;
    const uint32_t *unit_start = tab_unit_start(tables, S);
    const uint32_t u0 = unit_start[k], u1 = unit_start[k + 1];
    if (blockIdx.x == 0 && threadIdx.x == 0) {          // nothing reads them any more: zero for the next call
        tab_count(tables, S)[k] = 0;
        tab_cursor(tables, S)[k] = 0;
    }
    if (u0 == u1) return;                               // no record of this source in the batch
    constexpr int AHEAD = 8;                            // loads in flight per lane, as in lthash_fold_kernel
    u16x2 s = u16x2{0, 0};
    for (uint32_t u = u0 + row0; u < u1; u += ROWS * AHEAD) {
        uint32_t x[AHEAD];
#pragma unroll
        for (int a = 0; a < AHEAD; a++) {
            const uint32_t q = u + (uint32_t)a * ROWS;
            x[a] = q < u1 ? part[(uint64_t)q * LANE_WORDS + col] : 0u;
        }
#pragma unroll
        for (int a = 0; a < AHEAD; a++) s += u16x2{(unsigned short)x[a], (unsigned short)(x[a] >> 16)};
    }
    __shared__ uint32_t lds[ROWS][COLS];
    lds[row0][c] = (uint32_t)s.x | ((uint32_t)s.y << 16);
    __syncthreads();
    if (row0 == 0) {
        u16x2 t = u16x2{0, 0};
        for (int r = 0; r < ROWS; r++) {
            const uint32_t x = lds[r][c];
            t += u16x2{(unsigned short)x, (unsigned short)(x >> 16)};
        }
        uint16_t *row = acc + (uint64_t)k * SENTRY_LANES;
        row[2 * col] = (uint16_t)(row[2 * col] + t.x);
        row[2 * col + 1] = (uint16_t)(row[2 * col + 1] + t.y);
    }
}

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

int g_cu_count = 0;
inline int cu_count() { return sentry::lthash_cu_count(); }

}  // namespace

namespace sentry {

int lthash_cu_count()
{
    if (!g_cu_count) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            g_cu_count = n;
        else
            g_cu_count = 256;
    }
    return g_cu_count;
}

// Grow the per-record scratch once for the largest batch of a pipelined run.
int lthash_presize(uint64_t max_records, hipStream_t s)
{
    void *p;
    int rc = scratch_get(s, R_LT_H0, 64 * (max_records ? max_records : 1), &p);
    if (rc) return rc;
    if ((rc = scratch_get(s, R_LT_ORDER, 4 * (max_records ? max_records : 1), &p))) return rc;
    if ((rc = scratch_get(s, R_LT_COUNTS, 4 * (size_t)SORT_MAX_GROUPS * SORT_BINS, &p))) return rc;
    // the most partial rows any launch writes: two workgroups per CU, plus the running sum
    return scratch_get(s, R_LT_PART, ((size_t)cu_count() * 2 + 1) * LANE_WORDS * 4, &p);
}

// The same, and the partial rows of the lane sum over stored digests (four workgroups per CU and
// their group sums): everything the lattice calls on device-resident records of up to max_records
// take from the stream's scratch.
int lthash_reserve(uint64_t max_records, hipStream_t s)
{
    int rc = lthash_presize(max_records, s);
    if (rc) return rc;
    void *p;
    const uint64_t rows = (uint64_t)cu_count() * 4;
    return scratch_get(s, R_LT_PART, (rows + ceil_div(rows, 64) + 1) * LANE_WORDS * 4, &p);
}

// out = lane-wise sum of n_rows rows of 1024 lanes (rows are 2048 bytes apart, 4-byte aligned).
// Many rows are folded in two steps, groups of FOLD_GROUP rows first; `spare` then holds the group
// sums (ceil(n_rows / FOLD_GROUP) rows) and is not used otherwise.
constexpr uint32_t FOLD_GROUP = 64;
constexpr uint32_t FOLD_DIRECT = 640;     // up to here one launch (ten trips of 64 rows per workgroup)

static uint32_t fold_spare_rows(uint64_t n_rows) { return n_rows > FOLD_DIRECT ? (uint32_t)ceil_div(n_rows, FOLD_GROUP) : 0; }

static int fold_rows(const uint32_t *rows, uint32_t n_rows, uint32_t *spare, uint16_t *out, hipStream_t s,
                     bool add_to_out = false)
{
    if (n_rows > FOLD_DIRECT) {
        const uint32_t groups = fold_spare_rows(n_rows);
        hipLaunchKernelGGL(lthash_fold_kernel, dim3(LANE_WORDS / FOLD_COLS, groups), dim3(FOLD_WG), 0, s, rows, n_rows,
                           FOLD_GROUP, reinterpret_cast<uint16_t *>(spare), false);
        rows = spare;
        n_rows = groups;
    }
    hipLaunchKernelGGL(lthash_fold_kernel, dim3(LANE_WORDS / FOLD_COLS, 1), dim3(FOLD_WG), 0, s, rows, n_rows,
                       n_rows ? n_rows : 1u, out, add_to_out);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

int lthash_sum_rows(const uint16_t *rows, uint32_t n_rows, uint16_t *out, hipStream_t s)
{
    if (n_rows > FOLD_DIRECT) {
        set_error("lthash_sum_rows: at most %u rows", FOLD_DIRECT);
        return SENTRY_ERR_INVALID_ARG;
    }
    return fold_rows(reinterpret_cast<const uint32_t *>(rows), n_rows, nullptr, out, s);
}

// The three launches that put the records in length order for the four-lane path (see above).
static int launch_ordering(const uint64_t *dev_offsets, uint64_t n, hipStream_t s, void **order)
{
    void *counts;
    int rc;
    if ((rc = scratch_get(s, R_LT_ORDER, 4 * n, order))) return rc;
    uint32_t groups = (uint32_t)ceil_div(n, SORT_MIN_RUN);
    if (groups > SORT_MAX_GROUPS) groups = SORT_MAX_GROUPS;
    if ((rc = scratch_get(s, R_LT_COUNTS, 4 * (size_t)SORT_MAX_GROUPS * SORT_BINS, &counts))) return rc;
    hipLaunchKernelGGL(lthash_order_count_kernel, dim3(groups), dim3(SORT_WG), 0, s, dev_offsets, n, static_cast<uint32_t *>(counts));
    hipLaunchKernelGGL(lthash_order_scan_kernel, dim3(1), dim3(SORT_WG), 0, s, dev_offsets, n, static_cast<uint32_t *>(counts), groups);
    hipLaunchKernelGGL(lthash_order_place_kernel, dim3(groups), dim3(SORT_WG), 0, s, dev_offsets, n,
                       static_cast<const uint32_t *>(counts), static_cast<uint32_t *>(*order));
    return SENTRY_OK;
}

// The root hashes as lthash_roots launches them, with the sort by source riding in the two root
// launches (see lthash_root1_count_kernel).  Up to FEW_RECORDS records the one-lane kernel has
// nothing to hash: its launch is then the count alone, and the scatter still rides.
static int lthash_roots_sorting(const void *dev_records, const uint64_t *dev_offsets, uint64_t n, uint64_t *h0, hipStream_t s,
                                const SourceSort &sort)
{
    void *order = nullptr;
    int rc;
    if (n > ORDER_MIN_RECORDS && (rc = launch_ordering(dev_offsets, n, s, &order))) return rc;
    const uint32_t n_count = (uint32_t)ceil_div(n, SRC_TILE), n_scatter = (uint32_t)ceil_div(n, ROOT4_WG * SRC_ITEMS);
    const uint32_t root1_blocks = n > FEW_RECORDS ? (uint32_t)ceil_div(n, ROOT1_WG) : 0;
    hipLaunchKernelGGL(lthash_root1_count_kernel, dim3(root1_blocks + n_count), dim3(ROOT1_WG), 0, s,
                       static_cast<const uint8_t *>(dev_records), dev_offsets, (uint64_t)0, n, h0, LT_ROOT_P0, LT_ROOT_P1, sort, n_count);
    hipLaunchKernelGGL(lthash_root4_scatter_kernel, dim3((uint32_t)ceil_div(n, ROOT4_RECORDS) + n_scatter), dim3(ROOT4_WG), 0, s,
                       static_cast<const uint8_t *>(dev_records), dev_offsets, (uint64_t)0, n, static_cast<const uint32_t *>(order),
                       h0, LT_ROOT_P0, LT_ROOT_P1, sort, n_scatter);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

// Root hashes (64 bytes each) of n records at dev_records (offsets relative to offset_base).
int lthash_roots(const void *dev_records, const uint64_t *dev_offsets, uint64_t offset_base, uint64_t n,
                 uint64_t *h0, hipStream_t s, uint64_t p0, uint64_t p1)
{
    if (n == 0) return SENTRY_OK;
    // Both root kernels are launched; the device takes one path (see four_lane_mode).  The
    // four-lane path is kept for any number of long records: in length order it sustains
    // 1.7 TB/s, while one lane per record, which issues fewer instructions, has chains three
    // times as long and reaches that rate only with millions of records.
    void *order = nullptr;
    int rc;
    // Up to one wave per SIMD (16 records a wave) every wave has a SIMD to itself and the launch lasts as
    // long as its longest record whatever the order: no ordering then, which takes three launches
    // out of the way of a small batch.
    if (n > ORDER_MIN_RECORDS && (rc = launch_ordering(dev_offsets, n, s, &order))) return rc;
    if (n > FEW_RECORDS)   // up to there the device always takes the four-lane path: nothing for this kernel to do
        hipLaunchKernelGGL(lthash_root1_kernel, dim3((uint32_t)ceil_div(n, ROOT1_WG)), dim3(ROOT1_WG), 0, s,
                           static_cast<const uint8_t *>(dev_records), dev_offsets, offset_base, n, h0, p0, p1);
    hipLaunchKernelGGL(lthash_root4_kernel, dim3((uint32_t)ceil_div(n, ROOT4_RECORDS)), dim3(ROOT4_WG), 0, s,
                       static_cast<const uint8_t *>(dev_records), dev_offsets, offset_base, n,
                       static_cast<const uint32_t *>(order), h0, p0, p1);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

// Root hashes of n records of record_bytes bytes each, back to back at dev_records.  The host
// knows all there is to know about such a batch, so only the kernel that the rules above pick is
// launched (four lanes for few records or long ones), and nothing is ordered: the records are equal.
int lthash_roots_fixed(const void *dev_records, uint64_t record_bytes, uint64_t n, uint64_t *h0, hipStream_t s,
                       uint64_t p0, uint64_t p1)
{
    if (n == 0) return SENTRY_OK;
    if (n <= FEW_RECORDS || record_bytes >= FOUR_LANE_MEAN_BYTES)
        hipLaunchKernelGGL(lthash_root4_kernel, dim3((uint32_t)ceil_div(n, ROOT4_RECORDS)), dim3(ROOT4_WG), 0, s,
                           static_cast<const uint8_t *>(dev_records), (const uint64_t *)nullptr, record_bytes, n,
                           (const uint32_t *)nullptr, h0, p0, p1);
    else
        hipLaunchKernelGGL(lthash_root1_kernel, dim3((uint32_t)ceil_div(n, ROOT1_WG)), dim3(ROOT1_WG), 0, s,
                           static_cast<const uint8_t *>(dev_records), (const uint64_t *)nullptr, record_bytes, n, h0, p0, p1);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

// Expansion of n root hashes and the lane sum over them, written to out or (accumulate) added to it.
// only_source0: device array of n source ids, records with another id are left out; or NULL.
int lthash_expand_and_fold(const uint64_t *h0, uint64_t n, const uint32_t *only_source0, uint16_t *out,
                                  bool accumulate, hipStream_t s)
{
    // expansion grid: enough workgroups to give every SIMD two waves, no more than the work
    const uint64_t slots = ceil_div(n, 2);                        // one wave pass = two records
    uint64_t grid = ceil_div(slots, EXP_WAVES);
    const uint64_t cap = (uint64_t)cu_count() * 2;
    if (grid > cap) grid = cap;
    if (grid == 0) grid = 1;
    void *part;
    int rc = scratch_get(s, R_LT_PART, grid * LANE_WORDS * 4, &part);
    if (rc) return rc;
    if (only_source0)
        hipLaunchKernelGGL(lthash_expand_kernel<true>, dim3((uint32_t)grid), dim3(EXP_WG), 0, s, h0, n,
                           static_cast<uint32_t *>(part), only_source0);
    else
        hipLaunchKernelGGL(lthash_expand_kernel<false>, dim3((uint32_t)grid), dim3(EXP_WG), 0, s, h0, n,
                           static_cast<uint32_t *>(part), (const uint32_t *)nullptr);
    SENTRY_HIP_CHECK(hipGetLastError());
    return fold_rows(static_cast<const uint32_t *>(part), (uint32_t)grid, nullptr, out, s, accumulate);   // grid <= 512
}

// Lattice hash of n records at dev_records (offsets relative to offset_base; or, with
// dev_offsets == nullptr, records of offset_base bytes each, back to back); result either
// overwrites out (accumulate == false) or is added to it lane-wise.
int lthash_into(const void *dev_records, const uint64_t *dev_offsets, uint64_t offset_base, uint64_t n,
                uint16_t *out, bool accumulate, hipStream_t s)
{
    void *h0;
    int rc = scratch_get(s, R_LT_H0, 64 * (n ? n : 1), &h0);
    if (rc) return rc;
    rc = dev_offsets ? lthash_roots(dev_records, dev_offsets, offset_base, n, static_cast<uint64_t *>(h0), s)
                     : lthash_roots_fixed(dev_records, offset_base, n, static_cast<uint64_t *>(h0), s);
    if (rc) return rc;
    return lthash_expand_and_fold(static_cast<const uint64_t *>(h0), n, nullptr, out, accumulate, s);
}

}  // namespace sentry

extern "C" {

int sentry_lthash(const void *dev_records, const uint64_t *dev_offsets, size_t n, uint16_t *out_lanes, void *stream)
{
    sentry::clear_error();
    SENTRY_REQUIRE(out_lanes != nullptr && (reinterpret_cast<uintptr_t>(out_lanes) & 1) == 0,
                   "sentry_lthash: out_lanes must be non-NULL and 2-byte aligned");
    SENTRY_REQUIRE(n == 0 || (dev_offsets != nullptr && (reinterpret_cast<uintptr_t>(dev_offsets) & 7) == 0),
                   "sentry_lthash: dev_offsets must be non-NULL and 8-byte aligned when n > 0");
    // a launch holds fewer than 2^32 work-items in all
    SENTRY_REQUIRE(n <= 0xffffffffull / 4 - 64, "sentry_lthash: too many records");
    return sentry::lthash_into(dev_records, dev_offsets, 0, n, out_lanes, false, static_cast<hipStream_t>(stream));
}

int sentry_lthash_digests(const void *dev_records, const uint64_t *dev_offsets, size_t n, uint16_t *out_digests,
                          void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n == 0) return SENTRY_OK;
    SENTRY_REQUIRE(out_digests != nullptr && (reinterpret_cast<uintptr_t>(out_digests) & 15) == 0,
                   "sentry_lthash_digests: out_digests must be non-NULL and 16-byte aligned");
    SENTRY_REQUIRE(dev_offsets != nullptr && (reinterpret_cast<uintptr_t>(dev_offsets) & 7) == 0,
                   "sentry_lthash_digests: dev_offsets must be non-NULL and 8-byte aligned");
    SENTRY_REQUIRE(n <= 0xffffffffull / 4 - 64, "sentry_lthash_digests: too many records");
    void *h0;
    int rc = sentry::scratch_get(s, sentry::R_LT_H0, 64 * n, &h0);
    if (rc) return rc;
    if ((rc = sentry::lthash_roots(dev_records, dev_offsets, 0, n, static_cast<uint64_t *>(h0), s))) return rc;
    uint64_t grid = ceil_div(ceil_div(n, 2), EXP_WAVES);
    const uint64_t cap = (uint64_t)cu_count() * 8;
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL(lthash_digests_kernel, dim3((uint32_t)grid), dim3(EXP_WG), 0, s, static_cast<const uint64_t *>(h0),
                       (uint64_t)n, reinterpret_cast<uint4 *>(out_digests));
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

int sentry_lthash_sum(const uint16_t *dev_digests, size_t n, uint16_t *out_lanes, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(out_lanes != nullptr && (reinterpret_cast<uintptr_t>(out_lanes) & 1) == 0,
                   "sentry_lthash_sum: out_lanes must be non-NULL and 2-byte aligned");
    SENTRY_REQUIRE(n == 0 || (dev_digests != nullptr && (reinterpret_cast<uintptr_t>(dev_digests) & 15) == 0),
                   "sentry_lthash_sum: dev_digests must be non-NULL and 16-byte aligned when n > 0");
    // enough workgroups to keep HBM busy (four per CU), each with at least one full trip of rows
    uint64_t grid = ceil_div(n, SUM_HALVES * SUM_AHEAD);
    const uint64_t cap = (uint64_t)cu_count() * 4;
    if (grid > cap) grid = cap;
    if (grid == 0) grid = 1;
    void *part;
    int rc = sentry::scratch_get(s, sentry::R_LT_PART, (grid + sentry::fold_spare_rows(grid)) * LANE_WORDS * 4, &part);
    if (rc) return rc;
    if (n)
        hipLaunchKernelGGL(lthash_sum_kernel, dim3((uint32_t)grid), dim3(SUM_WG), 0, s,
                           reinterpret_cast<const uint4 *>(dev_digests), (uint64_t)n, static_cast<uint4 *>(part));
    return sentry::fold_rows(static_cast<const uint32_t *>(part), (uint32_t)(n ? grid : 0),
                             static_cast<uint32_t *>(part) + grid * LANE_WORDS, out_lanes, s);
}

static int addsub(const char *fn, uint16_t *acc, const uint16_t *x, void *stream, bool sub)
{
    sentry::clear_error();
    SENTRY_REQUIRE(acc != nullptr && x != nullptr, "%s: NULL argument", fn);
    SENTRY_REQUIRE(((reinterpret_cast<uintptr_t>(acc) | reinterpret_cast<uintptr_t>(x)) & 1) == 0,
                   "%s: lanes must be 2-byte aligned", fn);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (sub)
        hipLaunchKernelGGL(lthash_addsub_kernel<true>, dim3(1), dim3(LANE_WORDS), 0, s, acc, x);
    else
        hipLaunchKernelGGL(lthash_addsub_kernel<false>, dim3(1), dim3(LANE_WORDS), 0, s, acc, x);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

int sentry_lthash_sources(const void *dev_records, const uint64_t *dev_offsets, const uint32_t *dev_source_ids,
                          size_t n, size_t n_sources, uint16_t *acc_lanes, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(n_sources >= 1 && n_sources <= SRC_MAX_SOURCES, "sentry_lthash_sources: n_sources must be 1..%u",
                   SRC_MAX_SOURCES);
    SENTRY_REQUIRE(acc_lanes != nullptr && (reinterpret_cast<uintptr_t>(acc_lanes) & 1) == 0,
                   "sentry_lthash_sources: acc_lanes must be non-NULL and 2-byte aligned");
    if (n == 0) return SENTRY_OK;
    SENTRY_REQUIRE(dev_offsets != nullptr && (reinterpret_cast<uintptr_t>(dev_offsets) & 7) == 0,
                   "sentry_lthash_sources: dev_offsets must be non-NULL and 8-byte aligned");
    SENTRY_REQUIRE(dev_source_ids != nullptr && (reinterpret_cast<uintptr_t>(dev_source_ids) & 3) == 0,
                   "sentry_lthash_sources: dev_source_ids must be non-NULL and 4-byte aligned");
    SENTRY_REQUIRE(n <= 0xffffffffull / 4 - 64, "sentry_lthash_sources: too many records");
    const uint32_t S = (uint32_t)n_sources;
    if (S == 1) {
        // one source: nothing to sort; the plain launches, with records of other ids left out, and
        // the lane sum added to the running sum
        void *h0;
        int rc1 = sentry::scratch_get(s, sentry::R_LT_H0, 64 * n, &h0);
        if (rc1) return rc1;
        if ((rc1 = sentry::lthash_roots(dev_records, dev_offsets, 0, n, static_cast<uint64_t *>(h0), s))) return rc1;
        return sentry::lthash_expand_and_fold(static_cast<const uint64_t *>(h0), n, dev_source_ids, acc_lanes, true, s);
    }
    // Records per unit (one wave expands one unit, two records per pass).  A SIMD works off whole
    // units and every unit costs its wave some 3 us of loads one behind the other before the first
    // pass, so there is a best size, found by timing units of 2 to 128 records on 9000 to 500,000
    // records: four records up to 65,536 (50,000 records: 0.235 ms for the call with units of 16,
    // 3125 units on 1024 SIMDs of which some then had four and the others waited; 0.225 ms with
    // units of 4; 0.230 ms with units of 2, which make 51 MB of partial rows), eight up to 131,072
    // and so on: at most 64 units per compute unit.  Up to two records per SIMD a unit is one pass:
    // with units of eight, 128 records made 16 waves of four compressions per lane each, 19 us
    // where 5 us do.
    uint32_t unit = n <= (uint64_t)cu_count() * 8 ? 2 : 4;
    while (ceil_div(n, unit) > (uint64_t)cu_count() * 64) unit *= 2;
    const uint64_t max_units = ceil_div(n, unit) + S;          // every source may end in a short unit
    void *h0, *part, *tables, *perm;
    int rc;
    if ((rc = sentry::scratch_get(s, sentry::R_LT_H0, 64 * n, &h0))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_LT_PART, max_units * LANE_WORDS * 4, &part))) return rc;
    bool fresh_tables;
    if ((rc = sentry::scratch_get_fresh(s, sentry::R_SRC_TABLES, 4 * (size_t)SRC_TABLE_WORDS, &tables, &fresh_tables))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_SRC_PERM, 4 * n, &perm))) return rc;
    uint32_t *tab = static_cast<uint32_t *>(tables);
    const uint32_t *src = dev_source_ids;
    const uint32_t scan_grid = (uint32_t)ceil_div(n, SRC_TILE);

    if (fresh_tables) hipLaunchKernelGGL(src_zero_kernel, dim3(1), dim3(SRC_WG), 0, s, tab, SRC_TABLE_WORDS);
    if (n <= RIDER_MAX_RECORDS && S <= RIDER_MAX_SOURCES) {
        // a small batch: root hashes and sort in one launch
        const SourceSort sort{src, (uint32_t)n, S, unit, tab, static_cast<uint32_t *>(perm)};
        hipLaunchKernelGGL(lthash_root4_rider_kernel, dim3((uint32_t)ceil_div(n, ROOT4_RECORDS) + 1), dim3(ROOT4_WG), 0, s,
                           static_cast<const uint8_t *>(dev_records), dev_offsets, (uint64_t)0, (uint64_t)n,
                           static_cast<uint64_t *>(h0), sentry::LT_ROOT_P0, sentry::LT_ROOT_P1, sort);
        rc = SENTRY_OK;
    } else if (S <= RIDER_MAX_SOURCES) {
        const SourceSort sort{src, (uint32_t)n, S, unit, tab, static_cast<uint32_t *>(perm)};
        rc = sentry::lthash_roots_sorting(dev_records, dev_offsets, n, static_cast<uint64_t *>(h0), s, sort);
    } else {
        hipLaunchKernelGGL(src_count_kernel, dim3(scan_grid), dim3(SRC_WG), 0, s, src, (uint64_t)n, S, unit, tab);
        hipLaunchKernelGGL(src_scatter_kernel, dim3(scan_grid), dim3(SRC_WG), 0, s, src, (uint64_t)n, S, tab,
                           static_cast<uint32_t *>(perm));
        SENTRY_HIP_CHECK(hipGetLastError());
        // the root hashes do not depend on the sources: the same launches as for one sum
        rc = sentry::lthash_roots(dev_records, dev_offsets, 0, n, static_cast<uint64_t *>(h0), s);
    }
    if (rc) {   // the counts and cursors must not stay behind for the next call
        hipLaunchKernelGGL(src_zero_kernel, dim3(1), dim3(SRC_WG), 0, s, tab, SRC_TABLE_WORDS);
        (void)hipGetLastError();
        return rc;
    }
    hipLaunchKernelGGL(lthash_expand_units_kernel, dim3((uint32_t)ceil_div(max_units, EXP_WAVES)), dim3(EXP_WG), 0, s,
                       static_cast<const uint64_t *>(h0), static_cast<const uint32_t *>(perm), S, unit, tab,
                       static_cast<uint32_t *>(part));
    if (ceil_div(n, unit) / S >= 256)
        hipLaunchKernelGGL((lthash_fold_sources_kernel<4 * FOLD_WG, FOLD_COLS>), dim3(LANE_WORDS / FOLD_COLS, S),
                           dim3(4 * FOLD_WG), 0, s, static_cast<const uint32_t *>(part), S, tab, acc_lanes);
    else
        hipLaunchKernelGGL((lthash_fold_sources_kernel<FOLD_WG, FOLD_COLS>), dim3(LANE_WORDS / FOLD_COLS, S), dim3(FOLD_WG),
                           0, s, static_cast<const uint32_t *>(part), S, tab, acc_lanes);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

int sentry_lthash_combine(uint16_t *acc, const uint16_t *x, void *stream)
{
    return addsub("sentry_lthash_combine", acc, x, stream, false);
}

int sentry_lthash_remove(uint16_t *acc, const uint16_t *x, void *stream)
{
    return addsub("sentry_lthash_remove", acc, x, stream, true);
}

static int check_fixed(const char *fn, const void *dev_records, size_t record_bytes, size_t n, const uint16_t *out_lanes)
{
    SENTRY_REQUIRE(out_lanes != nullptr && (reinterpret_cast<uintptr_t>(out_lanes) & 1) == 0,
                   "%s: out_lanes must be non-NULL and 2-byte aligned", fn);
    SENTRY_REQUIRE(n <= 0xffffffffull / 4 - 64, "%s: too many records", fn);
    SENTRY_REQUIRE(n == 0 || record_bytes <= 0xffffffffffffffffull / n, "%s: n * record_bytes overflows", fn);
    SENTRY_REQUIRE(dev_records != nullptr || n == 0 || record_bytes == 0, "%s: NULL records", fn);
    return SENTRY_OK;
}

int sentry_lthash_fixed(const void *dev_records, size_t record_bytes, size_t n, uint16_t *out_lanes, void *stream)
{
    sentry::clear_error();
    const int rc = check_fixed("sentry_lthash_fixed", dev_records, record_bytes, n, out_lanes);
    if (rc) return rc;
    return sentry::lthash_into(dev_records, nullptr, record_bytes, n, out_lanes, false, static_cast<hipStream_t>(stream));
}

}  // extern "C"

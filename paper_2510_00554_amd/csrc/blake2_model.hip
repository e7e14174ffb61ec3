// Lattice hash of a model (section 4.2.2, Algorithm 4): every block of every tensor gets the
// digest BLAKE2b-512(LE64(block index) || block); the digests, read as 32 partitions of 16
// bits (the 64-byte layout of section 4.2.2), are added per tensor and over the model.
//
// One block per lane, one table-driven launch over all fragmented tensors (the lookup table
// of section 4.2.1).  Addition is order invariant, so there is nothing to schedule by tensor
// size as the paper does with streams: small tensors simply finish early inside the launch.
// A workgroup holds blocks of one tensor, adds its lanes' digests (wave butterfly, then LDS)
// and writes one 64-byte row; a second kernel adds the rows of each tensor, a third the
// tensors.
#include <cstring>
#include <vector>

#include "blake2b_device.h"
#include "sentry_internal.h"

namespace {

constexpr int MODEL_WG = 256;
constexpr int MODEL_WORDS = SENTRY_MODEL_LANES / 2;   // 16 packed 32-bit words = 64 bytes

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

struct MSeg {
    const uint8_t *base;
    uint64_t len;
};
struct MGroup {
    uint64_t first;   // first block of the group inside its tensor
    uint64_t index;   // model-wide index of that block
    uint32_t count;   // blocks in the group (<= MODEL_WG)
    uint32_t seg;
};

// data word w (8 bytes at offset 8w) of an n-byte block at p, zero beyond n
__device__ __forceinline__ uint64_t safe_word(const uint8_t *p, uint64_t n, uint32_t w)
{
    const uint64_t o = 8ull * w;
    if (o + 8 <= n) return *reinterpret_cast<const uint64_t *>(p + o);   // p is 16-byte aligned
    uint64_t v = 0;
    for (uint32_t i = 0; i < 8; i++)
        if (o + i < n) v |= (uint64_t)p[o + i] << (8 * i);
    return v;
}

// BLAKE2b-512(LE64(k) || p[0..n)), default parameter block.  The index shifts the data by
// one 64-bit word against the 128-byte message blocks: compression j takes the last word of
// data chunk j-1 (the index for j = 0) and the first fifteen words of the 16-byte aligned
// data chunk j, so every load is a whole aligned line.
__device__ __forceinline__ void blake2b_index_block(uint64_t k, const uint8_t *p, uint64_t n, uint64_t (&h)[8])
{
#pragma unroll
    for (int i = 0; i < 8; i++) h[i] = b2_iv(i);
    h[0] ^= 0x0000000001010040ull;   // digest 64, no key, fanout 1, depth 1
    const uint64_t M = n + 8;
    const uint64_t ncomp = (M + 127) >> 7;
    // compressions whose whole data chunk, carry word included, lies inside the block
    const uint64_t nfast = ncomp >= 2 ? ncomp - 2 : 0;
    uint64_t carry = k;
    const uint4 *q = reinterpret_cast<const uint4 *>(p);
    uint4 c[8] = {};
    if (nfast) {
#pragma unroll
        for (int i = 0; i < 8; i++) c[i] = q[i];
    }
    for (uint64_t j = 0; j < nfast; j++) {
        uint64_t m[16];
        m[0] = carry;
#pragma unroll
        for (int i = 0; i < 7; i++) {
            m[2 * i + 1] = pack64(c[i].x, c[i].y);
            m[2 * i + 2] = pack64(c[i].z, c[i].w);
        }
        m[15] = pack64(c[7].x, c[7].y);
        carry = pack64(c[7].z, c[7].w);
        q += 8;
        if (j + 1 < nfast) {
#pragma unroll
            for (int i = 0; i < 8; i++) c[i] = q[i];
        }
        blake2b_compress(h, m, 128 * (j + 1), false);
    }
    for (uint64_t j = nfast; j < ncomp; j++) {
        uint64_t m[16];
        m[0] = carry;
#pragma unroll
        for (int i = 0; i < 15; i++) m[i + 1] = safe_word(p, n, (uint32_t)(16 * j) + i);
        carry = safe_word(p, n, (uint32_t)(16 * j) + 15);
        const bool last = j + 1 == ncomp;
        blake2b_compress(h, m, last ? M : 128 * (j + 1), last);
    }
}

// One wave per group of up to 64 blocks of one tensor (a workgroup holds four such waves, each with a
// group of its own, so that a model of many small tensors still keeps all four SIMDs of a compute
// unit busy: with one group of up to 256 blocks per workgroup a tensor of nine blocks left three of
// its four waves empty, and the busy waves of the workgroups of a compute unit met on one SIMD).
__global__ void __launch_bounds__(MODEL_WG)
lthash_model_kernel(const MSeg *segs, const MGroup *groups, uint32_t n_groups, uint64_t block_bytes, uint32_t *rows_out)
{
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t g = blockIdx.x * (MODEL_WG / 64) + (threadIdx.x >> 6);
    if (g >= n_groups) return;                       // wave-uniform; no barrier below
    const MGroup gr = groups[g];
    const MSeg sg = segs[gr.seg];
    uint64_t h[8];
#pragma unroll
    for (int i = 0; i < 8; i++) h[i] = 0;
    if (lane < gr.count) {
        const uint64_t start = (gr.first + lane) * block_bytes;
        const uint64_t left = sg.len - start;
        blake2b_index_block(gr.index + lane, sg.base + start, left < block_bytes ? left : block_bytes, h);
    }
    // add the 64 digests of the wave: 16 packed words, butterfly over the lanes
#pragma unroll
    for (int i = 0; i < 8; i++) {
#pragma unroll
        for (int half = 0; half < 2; half++) {
            const uint32_t x0 = half ? (uint32_t)(h[i] >> 32) : (uint32_t)h[i];
            u16x2 s = u16x2{(unsigned short)x0, (unsigned short)(x0 >> 16)};
#pragma unroll
            for (int sft = 32; sft >= 1; sft >>= 1) {
                const uint32_t x = (uint32_t)s.x | ((uint32_t)s.y << 16);
                const uint32_t y = (uint32_t)__shfl_xor((int)x, sft, 64);
                s += u16x2{(unsigned short)y, (unsigned short)(y >> 16)};
            }
            if (lane == 0) rows_out[(uint64_t)g * MODEL_WORDS + 2 * i + half] = (uint32_t)s.x | ((uint32_t)s.y << 16);
        }
    }
}

// out_row[r] = sum of rows [row_start[r], row_start[r+1]) of `rows`, r = blockIdx.x; 16 columns x 16
// row slices per workgroup.  With row_start == nullptr there is one output: the sum of all n_rows.
__global__ void __launch_bounds__(MODEL_WG)
lthash_model_fold_kernel(const uint32_t *rows, const uint32_t *row_start, uint32_t n_rows, uint32_t *out_rows,
                         uint16_t *out_a, uint16_t *out_b)
{
    const uint32_t r = blockIdx.x, col = threadIdx.x % MODEL_WORDS, slice = threadIdx.x / MODEL_WORDS;
    const uint32_t lo = row_start ? row_start[r] : 0, hi = row_start ? row_start[r + 1] : n_rows;
    u16x2 s = u16x2{0, 0};
    for (uint32_t k = lo + slice; k < hi; k += MODEL_WG / MODEL_WORDS) {
        const uint32_t x = rows[(uint64_t)k * MODEL_WORDS + col];
        s += u16x2{(unsigned short)x, (unsigned short)(x >> 16)};
    }
    __shared__ uint32_t lds[MODEL_WG / MODEL_WORDS][MODEL_WORDS];
    lds[slice][col] = (uint32_t)s.x | ((uint32_t)s.y << 16);
    __syncthreads();
    if (slice == 0) {
        u16x2 t = u16x2{0, 0};
#pragma unroll
        for (int k = 0; k < MODEL_WG / MODEL_WORDS; k++) {
            const uint32_t x = lds[k][col];
            t += u16x2{(unsigned short)x, (unsigned short)(x >> 16)};
        }
        if (out_rows) out_rows[(uint64_t)r * MODEL_WORDS + col] = (uint32_t)t.x | ((uint32_t)t.y << 16);
        if (out_a) { out_a[(uint64_t)r * SENTRY_MODEL_LANES + 2 * col] = t.x; out_a[(uint64_t)r * SENTRY_MODEL_LANES + 2 * col + 1] = t.y; }
        if (out_b) { out_b[(uint64_t)r * SENTRY_MODEL_LANES + 2 * col] = t.x; out_b[(uint64_t)r * SENTRY_MODEL_LANES + 2 * col + 1] = t.y; }
    }
}

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

}  // namespace

extern "C" {

int sentry_lthash_model(const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t block_bytes,
                        uint16_t *out_layer_lanes, uint16_t *out_lanes, void *stream)
{
    return sentry_lthash_model_from(dev_ptrs, lens, n_seg, block_bytes, 0, out_layer_lanes, out_lanes, stream);
}

int sentry_lthash_model_from(const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t block_bytes,
                             uint64_t first_index, uint16_t *out_layer_lanes, uint16_t *out_lanes, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(n_seg >= 1 && n_seg <= 0x7fffffffull, "sentry_lthash_model: n_seg must be at least 1");
    SENTRY_REQUIRE(dev_ptrs && lens && out_lanes, "sentry_lthash_model: NULL argument");
    SENTRY_REQUIRE(block_bytes > 0 && block_bytes % 16 == 0,
                   "sentry_lthash_model: block_bytes must be a positive multiple of 16 (got %zu)", block_bytes);
    SENTRY_REQUIRE(((reinterpret_cast<uintptr_t>(out_lanes) | reinterpret_cast<uintptr_t>(out_layer_lanes)) & 1) == 0,
                   "sentry_lthash_model: lanes must be 2-byte aligned");
    // the lookup table: one row per wave, groups of up to 64 blocks of one tensor
    std::vector<MGroup> groups;
    std::vector<uint32_t> row_start(n_seg + 1);
    uint64_t index = first_index;
    for (size_t t = 0; t < n_seg; t++) {
        SENTRY_REQUIRE(dev_ptrs[t] != nullptr || lens[t] == 0, "sentry_lthash_model: segment %zu is NULL", t);
        SENTRY_REQUIRE((reinterpret_cast<uintptr_t>(dev_ptrs[t]) & 15) == 0,
                       "sentry_lthash_model: segment %zu is not 16-byte aligned", t);
        row_start[t] = (uint32_t)groups.size();
        const uint64_t nb = ceil_div(lens[t], block_bytes);
        for (uint64_t f = 0; f < nb; f += 64)
            groups.push_back(MGroup{f, index + f, (uint32_t)(nb - f < 64 ? nb - f : 64), (uint32_t)t});
        index += nb;
        SENTRY_REQUIRE(groups.size() <= 0xffffffffull / 64, "sentry_lthash_model: too many blocks");
    }
    row_start[n_seg] = (uint32_t)groups.size();
    const size_t n_groups = groups.size();

    const size_t seg_bytes = n_seg * sizeof(MSeg), grp_bytes = n_groups * sizeof(MGroup);
    const size_t table_bytes = seg_bytes + grp_bytes + 4 * (n_seg + 1);
    void *host_tab, *dev_tab, *rows, *layer_rows;
    int rc;
    if ((rc = sentry::table_staging_get(s, table_bytes, &host_tab))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_TABLES, table_bytes, &dev_tab))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_LT_PART, (n_groups ? n_groups : 1) * MODEL_WORDS * 4, &rows))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_LT_SUM, n_seg * MODEL_WORDS * 4, &layer_rows))) return rc;
    MSeg *hseg = static_cast<MSeg *>(host_tab);
    for (size_t t = 0; t < n_seg; t++) hseg[t] = MSeg{static_cast<const uint8_t *>(dev_ptrs[t]), lens[t]};
    char *hp = static_cast<char *>(host_tab);
    if (n_groups) std::memcpy(hp + seg_bytes, groups.data(), grp_bytes);
    std::memcpy(hp + seg_bytes + grp_bytes, row_start.data(), 4 * (n_seg + 1));
    SENTRY_HIP_CHECK(hipMemcpyAsync(dev_tab, host_tab, table_bytes, hipMemcpyHostToDevice, s));
    if ((rc = sentry::table_staging_mark(s))) return rc;
    char *dp = static_cast<char *>(dev_tab);
    if (n_groups) {
        hipLaunchKernelGGL(lthash_model_kernel, dim3((uint32_t)ceil_div(n_groups, MODEL_WG / 64)), dim3(MODEL_WG), 0, s,
                           reinterpret_cast<const MSeg *>(dp), reinterpret_cast<const MGroup *>(dp + seg_bytes),
                           (uint32_t)n_groups, (uint64_t)block_bytes, static_cast<uint32_t *>(rows));
        SENTRY_HIP_CHECK(hipGetLastError());
    }
    // per-tensor digests, then the model digest over them
    hipLaunchKernelGGL(lthash_model_fold_kernel, dim3((uint32_t)n_seg), dim3(MODEL_WG), 0, s,
                       static_cast<const uint32_t *>(rows), reinterpret_cast<const uint32_t *>(dp + seg_bytes + grp_bytes),
                       (uint32_t)n_groups, static_cast<uint32_t *>(layer_rows), out_layer_lanes, (uint16_t *)nullptr);
    hipLaunchKernelGGL(lthash_model_fold_kernel, dim3(1), dim3(MODEL_WG), 0, s,
                       static_cast<const uint32_t *>(layer_rows), (const uint32_t *)nullptr, (uint32_t)n_seg,
                       (uint32_t *)nullptr, out_lanes, (uint16_t *)nullptr);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

}  // extern "C"

// The dataset lattice hash at the digest width of section 4.2.2: one plain BLAKE2b-512 digest per
// sample, cut into 32 partitions of 16 bits, partition-wise sums mod 2^16 (section 2.2 Eq. (1)).
// The per-sample hashes are the root kernels of blake2_lthash.hip run with the plain parameter
// block; this file holds what comes after them: the sum over the 64-byte digests, the per-source
// sums (section 4.3), the lattice addition and subtraction on 32 partitions, and the entry points.
#include "lthash_internal.h"

namespace {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
inline int cu_count() { return sentry::lthash_cu_count(); }

constexpr uint64_t PLAIN_P0 = sentry::LT_PLAIN_P0, PLAIN_P1 = sentry::LT_PLAIN_P1;
constexpr uint32_t SRC_MAX_SOURCES = sentry::LT_MAX_SOURCES;
constexpr int ZERO_WG = 256;

__global__ void __launch_bounds__(ZERO_WG)
zero_words32_kernel(uint32_t *words, uint32_t n_words)
{
    for (uint32_t i = blockIdx.x * ZERO_WG + threadIdx.x; i < n_words; i += gridDim.x * ZERO_WG) words[i] = 0;
}

// acc[l] = acc[l] +/- x[l] mod 2^16 on 32 partitions, two per thread (section 4.2.2: the lattice
// addition; the 16-bit partitions cannot carry into each other)
template <bool SUB>
__global__ void __launch_bounds__(64)
lthash32_addsub_kernel(uint16_t *acc, const uint16_t *x)
{
    const uint32_t c = threadIdx.x;
    if (c >= SENTRY_LANES32 / 2) return;
    u16x2 a = u16x2{acc[2 * c], acc[2 * c + 1]};
    u16x2 b = u16x2{x[2 * c], x[2 * c + 1]};
    u16x2 r = SUB ? (a - b) : (a + b);
    acc[2 * c] = r.x;
    acc[2 * c + 1] = r.y;
}

// ---------------------------------------------------------------------------
// the 32-partition hash: the 64-byte digest itself cut into 32 lanes (section 4.2.2)
// ---------------------------------------------------------------------------
//
// The rows are the plain BLAKE2b-512 digests the root kernels leave: 16 packed words of two
// lanes each.  A workgroup takes a contiguous run of rows; thread t adds word t % 16 of every
// 16th row of the run, starting at row t / 16, so a wave reads four whole rows (256 adjacent
// bytes) at a time; the 16 partial sums of a word meet in LDS.  The first launch leaves one
// packed row per workgroup, the second (one workgroup, over those rows) writes the 32 lanes.
// Rows are row_words 32-bit words apart (16 for digests and partial rows).

constexpr int SUM32_WG = 256;
constexpr int SUM32_WORDS = SENTRY_LANES32 / 2;      // 16 packed words = one 64-byte digest
constexpr int SUM32_SLICES = SUM32_WG / SUM32_WORDS; // 16 rows in flight per trip
constexpr int SUM32_AHEAD = 4;                       // loads issued before the first add

__global__ void __launch_bounds__(SUM32_WG)
lthash32_sum_kernel(const uint32_t *rows, uint64_t n_rows, uint64_t row_words, uint32_t *packed_out, uint16_t *lanes_out,
                    bool add_to_out)
{
    __shared__ uint32_t lds[SUM32_SLICES][SUM32_WORDS];
    const uint32_t col = threadIdx.x % SUM32_WORDS;
    const uint32_t slice = threadIdx.x / SUM32_WORDS;
    const uint64_t per = (n_rows + gridDim.x - 1) / gridDim.x;
    const uint64_t lo = per * blockIdx.x < n_rows ? per * blockIdx.x : n_rows;
    const uint64_t hi = lo + per < n_rows ? lo + per : n_rows;
    u16x2 t = {0, 0};
    uint64_t r = lo + slice;
    for (; r + (uint64_t)(SUM32_AHEAD - 1) * SUM32_SLICES < hi; r += (uint64_t)SUM32_AHEAD * SUM32_SLICES) {
        uint32_t x[SUM32_AHEAD];
#pragma unroll
        for (int a = 0; a < SUM32_AHEAD; a++) x[a] = rows[(r + (uint64_t)a * SUM32_SLICES) * row_words + col];
#pragma unroll
        for (int a = 0; a < SUM32_AHEAD; a++) t += u16x2{(unsigned short)x[a], (unsigned short)(x[a] >> 16)};
    }
    for (; r < hi; r += SUM32_SLICES) {
        const uint32_t x = rows[r * row_words + col];
        t += u16x2{(unsigned short)x, (unsigned short)(x >> 16)};
    }
    lds[slice][col] = (uint32_t)t.x | ((uint32_t)t.y << 16);
    __syncthreads();
    if (threadIdx.x < SUM32_WORDS) {
        u16x2 sum = {0, 0};
#pragma unroll
        for (int k = 0; k < SUM32_SLICES; k++) {
            const uint32_t x = lds[k][threadIdx.x];
            sum += u16x2{(unsigned short)x, (unsigned short)(x >> 16)};
        }
        if (lanes_out) {
            if (add_to_out) sum += u16x2{lanes_out[2 * threadIdx.x], lanes_out[2 * threadIdx.x + 1]};
            lanes_out[2 * threadIdx.x] = sum.x;       // 16-bit stores: 2-byte alignment is enough
            lanes_out[2 * threadIdx.x + 1] = sum.y;
        } else {
            packed_out[(uint64_t)blockIdx.x * SUM32_WORDS + threadIdx.x] = (uint32_t)sum.x | ((uint32_t)sum.y << 16);
        }
    }
}

// Per-source sums of the 64-byte digests (section 4.3 at the width of section 4.2.2).  A sum
// mod 2^16 can be kept in a 32-bit counter whatever it overflows (2^16 divides 2^32), so every
// partition of every source gets a 32-bit counter and the digests are added with atomics:
// first in LDS, one set of counters per workgroup, for up to SRC32_LDS_SOURCES sources (a
// workgroup takes a long run of records, so most additions stay in LDS), then the non-zero
// counters go to the global ones; with more sources than that, where few records meet in a
// counter, straight to the global ones.  A last kernel adds the counters to the running sums.
constexpr int SRC32_WG = 256;
constexpr uint32_t SRC32_LDS_SOURCES = 256;       // 256 x 32 counters of 4 bytes = 32 KiB of LDS

template <bool IN_LDS>
__global__ void __launch_bounds__(SRC32_WG)
lthash32_src_sum_kernel(const uint32_t *rows, const uint32_t *src, uint64_t n, uint32_t n_sources, uint32_t *counters)
{
    extern __shared__ uint32_t lds_counters[];
    const uint32_t col = threadIdx.x % SUM32_WORDS;
    const uint32_t slice = threadIdx.x / SUM32_WORDS;
    const uint32_t words = n_sources * SENTRY_LANES32;
    if (IN_LDS) {
        for (uint32_t i = threadIdx.x; i < words; i += SRC32_WG) lds_counters[i] = 0;
        __syncthreads();
    }
    const uint64_t per = (n + gridDim.x - 1) / gridDim.x;
    const uint64_t lo = per * blockIdx.x < n ? per * blockIdx.x : n;
    const uint64_t hi = lo + per < n ? lo + per : n;
    uint32_t *to = IN_LDS ? lds_counters : counters;
    uint64_t r = lo + slice;
    for (; r + (uint64_t)(SUM32_AHEAD - 1) * SUM32_SLICES < hi; r += (uint64_t)SUM32_AHEAD * SUM32_SLICES) {
        uint32_t k[SUM32_AHEAD], x[SUM32_AHEAD];          // the loads of four records before their additions
#pragma unroll
        for (int a = 0; a < SUM32_AHEAD; a++) {
            k[a] = src[r + (uint64_t)a * SUM32_SLICES];
            x[a] = rows[(r + (uint64_t)a * SUM32_SLICES) * SUM32_WORDS + col];
        }
#pragma unroll
        for (int a = 0; a < SUM32_AHEAD; a++) {
            if (k[a] >= n_sources) continue;              // not a source of this call: left out
            atomicAdd(&to[k[a] * SENTRY_LANES32 + 2 * col], x[a] & 0xffffu);
            atomicAdd(&to[k[a] * SENTRY_LANES32 + 2 * col + 1], x[a] >> 16);
        }
    }
    for (; r < hi; r += SUM32_SLICES) {
        const uint32_t k = src[r];
        if (k >= n_sources) continue;
        const uint32_t x = rows[r * SUM32_WORDS + col];
        atomicAdd(&to[k * SENTRY_LANES32 + 2 * col], x & 0xffffu);
        atomicAdd(&to[k * SENTRY_LANES32 + 2 * col + 1], x >> 16);
    }
    if (IN_LDS) {
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < words; i += SRC32_WG) {
            const uint32_t v = lds_counters[i];
            if (v) atomicAdd(&counters[i], v);
        }
    }
}

// adds the counters to the running sums and leaves them zero for the next call
__global__ void __launch_bounds__(SRC32_WG)
lthash32_src_add_kernel(uint32_t *counters, uint32_t n_words, uint16_t *acc)
{
    const uint32_t i = blockIdx.x * SRC32_WG + threadIdx.x;
    if (i < n_words) {
        acc[i] = (uint16_t)(acc[i] + counters[i]);
        counters[i] = 0;
    }
}

}  // namespace

namespace sentry {

// The 32-partition hash of n records (offsets as for lthash_into): overwrites the 32 lanes at
// out or, with accumulate, is added to them.
int lthash32_into(const void *dev_records, const uint64_t *dev_offsets, uint64_t offset_base, uint64_t n,
                  uint16_t *out, bool accumulate, hipStream_t s)
{
    // one partial row per workgroup; a workgroup's run is at least one full trip of its 16 slices
    uint64_t grid = ceil_div(n, (uint64_t)SUM32_SLICES * SUM32_AHEAD * 4);
    const uint64_t cap = (uint64_t)cu_count() * 4;
    if (grid > cap) grid = cap;
    if (grid == 0) grid = 1;
    void *h0, *part;
    int rc;
    if ((rc = scratch_get(s, R_LT_H0, 64 * (n ? n : 1), &h0))) return rc;
    if ((rc = scratch_get(s, R_LT_PART, grid * SUM32_WORDS * 4, &part))) return rc;
    rc = dev_offsets ? lthash_roots(dev_records, dev_offsets, offset_base, n, static_cast<uint64_t *>(h0), s, PLAIN_P0, PLAIN_P1)
                     : lthash_roots_fixed(dev_records, offset_base, n, static_cast<uint64_t *>(h0), s, PLAIN_P0, PLAIN_P1);
    if (rc) return rc;
    if (grid == 1) {
        hipLaunchKernelGGL(lthash32_sum_kernel, dim3(1), dim3(SUM32_WG), 0, s, static_cast<const uint32_t *>(h0),
                           (uint64_t)n, (uint64_t)SUM32_WORDS, static_cast<uint32_t *>(nullptr), out, accumulate);
    } else {
        hipLaunchKernelGGL(lthash32_sum_kernel, dim3((uint32_t)grid), dim3(SUM32_WG), 0, s,
                           static_cast<const uint32_t *>(h0), (uint64_t)n, (uint64_t)SUM32_WORDS,
                           static_cast<uint32_t *>(part), static_cast<uint16_t *>(nullptr), false);
        hipLaunchKernelGGL(lthash32_sum_kernel, dim3(1), dim3(SUM32_WG), 0, s, static_cast<const uint32_t *>(part),
                           grid, (uint64_t)SUM32_WORDS, static_cast<uint32_t *>(nullptr), out, accumulate);
    }
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

// out (32 lanes) = sum of the first 32 lanes of n_rows rows that lie row_lanes uint16 apart
// (4-byte aligned rows: the slots of a running sum).
int lthash32_sum_rows(const uint16_t *rows, uint32_t n_rows, uint32_t row_lanes, uint16_t *out, hipStream_t s)
{
    hipLaunchKernelGGL(lthash32_sum_kernel, dim3(1), dim3(SUM32_WG), 0, s, reinterpret_cast<const uint32_t *>(rows),
                       (uint64_t)n_rows, (uint64_t)(row_lanes / 2), static_cast<uint32_t *>(nullptr), out, false);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

}  // namespace sentry

static int check_fixed(const char *fn, const void *dev_records, size_t record_bytes, size_t n, const uint16_t *out_lanes)
{
    SENTRY_REQUIRE(out_lanes != nullptr && (reinterpret_cast<uintptr_t>(out_lanes) & 1) == 0,
                   "%s: out_lanes must be non-NULL and 2-byte aligned", fn);
    SENTRY_REQUIRE(n <= sentry::LT_MAX_RECORDS, "%s: too many records", fn);
    SENTRY_REQUIRE(n == 0 || record_bytes <= 0xffffffffffffffffull / n, "%s: n * record_bytes overflows", fn);
    SENTRY_REQUIRE(dev_records != nullptr || n == 0 || record_bytes == 0, "%s: NULL records", fn);
    return SENTRY_OK;
}

static int addsub32(const char *fn, uint16_t *acc, const uint16_t *x, void *stream, bool sub)
{
    sentry::clear_error();
    SENTRY_REQUIRE(acc != nullptr && x != nullptr, "%s: NULL argument", fn);
    SENTRY_REQUIRE(((reinterpret_cast<uintptr_t>(acc) | reinterpret_cast<uintptr_t>(x)) & 1) == 0,
                   "%s: lanes must be 2-byte aligned", fn);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (sub)
        hipLaunchKernelGGL(lthash32_addsub_kernel<true>, dim3(1), dim3(64), 0, s, acc, x);
    else
        hipLaunchKernelGGL(lthash32_addsub_kernel<false>, dim3(1), dim3(64), 0, s, acc, x);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

extern "C" {

int sentry_lthash32(const void *dev_records, const uint64_t *dev_offsets, size_t n, uint16_t *out_lanes, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(out_lanes != nullptr && (reinterpret_cast<uintptr_t>(out_lanes) & 1) == 0,
                   "sentry_lthash32: out_lanes must be non-NULL and 2-byte aligned");
    SENTRY_REQUIRE(n == 0 || (dev_offsets != nullptr && (reinterpret_cast<uintptr_t>(dev_offsets) & 7) == 0),
                   "sentry_lthash32: dev_offsets must be non-NULL and 8-byte aligned when n > 0");
    SENTRY_REQUIRE(n <= sentry::LT_MAX_RECORDS, "sentry_lthash32: too many records");
    return sentry::lthash32_into(dev_records, dev_offsets, 0, n, out_lanes, false, s);
}

int sentry_lthash32_fixed(const void *dev_records, size_t record_bytes, size_t n, uint16_t *out_lanes, void *stream)
{
    sentry::clear_error();
    const int rc = check_fixed("sentry_lthash32_fixed", dev_records, record_bytes, n, out_lanes);
    if (rc) return rc;
    return sentry::lthash32_into(dev_records, nullptr, record_bytes, n, out_lanes, false, static_cast<hipStream_t>(stream));
}

int sentry_lthash32_sources(const void *dev_records, const uint64_t *dev_offsets, const uint32_t *dev_source_ids,
                            size_t n, size_t n_sources, uint16_t *acc_lanes, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(n_sources >= 1 && n_sources <= SRC_MAX_SOURCES, "sentry_lthash32_sources: n_sources must be 1..%u",
                   SRC_MAX_SOURCES);
    SENTRY_REQUIRE(acc_lanes != nullptr && (reinterpret_cast<uintptr_t>(acc_lanes) & 1) == 0,
                   "sentry_lthash32_sources: acc_lanes must be non-NULL and 2-byte aligned");
    if (n == 0) return SENTRY_OK;
    SENTRY_REQUIRE(dev_offsets != nullptr && (reinterpret_cast<uintptr_t>(dev_offsets) & 7) == 0,
                   "sentry_lthash32_sources: dev_offsets must be non-NULL and 8-byte aligned");
    SENTRY_REQUIRE(dev_source_ids != nullptr && (reinterpret_cast<uintptr_t>(dev_source_ids) & 3) == 0,
                   "sentry_lthash32_sources: dev_source_ids must be non-NULL and 4-byte aligned");
    SENTRY_REQUIRE(n <= sentry::LT_MAX_RECORDS, "sentry_lthash32_sources: too many records");
    const uint32_t S = (uint32_t)n_sources;
    const uint32_t words = S * SENTRY_LANES32;
    void *h0, *counters;
    int rc;
    bool fresh;
    if ((rc = sentry::scratch_get(s, sentry::R_LT_H0, 64 * n, &h0))) return rc;
    // the counters of every possible source, so that the region never grows and what the last call
    // left zero stays zero: cleared by a launch only when newly allocated (or after a failure)
    const uint32_t all_words = SRC_MAX_SOURCES * SENTRY_LANES32;
    if ((rc = sentry::scratch_get_fresh(s, sentry::R_SRC32, 4 * (size_t)all_words, &counters, &fresh))) return rc;
    uint32_t *cnt = static_cast<uint32_t *>(counters);
    if (fresh) hipLaunchKernelGGL(zero_words32_kernel, dim3(all_words / (16 * ZERO_WG)), dim3(ZERO_WG), 0, s, cnt, all_words);
    auto launches = [&]() -> int {
        int rc2 = sentry::lthash_roots(dev_records, dev_offsets, 0, n, static_cast<uint64_t *>(h0), s, PLAIN_P0, PLAIN_P1);
        if (rc2) return rc2;
        if (S <= SRC32_LDS_SOURCES) {
            // a workgroup's counters are worth their flush when its run of records is several times as
            // long as the table: 4 records per source, 256 at least; at most four workgroups per CU
            const uint64_t run = 4 * (uint64_t)S > 256 ? 4 * (uint64_t)S : 256;
            uint64_t grid = ceil_div(n, run);
            const uint64_t cap = (uint64_t)cu_count() * 4;
            if (grid > cap) grid = cap;
            hipLaunchKernelGGL(lthash32_src_sum_kernel<true>, dim3((uint32_t)grid), dim3(SRC32_WG), 4 * (size_t)words, s,
                               static_cast<const uint32_t *>(h0), dev_source_ids, (uint64_t)n, S, cnt);
        } else {
            uint64_t grid = ceil_div(n, 256);
            const uint64_t cap = (uint64_t)cu_count() * 8;
            if (grid > cap) grid = cap;
            hipLaunchKernelGGL(lthash32_src_sum_kernel<false>, dim3((uint32_t)grid), dim3(SRC32_WG), 0, s,
                               static_cast<const uint32_t *>(h0), dev_source_ids, (uint64_t)n, S, cnt);
        }
        hipLaunchKernelGGL(lthash32_src_add_kernel, dim3((uint32_t)ceil_div(words, SRC32_WG)), dim3(SRC32_WG), 0, s, cnt, words,
                           acc_lanes);
        SENTRY_HIP_CHECK(hipGetLastError());
        return SENTRY_OK;
    };
    if ((rc = launches())) {
        // whatever was queued may have left counters behind: clear them for the next call
        hipLaunchKernelGGL(zero_words32_kernel, dim3(all_words / (16 * ZERO_WG)), dim3(ZERO_WG), 0, s, cnt, all_words);
        (void)hipGetLastError();
    }
    return rc;
}

int sentry_lthash32_combine(uint16_t *acc, const uint16_t *x, void *stream)
{
    return addsub32("sentry_lthash32_combine", acc, x, stream, false);
}

int sentry_lthash32_remove(uint16_t *acc, const uint16_t *x, void *stream)
{
    return addsub32("sentry_lthash32_remove", acc, x, stream, true);
}

}  // extern "C"

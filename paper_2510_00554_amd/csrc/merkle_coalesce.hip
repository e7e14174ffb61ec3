// Coalesced hashing (Algorithm 1, section 4.2.1 "Coalesced Hashing"): the Merkle root of the
// tensors laid one behind the other in one buffer whose size is a whole number of blocks, the
// bytes behind the last tensor being zero.
//
// Two ways to the same root:
//   * with a buffer from the caller, the scheme as the paper states it: a gather kernel copies
//     every tensor to its place and clears the padding, then the tree runs over the buffer
//     (which the caller keeps: the coalesced model);
//   * without one, only the blocks that are made of bytes of more than one tensor (at most one
//     per tensor boundary, and the padded last block) are put together in the library's scratch
//     memory; every other block is hashed where it lies, through the table-driven leaf stage of
//     the in-place scheme, whose flat tree over a list of whole blocks is the same tree.  That
//     takes neither the second copy of the model nor the time to write and re-read it.
// The gather kernel is a plain copy bound by HBM; the hashing is all in the other files.
#include <algorithm>
#include <vector>

#include "sentry_internal.h"

namespace {

constexpr int GATHER_WG = 256;
constexpr uint64_t GATHER_CHUNK = 65536;   // bytes one workgroup moves

// One run of bytes to put at `dst` (byte offset in the destination): a tensor, or the part of
// one that falls into a block; src == nullptr writes zeros.  A piece is cut into chunks of
// GATHER_CHUNK bytes counted from its start; first_chunk = chunks of all pieces before it.
struct Piece {
    const uint8_t *src;
    uint64_t dst;
    uint64_t bytes;
    uint64_t first_chunk;
};

// n bytes from s to d in units of T where both are aligned for T at the same byte offsets
// (the caller checks that), single bytes before the first and after the last whole unit.
template <typename T, bool ZERO>
__device__ __forceinline__ void move_span(const uint8_t *s, uint8_t *d, uint64_t n)
{
    const uint32_t t = threadIdx.x;
    uint64_t head = (sizeof(T) - (reinterpret_cast<uintptr_t>(d) & (sizeof(T) - 1))) & (sizeof(T) - 1);
    if (head > n) head = n;
    if (t < head) d[t] = ZERO ? (uint8_t)0 : s[t];
    const uint64_t units = (n - head) / sizeof(T);
    const T *sv = reinterpret_cast<const T *>(s + head);
    T *dv = reinterpret_cast<T *>(d + head);
    uint64_t i = t;
    for (; i + 3 * GATHER_WG < units; i += 4 * GATHER_WG) {     // four loads in flight per lane
        T x[4];
#pragma unroll
        for (int k = 0; k < 4; k++) x[k] = ZERO ? T{} : sv[i + k * GATHER_WG];
#pragma unroll
        for (int k = 0; k < 4; k++) dv[i + k * GATHER_WG] = x[k];
    }
    for (; i < units; i += GATHER_WG) dv[i] = ZERO ? T{} : sv[i];
    const uint64_t done = head + units * sizeof(T);
    if (t < n - done) d[done + t] = ZERO ? (uint8_t)0 : s[done + t];
}

__global__ void __launch_bounds__(GATHER_WG)
gather_kernel(const Piece *pieces, uint32_t n_pieces, uint8_t *dst_base)
{
    const uint64_t chunk = blockIdx.x;
    uint32_t lo = 0, hi = n_pieces;            // the last piece whose first_chunk is <= chunk
    while (hi - lo > 1) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if (pieces[mid].first_chunk <= chunk) lo = mid; else hi = mid;
    }
    const Piece pc = pieces[lo];
    const uint64_t start = (chunk - pc.first_chunk) * GATHER_CHUNK;
    if (start >= pc.bytes) return;             // cannot happen with a well-formed table
    const uint64_t n = pc.bytes - start < GATHER_CHUNK ? pc.bytes - start : GATHER_CHUNK;
    uint8_t *d = dst_base + pc.dst + start;
    if (pc.src == nullptr) {
        move_span<uint4, true>(nullptr, d, n);
        return;
    }
    const uint8_t *s = pc.src + start;
    const uintptr_t apart = reinterpret_cast<uintptr_t>(s) ^ reinterpret_cast<uintptr_t>(d);
    if ((apart & 15) == 0) move_span<uint4, false>(s, d, n);
    else if ((apart & 3) == 0) move_span<uint32_t, false>(s, d, n);
    else move_span<uint8_t, false>(s, d, n);
}

struct Plan {
    std::vector<Piece> pieces;
    // the leaf stage's list of runs of whole blocks, in order: in a tensor (addr = its address)
    // or in the gathered memory (addr = byte offset in it)
    struct Run { bool gathered; uintptr_t addr; uint64_t bytes; };
    std::vector<Run> runs;
    uint64_t gathered_bytes = 0;
    uint64_t chunks = 0;

    void piece(const uint8_t *src, uint64_t dst, uint64_t bytes)
    {
        if (bytes == 0) return;
        if (src && !pieces.empty()) {
            Piece &last = pieces.back();
            if (last.src && last.src + last.bytes == src && last.dst + last.bytes == dst) { last.bytes += bytes; return; }
        }
        pieces.push_back(Piece{src, dst, bytes, 0});
    }
    void run(bool gathered, uintptr_t addr, uint64_t bytes)
    {
        if (!runs.empty()) {
            Run &last = runs.back();
            if (last.gathered == gathered && last.addr + last.bytes == addr) { last.bytes += bytes; return; }
        }
        runs.push_back(Run{gathered, addr, bytes});
    }
    void number_chunks()
    {
        chunks = 0;
        for (Piece &p : pieces) {
            p.first_chunk = chunks;
            chunks += (p.bytes + GATHER_CHUNK - 1) / GATHER_CHUNK;
        }
    }
};

// Everything into one buffer: a piece per tensor, zeros up to the padded size.
Plan plan_copy_all(const void *const *ptrs, const size_t *lens, size_t n_seg, uint64_t padded)
{
    Plan pl;
    uint64_t pos = 0;
    for (size_t t = 0; t < n_seg; t++) {
        pl.piece(static_cast<const uint8_t *>(ptrs[t]), pos, lens[t]);
        pos += lens[t];
    }
    pl.pieces.push_back(Piece{nullptr, pos, padded - pos, 0});
    if (padded == pos) pl.pieces.pop_back();
    pl.number_chunks();
    return pl;
}

// Only what cannot be hashed where it lies: a block is gathered when it holds bytes of more than
// one tensor, when it is the padded last one, or when its bytes in the tensor are not 16-byte
// aligned (the leaf stage reads 16-byte words).
Plan plan_in_place(const void *const *ptrs, const size_t *lens, size_t n_seg, uint64_t leaf)
{
    Plan pl;
    uint64_t pos = 0;          // bytes of the concatenation placed so far
    uint64_t open_at = 0;      // where the block that is being filled lies in the gathered memory
    for (size_t t = 0; t < n_seg; t++) {
        const uint8_t *p = static_cast<const uint8_t *>(ptrs[t]);
        uint64_t left = lens[t];
        while (left) {
            const uint64_t in_block = pos % leaf;
            if (in_block == 0 && left >= leaf) {            // whole blocks of this tensor, in one step
                const uint64_t whole = left / leaf * leaf;
                if ((reinterpret_cast<uintptr_t>(p) & 15) == 0) {
                    pl.run(false, reinterpret_cast<uintptr_t>(p), whole);
                } else {
                    pl.run(true, (uintptr_t)pl.gathered_bytes, whole);
                    pl.piece(p, pl.gathered_bytes, whole);
                    pl.gathered_bytes += whole;
                }
                p += whole; left -= whole; pos += whole;
                continue;
            }
            if (in_block == 0) {
                open_at = pl.gathered_bytes;
                pl.run(true, (uintptr_t)open_at, leaf);
                pl.gathered_bytes += leaf;
            }
            const uint64_t take = std::min(leaf - in_block, left);
            pl.piece(p, open_at + in_block, take);
            p += take; left -= take; pos += take;
        }
    }
    if (pos % leaf) pl.pieces.push_back(Piece{nullptr, open_at + pos % leaf, leaf - pos % leaf, 0});
    pl.number_chunks();
    return pl;
}

int launch_gather(const Plan &pl, uint8_t *dst, hipStream_t s)
{
    if (pl.pieces.empty()) return SENTRY_OK;
    SENTRY_REQUIRE(pl.chunks <= 0x7fffffffull && pl.pieces.size() <= 0xffffffffull,
                   "sentry_merkle_coalesced_h: too many bytes to copy in one launch");
    const size_t table_bytes = pl.pieces.size() * sizeof(Piece);
    void *host_tab, *dev_tab;
    int rc;
    if ((rc = sentry::table_staging_get(s, table_bytes, &host_tab, 1))) return rc;
    if ((rc = sentry::scratch_get(s, sentry::R_GATHER_TAB, table_bytes, &dev_tab))) return rc;
    std::copy(pl.pieces.begin(), pl.pieces.end(), static_cast<Piece *>(host_tab));
    SENTRY_HIP_CHECK(hipMemcpyAsync(dev_tab, host_tab, table_bytes, hipMemcpyHostToDevice, s));
    if ((rc = sentry::table_staging_mark(s, 1))) return rc;
    hipLaunchKernelGGL(gather_kernel, dim3((uint32_t)pl.chunks), dim3(GATHER_WG), 0, s, static_cast<const Piece *>(dev_tab),
                       (uint32_t)pl.pieces.size(), dst);
    SENTRY_HIP_CHECK(hipGetLastError());
    return SENTRY_OK;
}

}  // namespace

extern "C" {

int sentry_merkle_coalesced_h(int hash, const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes,
                              void *dev_buffer, size_t buffer_bytes, uint8_t *out_root, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(hash == SENTRY_HASH_SHA256 || hash == SENTRY_HASH_BLAKE2B || hash == SENTRY_HASH_SHA3_256,
                   "sentry_merkle_coalesced_h: unknown hash %d", hash);
    SENTRY_REQUIRE(n_seg >= 1, "sentry_merkle_coalesced_h: n_seg must be at least 1");
    SENTRY_REQUIRE(dev_ptrs && lens && out_root, "sentry_merkle_coalesced_h: NULL argument");
    SENTRY_REQUIRE(leaf_bytes > 0 && leaf_bytes % 64 == 0,
                   "sentry_merkle_coalesced_h: leaf_bytes must be a positive multiple of 64 (got %zu)", leaf_bytes);
    uint64_t total = 0;
    for (size_t t = 0; t < n_seg; t++) {
        SENTRY_REQUIRE(dev_ptrs[t] != nullptr || lens[t] == 0, "sentry_merkle_coalesced_h: segment %zu is NULL", t);
        SENTRY_REQUIRE(total + lens[t] >= total, "sentry_merkle_coalesced_h: the lengths overflow");
        total += lens[t];
    }
    const uint64_t padded = (total + leaf_bytes - 1) / leaf_bytes * leaf_bytes;
    SENTRY_REQUIRE(padded >= total, "sentry_merkle_coalesced_h: the lengths overflow");

    if (dev_buffer != nullptr) {
        SENTRY_REQUIRE((reinterpret_cast<uintptr_t>(dev_buffer) & 15) == 0,
                       "sentry_merkle_coalesced_h: dev_buffer %p is not 16-byte aligned", dev_buffer);
        SENTRY_REQUIRE(buffer_bytes >= padded, "sentry_merkle_coalesced_h: dev_buffer holds %zu bytes, %llu are needed",
                       buffer_bytes, (unsigned long long)padded);
        const uintptr_t b0 = reinterpret_cast<uintptr_t>(dev_buffer), b1 = b0 + padded;
        for (size_t t = 0; t < n_seg; t++) {
            const uintptr_t t0 = reinterpret_cast<uintptr_t>(dev_ptrs[t]), t1 = t0 + lens[t];
            SENTRY_REQUIRE(lens[t] == 0 || t1 <= b0 || b1 <= t0, "sentry_merkle_coalesced_h: segment %zu overlaps dev_buffer", t);
        }
        const Plan pl = plan_copy_all(dev_ptrs, lens, n_seg, padded);
        int rc = launch_gather(pl, static_cast<uint8_t *>(dev_buffer), s);
        if (rc) return rc;
        return sentry_merkle_root_h(hash, dev_buffer, padded, leaf_bytes, out_root, stream);
    }

    if (total == 0) return sentry_merkle_root_h(hash, nullptr, 0, leaf_bytes, out_root, stream);   // the empty leaf
    const Plan pl = plan_in_place(dev_ptrs, lens, n_seg, leaf_bytes);
    void *gathered = nullptr;
    int rc;
    if ((rc = sentry::scratch_get(s, sentry::R_GATHER, pl.gathered_bytes, &gathered))) return rc;
    if ((rc = launch_gather(pl, static_cast<uint8_t *>(gathered), s))) return rc;
    std::vector<const void *> run_ptrs(pl.runs.size());
    std::vector<size_t> run_lens(pl.runs.size());
    uint64_t covered = 0;
    for (size_t r = 0; r < pl.runs.size(); r++) {
        const Plan::Run &run = pl.runs[r];
        run_ptrs[r] = run.gathered ? static_cast<const void *>(static_cast<const uint8_t *>(gathered) + run.addr)
                                   : reinterpret_cast<const void *>(run.addr);
        run_lens[r] = run.bytes;
        covered += run.bytes;
    }
    if (covered != padded) {   // the plan is wrong: say so rather than hash something else
        sentry::set_error("sentry_merkle_coalesced_h: internal error, the block list covers %llu of %llu bytes",
                          (unsigned long long)covered, (unsigned long long)padded);
        return SENTRY_ERR_INVALID_ARG;
    }
    return sentry_merkle_inplace_h(hash, run_ptrs.data(), run_lens.data(), run_ptrs.size(), leaf_bytes, out_root, stream);
}

int sentry_merkle_coalesced_plan(const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes,
                                 size_t *out_gathered_bytes, size_t *out_copied_bytes, size_t *out_runs)
{
    sentry::clear_error();
    SENTRY_REQUIRE(n_seg >= 1, "sentry_merkle_coalesced_plan: n_seg must be at least 1");
    SENTRY_REQUIRE(dev_ptrs && lens, "sentry_merkle_coalesced_plan: NULL argument");
    SENTRY_REQUIRE(leaf_bytes > 0 && leaf_bytes % 64 == 0,
                   "sentry_merkle_coalesced_plan: leaf_bytes must be a positive multiple of 64 (got %zu)", leaf_bytes);
    uint64_t total = 0;
    for (size_t t = 0; t < n_seg; t++) {
        SENTRY_REQUIRE(dev_ptrs[t] != nullptr || lens[t] == 0, "sentry_merkle_coalesced_plan: segment %zu is NULL", t);
        SENTRY_REQUIRE(total + lens[t] >= total, "sentry_merkle_coalesced_plan: the lengths overflow");
        total += lens[t];
    }
    const Plan pl = plan_in_place(dev_ptrs, lens, n_seg, leaf_bytes);
    uint64_t copied = 0;
    for (const Piece &p : pl.pieces)
        if (p.src) copied += p.bytes;
    if (out_gathered_bytes) *out_gathered_bytes = pl.gathered_bytes;
    if (out_copied_bytes) *out_copied_bytes = copied;
    if (out_runs) *out_runs = pl.runs.size();
    return SENTRY_OK;
}

int sentry_merkle_coalesced(const void *const *dev_ptrs, const size_t *lens, size_t n_seg, size_t leaf_bytes,
                            void *dev_buffer, size_t buffer_bytes, uint8_t *out_root, void *stream)
{
    return sentry_merkle_coalesced_h(SENTRY_HASH_SHA256, dev_ptrs, lens, n_seg, leaf_bytes, dev_buffer, buffer_bytes,
                                     out_root, stream);
}

}  // extern "C"

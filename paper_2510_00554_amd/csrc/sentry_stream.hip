// Chunked and host-streaming entry points: a Merkle tree over a byte stream that arrives in
// device chunks, and hashing while loading from pinned host memory (section 4.4: artifacts
// are authenticated on the fly as they are loaded; a load on a side HIP stream takes the
// place of the paper's GPUDirect loads).
//
// Pipeline of the *_h2d calls: chunk k is loaded on the side stream into staging buffer
// k%2 while the kernels of chunk k-1 read buffer (k-1)%2 on the caller's stream.  Events
// order "load done -> hash" and "hash done -> buffer may be overwritten"; the host only
// enqueues and never waits.
//
// The load itself: pinned host memory is mapped into the GPU's address space, so a small
// kernel (48 workgroups) that reads it with 16-byte loads and writes the staging buffer moves
// data at the full PCIe rate (57 GB/s here, the same as hipMemcpyAsync) without going through
// the runtime's copy engines, whose choice of engine for back-to-back chunk copies that wait
// on events now and then halved the copy rate for whole runs.  Pageable host memory cannot be
// read by a kernel and still goes through hipMemcpyAsync.
#include <new>
#include <vector>

#include "sentry_internal.h"

namespace sentry {
int merkle_leaves_into(const void *dev_buf, size_t len, size_t leaf_bytes, uint8_t *dst, hipStream_t s);
int merkle_reduce_into(const uint8_t *dev_nodes, uint64_t n, uint8_t *out_digest, hipStream_t s);
int lthash_into(const void *dev_records, const uint64_t *dev_offsets, uint64_t offset_base, uint64_t n,
                uint16_t *out, bool accumulate, hipStream_t s);
int lthash_presize(uint64_t max_records, hipStream_t s);
int lthash_sum_rows(const uint16_t *rows, uint32_t n_rows, uint16_t *out, hipStream_t s);
int lthash32_into(const void *dev_records, const uint64_t *dev_offsets, uint64_t offset_base, uint64_t n,
                  uint16_t *out, bool accumulate, hipStream_t s);
int lthash32_sum_rows(const uint16_t *rows, uint32_t n_rows, uint32_t row_lanes, uint16_t *out, hipStream_t s);
}  // namespace sentry

namespace {

constexpr int LOAD_WG = 256;
// 48 workgroups with one 16-byte load per lane in flight (192 KiB in all) fill the PCIe link.
// More loads in flight per wave buy no bandwidth and slow the hash kernels that run beside the
// load down (measured: four per lane made the chunk hashes take 5.4 ms instead of 2.0).
constexpr int LOAD_GRID = 48;

// dst[0..n) = src[0..n) for src in pinned host (or device) memory; src and dst have the same
// alignment modulo 16, so that the body moves whole aligned 16-byte words
__global__ void __launch_bounds__(LOAD_WG)
host_load_kernel(const uint8_t *src, uint8_t *dst, uint64_t n)
{
    const uint64_t gtid = (uint64_t)blockIdx.x * LOAD_WG + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * LOAD_WG;
    uint64_t head = (16 - (reinterpret_cast<uintptr_t>(src) & 15)) & 15;   // bytes before the first aligned word
    if (head > n) head = n;
    const uint64_t body = (n - head) >> 4;                                   // whole 16-byte words
    const uint64_t tail_at = head + (body << 4);
    if (gtid < head) dst[gtid] = src[gtid];
    if (gtid < n - tail_at) dst[tail_at + gtid] = src[tail_at + gtid];
    const uint4 *s = reinterpret_cast<const uint4 *>(src + head);
    uint4 *d = reinterpret_cast<uint4 *>(dst + head);
#pragma unroll 1
    for (uint64_t i = gtid; i < body; i += stride) d[i] = s[i];
}

// Address at which a kernel can read [p, p + len) of caller memory, or NULL if it cannot
// (pageable host memory).  Pinned host memory and device memory qualify.
const uint8_t *kernel_readable(const void *p, size_t len)
{
    if (!p || !len) return nullptr;
    hipPointerAttribute_t first, last;
    if (hipPointerGetAttributes(&first, p) != hipSuccess ||
        hipPointerGetAttributes(&last, static_cast<const uint8_t *>(p) + (len - 1)) != hipSuccess) {
        (void)hipGetLastError();   // not known to the runtime: ordinary pageable memory
        return nullptr;
    }
    if (first.type == hipMemoryTypeDevice && last.type == hipMemoryTypeDevice) return static_cast<const uint8_t *>(p);
    if (first.type != hipMemoryTypeHost || last.type != hipMemoryTypeHost || !first.devicePointer || !last.devicePointer)
        return nullptr;
    // one mapping: the device view of the last byte lies len - 1 after that of the first
    const uint8_t *d0 = static_cast<const uint8_t *>(first.devicePointer);
    if (static_cast<const uint8_t *>(last.devicePointer) != d0 + (len - 1)) return nullptr;
    return d0;
}

// Enqueue the load of n bytes from host memory to dst on `s`: the load kernel if `readable`
// (the kernel-visible address of src) is set, else hipMemcpyAsync.
int enqueue_load(uint8_t *dst, const uint8_t *src, const uint8_t *readable, size_t n, hipStream_t s)
{
    if (!n) return SENTRY_OK;
    if (readable) {
        hipLaunchKernelGGL(host_load_kernel, dim3(LOAD_GRID), dim3(LOAD_WG), 0, s, readable, dst, (uint64_t)n);
        SENTRY_HIP_CHECK(hipGetLastError());
    } else {
        SENTRY_HIP_CHECK(hipMemcpyAsync(dst, src, n, hipMemcpyHostToDevice, s));
    }
    return SENTRY_OK;
}

struct MerkleStream {
    uint64_t magic;
    size_t total_len, leaf_bytes, fed;
    uint64_t n_leaves;
    uint8_t *leaf_digests;   // device, 32 bytes per leaf of the whole stream
};
constexpr uint64_t STREAM_MAGIC = 0x53454e5452594d53ull;

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------------------
// Lattice hash of batches that arrive from host memory: the pipeline behind sentry_lthash_h2d and
// sentry_lthash_stream_*.  Up to three batches are in flight: each has a staging buffer (held in
// the caller stream's scratch) and a stream of its own (the caller's stream for slot 0, a side
// stream for the others), so the hash of batch k (bound by its longest record, most of the chip
// idle) overlaps the loads and hashes of batches k+1 and k+2.  Slot i keeps a running sum of its
// batches; the caller's stream adds the sums at the end.
// ---------------------------------------------------------------------------
constexpr int LT_SLOTS = sentry::PIPE_SLOTS;
static_assert(LT_SLOTS == 3, "three staging regions exist");
const sentry::Region LT_STAGE_R[3] = {sentry::R_STAGE0, sentry::R_STAGE1, sentry::R_STAGE2};
const sentry::Region LT_OFF_R[3] = {sentry::R_STAGE_OFF0, sentry::R_STAGE_OFF1, sentry::R_STAGE_OFF2};

struct LtStream {
    uint64_t magic;
    uint64_t batches;              // batches fed so far: batch k goes to slot k % 3
    uint16_t *sums;                // device, one row of 1024 lanes per slot
    bool owns_sums;                // allocated by begin (else scratch of the one-call entry point)
    hipStream_t stream;            // the caller's stream, fixed by the first update
    sentry::CopyPipe *pipe;
    bool narrow;                   // the 32-partition hash: only the first 32 lanes of each row are used
};
constexpr uint64_t LT_STREAM_MAGIC = 0x53454e5452594c54ull;

// Feed one batch: n records, record i = host_records[host_offsets[i] .. host_offsets[i+1]).
int lt_stream_feed(LtStream *st, const uint8_t *host_records, const uint64_t *host_offsets, size_t n, hipStream_t s)
{
    if (n == 0) return SENTRY_OK;
    int rc;
    if (st->batches == 0) {
        st->stream = s;
        if ((rc = sentry::copy_pipe_get(s, true, &st->pipe))) return rc;
    }
    SENTRY_REQUIRE(st->stream == s, "lattice stream: all batches of one running sum are fed on one stream");
    sentry::CopyPipe *pipe = st->pipe;
    const int b = (int)(st->batches % LT_SLOTS);
    hipStream_t hs = b == 0 ? s : pipe->hash_stream[b - 1];
    const uint64_t beg = host_offsets[0], end = host_offsets[n];
    // A batch whose records all have one size needs no offsets on the device, and the host, which
    // sees that here, picks the kernel itself (the scan ends at the first record of another size).
    const uint64_t rec = host_offsets[1] - beg;
    bool one_size = host_offsets[1] >= beg;
    for (size_t i = 1; i < n && one_size; i++) one_size = host_offsets[i + 1] - host_offsets[i] == rec;
    // spare bytes: a batch sits at the same offset modulo 16 as in host memory, and the hash kernel
    // reads the whole aligned word that holds a record's last byte
    const size_t need = (end - beg) + 32, need_off = 8 * (n + 1) + 16;
    if (sentry::scratch_capacity(s, LT_STAGE_R[b]) < need || (!one_size && sentry::scratch_capacity(s, LT_OFF_R[b]) < need_off))
        sentry::copy_pipe_drain(pipe, true);   // a buffer is replaced: nothing on the side streams may still use it
    void *stage, *stage_off = nullptr;
    if ((rc = sentry::scratch_get(s, LT_STAGE_R[b], need, &stage))) return rc;
    if (!one_size && (rc = sentry::scratch_get(s, LT_OFF_R[b], need_off, &stage_off))) return rc;
    if ((rc = sentry::lthash_presize(n, hs))) return rc;
    if (st->batches == 0) {
        // nothing of this running sum may start before earlier work on the caller's stream is done
        // with the staging buffers (a previous call ends on that stream)
        SENTRY_HIP_CHECK(hipEventRecord(pipe->start, s));
        SENTRY_HIP_CHECK(hipStreamWaitEvent(pipe->copy_stream, pipe->start, 0));
        for (int i = 0; i < LT_SLOTS - 1; i++) SENTRY_HIP_CHECK(hipStreamWaitEvent(pipe->hash_stream[i], pipe->start, 0));
    }
    // the staging buffer is free once the last hash that read it is done (whichever running sum it
    // belonged to; an event that was never recorded does not hold anything up)
    SENTRY_HIP_CHECK(hipStreamWaitEvent(pipe->copy_stream, pipe->consumed[b], 0));
    const uint8_t *readable = end > beg ? kernel_readable(host_records + beg, end - beg) : nullptr;
    // the batch keeps its alignment modulo 16, so that the load moves whole aligned words
    const uint8_t *from = readable ? readable : host_records + beg;
    uint8_t *to = static_cast<uint8_t *>(stage) + (reinterpret_cast<uintptr_t>(from) & 15);
    if ((rc = enqueue_load(to, host_records + beg, readable, end - beg, pipe->copy_stream))) return rc;
    const uint64_t *dev_offsets = nullptr;
    if (!one_size) {
        // the offsets of the batch, staged at the same offset modulo 16 as in host memory (0 or 8)
        const uint8_t *off_readable = kernel_readable(host_offsets, 8 * (n + 1));
        const uint8_t *off_from = off_readable ? off_readable : reinterpret_cast<const uint8_t *>(host_offsets);
        uint8_t *off_to = static_cast<uint8_t *>(stage_off) + (reinterpret_cast<uintptr_t>(off_from) & 15);
        if ((rc = enqueue_load(off_to, reinterpret_cast<const uint8_t *>(host_offsets), off_readable, 8 * (n + 1), pipe->copy_stream)))
            return rc;
        dev_offsets = reinterpret_cast<const uint64_t *>(off_to);
    }
    SENTRY_HIP_CHECK(hipEventRecord(pipe->copied[b], pipe->copy_stream));
    SENTRY_HIP_CHECK(hipStreamWaitEvent(hs, pipe->copied[b], 0));
    // the caller's stream passes this call once the batch has left host memory
    if (hs != s) SENTRY_HIP_CHECK(hipStreamWaitEvent(s, pipe->copied[b], 0));
    // record i of the batch sits at to + (offset[i] - beg); the kernel copes with any byte alignment
    // (without offsets the third argument is the size of a record)
    rc = (st->narrow ? sentry::lthash32_into : sentry::lthash_into)(
        to, dev_offsets, one_size ? rec : beg, n, st->sums + (size_t)b * SENTRY_LANES,
        st->batches >= (uint64_t)LT_SLOTS, hs);
    if (rc) return rc;
    SENTRY_HIP_CHECK(hipEventRecord(pipe->consumed[b], hs));
    st->batches++;
    return SENTRY_OK;
}

// Join the side streams and write the sum over everything fed to out_lanes.
int lt_stream_finish(LtStream *st, uint16_t *out_lanes, hipStream_t s)
{
    const int used = st->batches < (uint64_t)LT_SLOTS ? (int)st->batches : LT_SLOTS;
    for (int i = 1; i < used; i++) SENTRY_HIP_CHECK(hipStreamWaitEvent(s, st->pipe->consumed[i], 0));
    if (st->narrow) return sentry::lthash32_sum_rows(st->sums, (uint32_t)used, SENTRY_LANES, out_lanes, s);
    return sentry::lthash_sum_rows(st->sums, (uint32_t)used, out_lanes, s);
}

}  // namespace

extern "C" {

int sentry_merkle_stream_begin(size_t total_len, size_t leaf_bytes, void **state)
{
    sentry::clear_error();
    SENTRY_REQUIRE(state != nullptr, "sentry_merkle_stream_begin: NULL state");
    SENTRY_REQUIRE(leaf_bytes > 0 && leaf_bytes % 64 == 0,
                   "sentry_merkle_stream_begin: leaf_bytes must be a positive multiple of 64 (got %zu)", leaf_bytes);
    MerkleStream *st = new (std::nothrow) MerkleStream();
    if (!st) { sentry::set_error("sentry_merkle_stream_begin: out of host memory"); return SENTRY_ERR_NOMEM; }
    st->magic = STREAM_MAGIC;
    st->total_len = total_len;
    st->leaf_bytes = leaf_bytes;
    st->fed = 0;
    st->n_leaves = ceil_div(total_len, leaf_bytes);
    if (st->n_leaves == 0) st->n_leaves = 1;
    (void)sentry::sweep_retired();
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, 32 * st->n_leaves);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        sentry::set_error("sentry_merkle_stream_begin: %zu bytes of leaf digests: %s", (size_t)(32 * st->n_leaves),
                          hipGetErrorString(e));
        delete st;
        return SENTRY_ERR_NOMEM;
    }
    st->leaf_digests = static_cast<uint8_t *>(p);
    *state = st;
    return SENTRY_OK;
}

int sentry_merkle_stream_update(void *state, const void *dev_chunk, size_t len, void *stream)
{
    sentry::clear_error();
    MerkleStream *st = static_cast<MerkleStream *>(state);
    SENTRY_REQUIRE(st && st->magic == STREAM_MAGIC, "sentry_merkle_stream_update: bad state");
    if (len == 0) return SENTRY_OK;
    SENTRY_REQUIRE(dev_chunk != nullptr && (reinterpret_cast<uintptr_t>(dev_chunk) & 15) == 0,
                   "sentry_merkle_stream_update: chunk must be non-NULL and 16-byte aligned");
    SENTRY_REQUIRE(st->fed % st->leaf_bytes == 0,
                   "sentry_merkle_stream_update: a chunk that is not a multiple of leaf_bytes must be the last");
    SENTRY_REQUIRE(len <= st->total_len - st->fed, "sentry_merkle_stream_update: more than total_len bytes fed");
    SENTRY_REQUIRE(len % st->leaf_bytes == 0 || st->fed + len == st->total_len,
                   "sentry_merkle_stream_update: only the last chunk may end inside a leaf");
    uint8_t *dst = st->leaf_digests + 32 * (st->fed / st->leaf_bytes);
    int rc = sentry::merkle_leaves_into(dev_chunk, len, st->leaf_bytes, dst, static_cast<hipStream_t>(stream));
    if (rc) return rc;
    st->fed += len;
    return SENTRY_OK;
}

int sentry_merkle_stream_update_h2d(void *state, const void *host_chunk, size_t len, void *stream)
{
    sentry::clear_error();
    MerkleStream *st = static_cast<MerkleStream *>(state);
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(st && st->magic == STREAM_MAGIC, "sentry_merkle_stream_update_h2d: bad state");
    if (len == 0) return SENTRY_OK;
    SENTRY_REQUIRE(host_chunk != nullptr && (reinterpret_cast<uintptr_t>(host_chunk) & 15) == 0,
                   "sentry_merkle_stream_update_h2d: chunk must be non-NULL and 16-byte aligned");
    SENTRY_REQUIRE(st->fed % st->leaf_bytes == 0,
                   "sentry_merkle_stream_update_h2d: a chunk that is not a multiple of leaf_bytes must be the last");
    SENTRY_REQUIRE(len <= st->total_len - st->fed, "sentry_merkle_stream_update_h2d: more than total_len bytes fed");
    SENTRY_REQUIRE(len % st->leaf_bytes == 0 || st->fed + len == st->total_len,
                   "sentry_merkle_stream_update_h2d: only the last chunk may end inside a leaf");
    sentry::CopyPipe *pipe;
    int rc = sentry::copy_pipe_get(s, false, &pipe);
    if (rc) return rc;
    // two staging buffers per caller stream, used in turn; growing one waits for the stream, whose
    // hash kernels wait for the loads, so nothing is in flight on a buffer that is replaced
    const int b = (int)(pipe->chunk_seq & 1);
    void *stage;
    if ((rc = sentry::scratch_get(s, b ? sentry::R_STAGE1 : sentry::R_STAGE0, len, &stage))) return rc;
    if (st->fed == 0) {
        // first chunk of this tree: the loads start after everything queued on the stream so far,
        // whatever used the staging buffers before
        SENTRY_HIP_CHECK(hipEventRecord(pipe->start, s));
        SENTRY_HIP_CHECK(hipStreamWaitEvent(pipe->copy_stream, pipe->start, 0));
    }
    // the buffer is free once the hash of the chunk that used it last has read it
    SENTRY_HIP_CHECK(hipStreamWaitEvent(pipe->copy_stream, pipe->consumed[b], 0));
    const uint8_t *readable = kernel_readable(host_chunk, len);
    rc = enqueue_load(static_cast<uint8_t *>(stage), static_cast<const uint8_t *>(host_chunk), readable, len, pipe->copy_stream);
    if (rc) return rc;
    pipe->chunk_seq++;
    hipError_t e = hipEventRecord(pipe->copied[b], pipe->copy_stream);
    if (e == hipSuccess) e = hipStreamWaitEvent(s, pipe->copied[b], 0);
    if (e != hipSuccess) {   // the load is queued but the stream does not wait for it: drain it here
        sentry::copy_pipe_drain(pipe, false);
        SENTRY_HIP_CHECK(e);
    }
    uint8_t *dst = st->leaf_digests + 32 * (st->fed / st->leaf_bytes);
    if ((rc = sentry::merkle_leaves_into(stage, len, st->leaf_bytes, dst, s))) return rc;
    SENTRY_HIP_CHECK(hipEventRecord(pipe->consumed[b], s));
    st->fed += len;
    return SENTRY_OK;
}

int sentry_merkle_stream_final(void *state, uint8_t *out_digest, void *stream)
{
    sentry::clear_error();
    MerkleStream *st = static_cast<MerkleStream *>(state);
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(st && st->magic == STREAM_MAGIC, "sentry_merkle_stream_final: bad state");
    SENTRY_REQUIRE(out_digest != nullptr, "sentry_merkle_stream_final: NULL out_digest");
    SENTRY_REQUIRE(st->fed == st->total_len, "sentry_merkle_stream_final: %zu of %zu bytes fed", st->fed, st->total_len);
    if (st->total_len == 0) {   // one empty leaf
        int rc = sentry::merkle_leaves_into(nullptr, 0, st->leaf_bytes, st->leaf_digests, s);
        if (rc) return rc;
    }
    int rc = sentry::merkle_reduce_into(st->leaf_digests, st->n_leaves, out_digest, s);
    if (rc) return rc;
    // the leaf digests are still being read by the enqueued kernels: hand them to the
    // retired list, which frees them once the stream has passed this point
    rc = sentry::retire_device_memory(st->leaf_digests, s);
    st->magic = 0;
    delete st;
    return rc;
}

int sentry_merkle_stream_abort(void *state)
{
    sentry::clear_error();
    MerkleStream *st = static_cast<MerkleStream *>(state);
    SENTRY_REQUIRE(st && st->magic == STREAM_MAGIC, "sentry_merkle_stream_abort: bad state");
    SENTRY_HIP_CHECK(hipDeviceSynchronize());
    SENTRY_HIP_CHECK(hipFree(st->leaf_digests));
    st->magic = 0;
    delete st;
    return SENTRY_OK;
}

int sentry_merkle_root_h2d(const void *host_buf, size_t len, size_t leaf_bytes, size_t chunk_bytes,
                           uint8_t *out_digest, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(leaf_bytes > 0 && leaf_bytes % 64 == 0,
                   "sentry_merkle_root_h2d: leaf_bytes must be a positive multiple of 64 (got %zu)", leaf_bytes);
    SENTRY_REQUIRE(chunk_bytes > 0 && chunk_bytes % leaf_bytes == 0,
                   "sentry_merkle_root_h2d: chunk_bytes must be a positive multiple of leaf_bytes");
    SENTRY_REQUIRE(host_buf != nullptr || len == 0, "sentry_merkle_root_h2d: NULL buffer");
    SENTRY_REQUIRE((reinterpret_cast<uintptr_t>(host_buf) & 15) == 0, "sentry_merkle_root_h2d: buffer not 16-byte aligned");
    SENTRY_REQUIRE(out_digest != nullptr, "sentry_merkle_root_h2d: NULL out_digest");
    uint64_t n_leaves = ceil_div(len, leaf_bytes);
    if (n_leaves == 0) n_leaves = 1;

    void *stage[2], *digests;
    const size_t stage_bytes = len < chunk_bytes ? (len ? len : 256) : chunk_bytes;
    int rc = sentry::scratch_get(s, sentry::R_STAGE0, stage_bytes, &stage[0]);
    if (rc) return rc;
    rc = sentry::scratch_get(s, sentry::R_STAGE1, stage_bytes, &stage[1]);
    if (rc) return rc;
    rc = sentry::scratch_get(s, sentry::R_NODES_B, 32 * n_leaves, &digests);
    if (rc) return rc;
    sentry::CopyPipe *pipe;
    rc = sentry::copy_pipe_get(s, false, &pipe);
    if (rc) return rc;

    // the side stream must not start overwriting the staging buffers before earlier work on
    // the caller's stream (a previous call's kernels) has finished with them
    SENTRY_HIP_CHECK(hipEventRecord(pipe->consumed[0], s));
    SENTRY_HIP_CHECK(hipEventRecord(pipe->consumed[1], s));

    const uint8_t *src = static_cast<const uint8_t *>(host_buf);
    const uint8_t *readable = kernel_readable(host_buf, len);
    // the enqueue loop; if it fails half way the side stream is drained before the call returns, so
    // that no load still writes a staging buffer that a later call may replace
    auto enqueue_all = [&]() -> int {
    size_t off = 0;
    uint64_t k = 0;
    do {
        const size_t sz = len - off < chunk_bytes ? len - off : chunk_bytes;
        const int b = (int)(k & 1);
        SENTRY_HIP_CHECK(hipStreamWaitEvent(pipe->copy_stream, pipe->consumed[b], 0));
        // chunk starts are multiples of leaf_bytes, so source and staging buffer are both 16-byte aligned
        rc = enqueue_load(static_cast<uint8_t *>(stage[b]), src + off, readable ? readable + off : nullptr, sz,
                          pipe->copy_stream);
        if (rc) return rc;
        SENTRY_HIP_CHECK(hipEventRecord(pipe->copied[b], pipe->copy_stream));
        SENTRY_HIP_CHECK(hipStreamWaitEvent(s, pipe->copied[b], 0));
        rc = sentry::merkle_leaves_into(stage[b], sz, leaf_bytes,
                                        static_cast<uint8_t *>(digests) + 32 * (off / leaf_bytes), s);
        if (rc) return rc;
        SENTRY_HIP_CHECK(hipEventRecord(pipe->consumed[b], s));
        off += sz;
        k++;
    } while (off < len);
    return SENTRY_OK;
    };
    if ((rc = enqueue_all())) {
        sentry::copy_pipe_drain(pipe, false);
        return rc;
    }
    return sentry::merkle_reduce_into(static_cast<const uint8_t *>(digests), n_leaves, out_digest, s);
}

int sentry_lthash_h2d(const void *host_records, const uint64_t *host_offsets, size_t n, size_t batch_bytes,
                      uint16_t *out_lanes, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(out_lanes != nullptr && (reinterpret_cast<uintptr_t>(out_lanes) & 1) == 0,
                   "sentry_lthash_h2d: out_lanes must be non-NULL and 2-byte aligned");
    SENTRY_REQUIRE(batch_bytes > 0, "sentry_lthash_h2d: batch_bytes must be positive");
    SENTRY_REQUIRE(n == 0 || host_offsets != nullptr, "sentry_lthash_h2d: NULL offsets");
    if (n == 0) return sentry::lthash_into(nullptr, nullptr, 0, 0, out_lanes, false, s);
    SENTRY_REQUIRE(host_records != nullptr || host_offsets[n] == host_offsets[0], "sentry_lthash_h2d: NULL records");

    // cut the records into batches of at most batch_bytes at record boundaries (host side,
    // offsets are host memory here); also the largest batch, to size the staging buffers
    struct Batch { size_t first, count; };
    std::vector<Batch> batches;
    size_t max_bytes = 0, max_count = 0;
    for (size_t i = 0; i < n;) {
        size_t j = i;
        while (j < n && host_offsets[j + 1] - host_offsets[i] <= batch_bytes) {
            SENTRY_REQUIRE(host_offsets[j + 1] >= host_offsets[j], "sentry_lthash_h2d: offsets decrease at record %zu", j);
            j++;
        }
        SENTRY_REQUIRE(j > i, "sentry_lthash_h2d: record %zu is longer than batch_bytes", i);
        batches.push_back(Batch{i, j - i});
        const size_t bytes = host_offsets[j] - host_offsets[i];
        if (bytes > max_bytes) max_bytes = bytes;
        if (j - i > max_count) max_count = j - i;
        i = j;
    }

    // pre-size everything for the largest batch, so that no buffer is replaced while the pipeline runs
    void *p, *sums;
    int rc;
    sentry::CopyPipe *pipe;
    if ((rc = sentry::copy_pipe_get(s, true, &pipe))) return rc;
    const int used = batches.size() < (size_t)LT_SLOTS ? (int)batches.size() : LT_SLOTS;
    for (int i = 0; i < used; i++)
        if (sentry::scratch_capacity(s, LT_STAGE_R[i]) < max_bytes + 32 ||
            sentry::scratch_capacity(s, LT_OFF_R[i]) < 8 * (max_count + 1) + 16) {
            sentry::copy_pipe_drain(pipe, true);   // a buffer will be replaced: the side streams must be done with it
            break;
        }
    for (int i = 0; i < used; i++) {
        if ((rc = sentry::scratch_get(s, LT_STAGE_R[i], max_bytes + 32, &p))) return rc;
        if ((rc = sentry::scratch_get(s, LT_OFF_R[i], 8 * (max_count + 1) + 16, &p))) return rc;
        if ((rc = sentry::lthash_presize(max_count, i == 0 ? s : pipe->hash_stream[i - 1]))) return rc;
    }
    if ((rc = sentry::scratch_get(s, sentry::R_LT_SUM, (size_t)LT_SLOTS * 2 * SENTRY_LANES, &sums))) return rc;
    LtStream st = {LT_STREAM_MAGIC, 0, static_cast<uint16_t *>(sums), false, s, nullptr, false};
    const uint8_t *src = static_cast<const uint8_t *>(host_records);
    for (const Batch &bt : batches) {
        // a failure half way leaves loads and hashes queued on the side streams that the caller's
        // stream does not wait for: drain them before returning, they use this stream's staging memory
        if ((rc = lt_stream_feed(&st, src, host_offsets + bt.first, bt.count, s))) {
            sentry::copy_pipe_drain(pipe, true);
            return rc;
        }
    }
    if ((rc = lt_stream_finish(&st, out_lanes, s))) {
        sentry::copy_pipe_drain(pipe, true);
        return rc;
    }
    return SENTRY_OK;
}

static int lt_stream_begin(const char *fn, void **state, bool narrow)
{
    sentry::clear_error();
    SENTRY_REQUIRE(state != nullptr, "%s: NULL state", fn);
    LtStream *st = new (std::nothrow) LtStream();
    if (!st) { sentry::set_error("%s: out of host memory", fn); return SENTRY_ERR_NOMEM; }
    (void)sentry::sweep_retired();
    void *p = nullptr;
    const hipError_t e = hipMalloc(&p, (size_t)LT_SLOTS * 2 * SENTRY_LANES);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        sentry::set_error("%s: %s", fn, hipGetErrorString(e));
        delete st;
        return SENTRY_ERR_NOMEM;
    }
    *st = LtStream{LT_STREAM_MAGIC, 0, static_cast<uint16_t *>(p), true, nullptr, nullptr, narrow};
    *state = st;
    return SENTRY_OK;
}

int sentry_lthash_stream_begin(void **state) { return lt_stream_begin("sentry_lthash_stream_begin", state, false); }

int sentry_lthash32_stream_begin(void **state) { return lt_stream_begin("sentry_lthash32_stream_begin", state, true); }

int sentry_lthash_stream_update_h2d(void *state, const void *host_records, const uint64_t *host_offsets, size_t n,
                                    void *stream)
{
    sentry::clear_error();
    LtStream *st = static_cast<LtStream *>(state);
    SENTRY_REQUIRE(st && st->magic == LT_STREAM_MAGIC, "sentry_lthash_stream_update_h2d: bad state");
    if (n == 0) return SENTRY_OK;
    SENTRY_REQUIRE(host_offsets != nullptr && (reinterpret_cast<uintptr_t>(host_offsets) & 7) == 0,
                   "sentry_lthash_stream_update_h2d: host_offsets must be non-NULL and 8-byte aligned");
    SENTRY_REQUIRE(n <= 0xffffffffull / 4 - 64, "sentry_lthash_stream_update_h2d: too many records");
    SENTRY_REQUIRE(host_offsets[n] >= host_offsets[0], "sentry_lthash_stream_update_h2d: offsets decrease");
    SENTRY_REQUIRE(host_records != nullptr || host_offsets[n] == host_offsets[0], "sentry_lthash_stream_update_h2d: NULL records");
    const int rc = lt_stream_feed(st, static_cast<const uint8_t *>(host_records), host_offsets, n, static_cast<hipStream_t>(stream));
    if (rc && st->pipe) sentry::copy_pipe_drain(st->pipe, true);
    return rc;
}

int sentry_lthash_stream_final(void *state, uint16_t *out_lanes, void *stream)
{
    sentry::clear_error();
    LtStream *st = static_cast<LtStream *>(state);
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(st && st->magic == LT_STREAM_MAGIC, "sentry_lthash_stream_final: bad state");
    SENTRY_REQUIRE(out_lanes != nullptr && (reinterpret_cast<uintptr_t>(out_lanes) & 1) == 0,
                   "sentry_lthash_stream_final: out_lanes must be non-NULL and 2-byte aligned");
    SENTRY_REQUIRE(st->batches == 0 || st->stream == s, "sentry_lthash_stream_final: not the stream the batches were fed on");
    int rc;
    if (st->batches == 0) {                                          // nothing fed: all-zero lanes
        rc = st->narrow ? sentry::lthash32_sum_rows(st->sums, 0, SENTRY_LANES, out_lanes, s)
                        : sentry::lthash_sum_rows(st->sums, 0, out_lanes, s);
    } else if ((rc = lt_stream_finish(st, out_lanes, s))) {
        sentry::copy_pipe_drain(st->pipe, true);
    }
    if (rc) return rc;
    // the sums are still read by the kernel just queued: freed once the stream has passed this point
    rc = sentry::retire_device_memory(st->sums, s);
    st->magic = 0;
    delete st;
    return rc;
}

int sentry_lthash_stream_abort(void *state)
{
    sentry::clear_error();
    LtStream *st = static_cast<LtStream *>(state);
    SENTRY_REQUIRE(st && st->magic == LT_STREAM_MAGIC, "sentry_lthash_stream_abort: bad state");
    SENTRY_HIP_CHECK(hipDeviceSynchronize());
    if (st->owns_sums) SENTRY_HIP_CHECK(hipFree(st->sums));
    st->magic = 0;
    delete st;
    return SENTRY_OK;
}

}  // extern "C"

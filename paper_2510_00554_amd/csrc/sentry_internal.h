// Host-side plumbing shared by the HIP translation units of the library:
// error reporting and the per-stream scratch arena.  No hashing arithmetic here.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <cstdio>

#include "sentry.h"

namespace sentry {

// thread-local error text returned by sentry_last_error()
void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
void clear_error();

#define SENTRY_HIP_CHECK(expr)                                                        \
    do {                                                                              \
        hipError_t _e = (expr);                                                       \
        if (_e != hipSuccess) {                                                       \
            ::sentry::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), \
                                __FILE__, __LINE__);                                  \
            return SENTRY_ERR_HIP;                                                    \
        }                                                                             \
    } while (0)

#define SENTRY_REQUIRE(cond, ...)              \
    do {                                       \
        if (!(cond)) {                         \
            ::sentry::set_error(__VA_ARGS__);  \
            return SENTRY_ERR_INVALID_ARG;     \
        }                                      \
    } while (0)

// Named regions of the per-(device, stream) scratch arena.  Each region is its
// own grow-only device allocation, so a region that grows does not move others.
enum Region {
    R_NODES_A = 0,   // Merkle stage output (leaf stage, even segment stages)
    R_NODES_B,       // Merkle stage output (odd segment stages)
    R_RED_0,         // ping-pong level buffers private to the node reduction
    R_RED_1,
    R_TABLES,        // segment / group tables on the device
    R_SEG_ROOTS,     // per-segment roots when the caller does not want them
    R_LT_H0,         // BLAKE2Xb root hashes, 64 B per record
    R_LT_PART,       // per-workgroup lane partial sums
    R_LT_SUM,        // running lane sum of the host-streaming entry point
    R_LT_ORDER,      // record indices ordered by length for the four-lane root hash
    R_LT_COUNTS,     // per-workgroup bin counts, then places, of the ordering
    R_SRC_TABLES,    // per-source counts, starts, unit starts, cursors
    R_SRC_PERM,      // record indices grouped by source
    R_STAGE0,        // device staging buffers of the host-streaming entry points
    R_STAGE1,
    R_STAGE2,
    R_STAGE_OFF0,    // staged record offsets
    R_STAGE_OFF1,
    R_STAGE_OFF2,
    R_TICKET,        // "last workgroup" counter of the one-launch Merkle tree (zero between launches)
    R_SRC32,         // per-source 32-bit counters of the 32-partition hash (zero between calls)
    R_GATHER,        // blocks of the coalesced scheme that are put together from several tensors
    R_GATHER_TAB,    // copy table of the gather kernel
    R_COUNT
};

// Returns a device pointer of at least `bytes` bytes for (current device, stream, region).
// Growing a region frees the old allocation, which synchronises the device.
int scratch_get(hipStream_t stream, Region r, size_t bytes, void **out);
// Bytes the region holds now (0 if it was never allocated).
size_t scratch_capacity(hipStream_t stream, Region r);
// The same; *fresh is set when the memory was allocated by this call (its contents are undefined).
int scratch_get_fresh(hipStream_t stream, Region r, size_t bytes, void **out, bool *fresh);

// Pinned host staging for tables (per stream): returns a host pointer of >= bytes.  Before
// the memory is reused the previous upload from it has completed (tracked by an event).
// Two independent slots, so that a call which uploads a table of its own and then runs an
// entry point that uploads another does not wait for its first upload.
constexpr int TABLE_SLOTS = 2;
int table_staging_get(hipStream_t stream, size_t bytes, void **host_ptr, int slot = 0);
// Record that an upload from the staging memory was enqueued on `stream`.
int table_staging_mark(hipStream_t stream, int slot = 0);

// Side stream and events for the host-streaming entry points (per stream).
// PIPE_SLOTS = batches in flight in the lattice host-streaming call.  Slot 0 hashes on the
// caller's stream, the others on side streams: with the copy stream that makes four streams,
// the number of hardware queues a process gets by default, so no two of them share a queue.
constexpr int PIPE_SLOTS = 3;
struct CopyPipe {
    hipStream_t copy_stream;
    hipStream_t hash_stream[PIPE_SLOTS - 1];   // side streams for batches hashed concurrently
    hipEvent_t copied[PIPE_SLOTS];     // chunk k%slots has landed in its staging buffer
    hipEvent_t consumed[PIPE_SLOTS];   // the hash kernels have finished reading that staging buffer
    hipEvent_t start;                  // everything enqueued on the caller's stream before the call
    uint64_t chunk_seq;                // chunks fed through sentry_merkle_stream_update_h2d (picks the staging slot)
};
// Error path of the host-streaming calls: wait (on the host) until the pipe's side streams have
// drained, so that nothing still uses the caller stream's staging memory when the call returns.
void copy_pipe_drain(CopyPipe *pipe, bool with_hash_streams);
// with_hash_streams: also create the side hash streams (only the lattice call needs them;
// streams that exist share the few hardware queues even when idle)
int copy_pipe_get(hipStream_t stream, bool with_hash_streams, CopyPipe **out);

// Device memory that kernels already enqueued on `stream` still read: freed by a later
// sweep once the stream has passed the point of this call.
int retire_device_memory(void *dev_ptr, hipStream_t stream);
int sweep_retired();

int release_all_scratch();
// Bytes held for (current device, stream): scratch regions, and pinned table staging.
int scratch_bytes(hipStream_t stream, size_t *device_bytes, size_t *pinned_bytes);

}  // namespace sentry

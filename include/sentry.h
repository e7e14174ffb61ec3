/*
 * sentry.h: C ABI of the MI355X (gfx950) artifact-hashing library.
 *
 * The library hashes ML artifacts that already sit in GPU memory, as in Sentry
 * (CCS '25): a SHA-256 Merkle tree over model-weight bytes and a lattice
 * (homomorphic, LtHash-style) hash over dataset samples.  Every step runs in
 * hand-written HIP kernels; signing and signature checks stay with the caller.
 *
 * Conventions shared by all entry points
 *   - Return value: SENTRY_OK (0) on success, SENTRY_MISMATCH (1) only from
 *     sentry_verify, a negative SENTRY_ERR_* otherwise.  Nothing throws or
 *     aborts.  sentry_last_error() returns a thread-local text for the last
 *     failing call of the calling thread.
 *   - "device" pointers are HIP device allocations of the current device;
 *     "device-accessible" means device memory or pinned host memory (the result
 *     is written by a kernel); "host" means ordinary process memory.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return; outputs are valid once the caller
 *     has synchronised the stream.  Inputs must stay alive and unchanged until
 *     then.  The library never writes to an input and never frees caller memory
 *     (section 4.2.1, "In-place Hashing": the state dict must stay unchanged).
 *   - The library owns its scratch memory (leaf digests, level buffers, lane
 *     partials, tables), allocated lazily per stream and reused; concurrent
 *     calls on one stream from several host threads are not supported.
 *     sentry_release_scratch() frees it.
 *   - Graph capture: sentry_merkle_root, sentry_merkle_root_h, sentry_merkle_leaves,
 *     sentry_merkle_reduce, sentry_lthash, sentry_lthash32, their _fixed forms, sentry_lthash_digests,
 *     sentry_lthash_sum and the combine and remove calls only launch kernels once the
 *     stream's scratch is large enough, so a caller may capture them into a HIP
 *     graph after one plain call with the same sizes on the same stream; the graph
 *     then refers to that stream's scratch, which must not be released, or grown
 *     by a larger plain call, while the graph is in use.  The entry points that
 *     take tensor lists or host memory upload tables or run their own pipeline of
 *     streams and are not meant for capture.
 *   - Digests are the 32 bytes of FIPS 180-4 SHA-256 in their usual byte order.
 *     Lattice digests are SENTRY_LANES uint16 values.
 */
#ifndef SENTRY_H
#define SENTRY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* the library is built with hidden visibility; only these entry points are exported */
#define SENTRY_API __attribute__((visibility("default")))

enum {
    SENTRY_OK = 0,
    SENTRY_MISMATCH = 1,
    SENTRY_ERR_INVALID_ARG = -1,
    SENTRY_ERR_HIP = -2,
    SENTRY_ERR_NOMEM = -3
};

#define SENTRY_DIGEST_BYTES 32
/* leaf functions of sentry_merkle_root_h */
#define SENTRY_HASH_SHA256 0
#define SENTRY_HASH_BLAKE2B 1      /* BLAKE2b-512, 64-byte nodes */
#define SENTRY_HASH_SHA3_256 2     /* 32-byte nodes */
#define SENTRY_LANES 1024
#define SENTRY_LANES32 32   /* lanes of the 32-partition lattice hash (section 4.2.2) */
#define SENTRY_MODEL_LANES 32

/* ------------------------------------------------------------------------ */
/* Merkle tree over weight bytes (section 2.2 "Merkle Tree"; section 4.2.1) */
/* ------------------------------------------------------------------------ */

/*
 * Root of the binary SHA-256 Merkle tree over one contiguous device buffer
 * (Algorithm 1 once the tensors are one buffer; block hashing kernel and
 * reduction kernel of section 4.2.1).
 *   leaf i   = bytes [i*leaf_bytes, min((i+1)*leaf_bytes, len)); the last leaf
 *              may be short and is hashed at its true length; len == 0 is one
 *              empty leaf.
 *   node     = SHA-256(left || right); a level's lone last node moves up
 *              unchanged.
 * dev_buf     device, 16-byte aligned (may be NULL only if len == 0).
 * leaf_bytes  > 0 and a multiple of 64.
 * out_digest  device-accessible, 32 bytes.
 * Errors: SENTRY_ERR_INVALID_ARG for NULL/misaligned pointers or a bad
 * leaf_bytes; SENTRY_ERR_NOMEM / SENTRY_ERR_HIP if scratch or a launch fails.
 */
SENTRY_API int sentry_merkle_root(const void *dev_buf, size_t len, size_t leaf_bytes,
                       uint8_t *out_digest, void *stream);

/*
 * sentry_merkle_root for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * result, same kernels, but the workgroup nodes, level buffers and the ticket
 * counter live in one fixed device array of the library (about 2 MiB, held on
 * every GPU the library runs on until the process ends) instead of the
 * per-stream scratch, and the call makes no hipMalloc, hipFree or other
 * allocating call, first call included.
 * Limit: at most 4,194,304 leaves (len <= 4,194,304 * leaf_bytes); more is
 * SENTRY_ERR_INVALID_ARG, and sentry_merkle_root takes such inputs.
 * All calls on one GPU share the array, whatever their stream: calls that
 * overlap in time on one GPU race and give undefined digests; calls ordered one
 * after the other (one stream, or events) are safe.
 */
SENTRY_API int sentry_merkle_root_noalloc(const void *dev_buf, size_t len, size_t leaf_bytes,
                                          uint8_t *out_digest, void *stream);

/*
 * The same tree over one of the paper's three leaf functions (section 4.2.1:
 * SHA256, BLAKE2B and SHA3): node = H(left || right) with the full hash H, same
 * leaf, short-tail, odd-node and empty-buffer rules as sentry_merkle_root.
 * hash        SENTRY_HASH_SHA256 (identical to sentry_merkle_root),
 *             SENTRY_HASH_BLAKE2B or SENTRY_HASH_SHA3_256.
 * out_digest  device-accessible, 32 bytes (64 for BLAKE2b).
 * Other arguments and errors as for sentry_merkle_root.
 */
SENTRY_API int sentry_merkle_root_h(int hash, const void *dev_buf, size_t len, size_t leaf_bytes,
                                    uint8_t *out_digest, void *stream);

/*
 * Per-tensor trees and the model digest over them (Algorithm 2, per-layer
 * hashing) in one table-driven launch over fragmented tensors (the lookup
 * table of section 4.2.1, "In-place Hashing").
 *   seg_root[t] = sentry_merkle_root of tensor t (same leaf rules);
 *   out_root    = the pairwise reduction of [seg_root[0..n_seg)] taken as
 *                 ready-made nodes (they are not hashed again as leaves).
 * dev_ptrs       host array of n_seg device pointers, each 16-byte aligned.
 * lens           host array of n_seg byte lengths.
 * out_seg_roots  device-accessible, n_seg*32 bytes, or NULL if not wanted.
 * out_root       device-accessible, 32 bytes.
 * n_seg >= 1.  The two host arrays are read before the call returns.
 */
SENTRY_API int sentry_merkle_segments(const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                           size_t leaf_bytes, uint8_t *out_seg_roots, uint8_t *out_root,
                           void *stream);

/*
 * In-place hashing (Algorithm 3): ONE flat tree whose leaves are the blocks of
 * all tensors in order, hashed where they lie by one table-driven launch (the
 * lookup table of section 4.2.1: per range of lanes the tensor's address, block
 * size and length).  The last block of a tensor is short, never padded and
 * never completed from the next tensor; a tensor of length 0 has no block; if no
 * tensor has a block the root is that of the single empty leaf.  When every
 * length is a multiple of leaf_bytes the root equals sentry_merkle_root over the
 * concatenated tensors.
 * Arguments as for sentry_merkle_segments (host arrays of device pointers and
 * lengths, read before the call returns); out_root device-accessible, 32 bytes.
 */
SENTRY_API int sentry_merkle_inplace(const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                                     size_t leaf_bytes, uint8_t *out_root, void *stream);

/*
 * Per-tensor trees (Algorithm 2) and the in-place flat tree (Algorithm 3) over any
 * of the three leaf functions: same rules as sentry_merkle_segments and
 * sentry_merkle_inplace with H in place of SHA-256 (an empty tensor's root is
 * H("") in the per-tensor scheme and it has no block in the flat one).
 * hash           as for sentry_merkle_root_h; SENTRY_HASH_SHA256 gives exactly the
 *                two functions above.
 * out_seg_roots  device-accessible, n_seg digests of 32 bytes (64 for BLAKE2b),
 *                or NULL.
 * out_root       device-accessible, one digest.
 * Other arguments and errors as for sentry_merkle_segments.
 */
SENTRY_API int sentry_merkle_segments_h(int hash, const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                                        size_t leaf_bytes, uint8_t *out_seg_roots, uint8_t *out_root,
                                        void *stream);
SENTRY_API int sentry_merkle_inplace_h(int hash, const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                                       size_t leaf_bytes, uint8_t *out_root, void *stream);

/*
 * Coalesced hashing (Algorithm 1; section 4.2.1, "Coalesced Hashing"): the root
 * of the Merkle tree over ONE buffer that holds the tensors one behind the
 * other, in order, without gaps; the buffer is a whole number of blocks long
 * and the bytes behind the last tensor are zero (the paper does not give the
 * fill value).  Blocks run across tensor boundaries, so the root depends on the
 * concatenated bytes only, not on where one tensor ends: it equals
 * sentry_merkle_root_h over the zero-padded concatenation.
 * dev_ptrs, lens, n_seg  host arrays (read before the call returns) of n_seg >= 1
 *              device pointers and byte lengths; ANY alignment and length; a
 *              pointer may be NULL where its length is 0.  Not modified.
 * leaf_bytes   block size, a positive multiple of 64.
 * dev_buffer   device, 16-byte aligned, at least ceil(total / leaf_bytes) *
 *              leaf_bytes bytes (buffer_bytes says how many it has), disjoint
 *              from every tensor: the scheme as stated.  A copy kernel lays the
 *              tensors into it and clears the padding, then the tree runs over
 *              it; on return (once the stream has been synchronised) it holds
 *              the coalesced model.  Bytes behind the padded size are not
 *              touched.
 *              NULL (buffer_bytes ignored): the same root without the second
 *              copy of the model.  Only blocks that hold bytes of more than one
 *              tensor, the padded last block, and blocks whose bytes are not
 *              16-byte aligned in their tensor are put together in library
 *              scratch (at most one block per tensor when all tensors are
 *              16-byte aligned and their lengths multiples of 16); all other
 *              blocks are hashed where they lie.
 * out_root     device-accessible, one digest (32 bytes, 64 for BLAKE2b).
 * hash         as for sentry_merkle_root_h; sentry_merkle_coalesced is SHA-256.
 * No byte at all (every length 0) gives the root of the single empty leaf.
 * Errors: SENTRY_ERR_INVALID_ARG for a NULL argument, an unknown hash, a bad
 * leaf_bytes, a buffer that is too small, misaligned or overlaps a tensor;
 * SENTRY_ERR_NOMEM / SENTRY_ERR_HIP from scratch or a launch.  Uploads a table:
 * not meant for graph capture.
 */
SENTRY_API int sentry_merkle_coalesced(const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                                       size_t leaf_bytes, void *dev_buffer, size_t buffer_bytes,
                                       uint8_t *out_root, void *stream);
/*
 * What the call above would do with dev_buffer == NULL, without doing it (host
 * only, no GPU work; the pointers are looked at, never followed):
 * out_gathered_bytes  bytes of library scratch the gathered blocks take (a
 *                     multiple of leaf_bytes);
 * out_copied_bytes    bytes of the tensors that are copied into them (the rest
 *                     of the scratch is the zero padding of the last block);
 * out_runs            runs of whole blocks the leaf stage is given.
 * Each may be NULL.  Errors: SENTRY_ERR_INVALID_ARG as above.
 */
SENTRY_API int sentry_merkle_coalesced_plan(const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                                            size_t leaf_bytes, size_t *out_gathered_bytes,
                                            size_t *out_copied_bytes, size_t *out_runs);
SENTRY_API int sentry_merkle_coalesced_h(int hash, const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                                         size_t leaf_bytes, void *dev_buffer, size_t buffer_bytes,
                                         uint8_t *out_root, void *stream);

/*
 * The block hashing kernel alone: the max(1, ceil(len/leaf_bytes)) leaf digests
 * of a buffer, 32 bytes each, in leaf order (section 4.2.1).
 * out_leaf_digests  device, 16-byte aligned, 32 bytes per leaf.
 */
SENTRY_API int sentry_merkle_leaves(const void *dev_buf, size_t len, size_t leaf_bytes,
                         uint8_t *out_leaf_digests, void *stream);

/*
 * The reduction kernel alone: n >= 1 ready-made 32-byte nodes to one root by
 * the pairwise rule above (section 4.2.1; HashReduce in Algorithms 1-3).
 * dev_nodes   device, 16-byte aligned, n*32 bytes, not modified.
 */
SENTRY_API int sentry_merkle_reduce(const uint8_t *dev_nodes, size_t n, uint8_t *out_digest, void *stream);

/*
 * One tree over a byte stream that arrives in chunks already on the device.
 * begin   sizes the state for total_len bytes and leaf_bytes; *state is an
 *         opaque handle owned by the library until final (or abort).
 * update  hashes the leaves of the next chunk; every chunk but the last must be
 *         a multiple of leaf_bytes; the chunk buffer may be reused once the
 *         stream has passed the update.  dev_chunk: device, 16-byte aligned.
 * final   reduces the leaf digests to the root (equal to sentry_merkle_root over
 *         the concatenated chunks), writes it to out_digest (device-accessible)
 *         and releases the state after the stream has drained it.
 *         SENTRY_ERR_INVALID_ARG if fewer than total_len bytes were fed.
 * abort   releases a state without a result.
 * update_h2d  the same as update for a chunk that still sits in host memory (section
 *         4.4: the model is authenticated while it is loaded): the chunk is loaded
 *         on a side stream into one of two staging buffers the library holds per
 *         caller stream (each as large as the largest chunk fed so far) and hashed
 *         on `stream` once it has landed, so that the load of one chunk overlaps
 *         the hashing of the one before when the caller feeds chunks without
 *         waiting in between.  host_chunk: host, 16-byte aligned; pinned memory is
 *         read by a load kernel at the PCIe rate, pageable memory goes through
 *         hipMemcpyAsync; it must stay unchanged until `stream` has passed the
 *         update (record an event after the call to learn when).  Chunks of one
 *         tree are fed on one stream; update and update_h2d may be mixed.
 */
SENTRY_API int sentry_merkle_stream_begin(size_t total_len, size_t leaf_bytes, void **state);
SENTRY_API int sentry_merkle_stream_update(void *state, const void *dev_chunk, size_t len, void *stream);
SENTRY_API int sentry_merkle_stream_update_h2d(void *state, const void *host_chunk, size_t len, void *stream);
SENTRY_API int sentry_merkle_stream_final(void *state, uint8_t *out_digest, void *stream);
SENTRY_API int sentry_merkle_stream_abort(void *state);

/*
 * Hash while loading (section 4.4: authentication on the fly as the model is
 * loaded; a load on a side stream stands in for the paper's GPUDirect loads):
 * the root of the tree over a host buffer, loaded in chunks on a side stream
 * into two device staging buffers while the previous chunk is hashed on
 * `stream`.  Equal to sentry_merkle_root over the same bytes.
 * host_buf     host, 16-byte aligned.  Pinned memory (hipHostMalloc) is read
 *              directly by a small load kernel at the PCIe rate and overlaps
 *              with the hashing; pageable memory goes through hipMemcpyAsync,
 *              which works but serialises.  A device pointer is accepted too.
 * chunk_bytes  > 0 and a multiple of leaf_bytes; two device buffers of this
 *              size are held in the library's scratch.
 * The call returns after enqueuing everything; host_buf must stay unchanged
 * until `stream` is synchronised.
 */
SENTRY_API int sentry_merkle_root_h2d(const void *host_buf, size_t len, size_t leaf_bytes,
                           size_t chunk_bytes, uint8_t *out_digest, void *stream);

/* Constant-time comparison of two host digests: the check of a recomputed model
 * digest against the expected one (section 4.1.1).  SENTRY_OK if equal, SENTRY_MISMATCH if not,
 * SENTRY_ERR_INVALID_ARG for NULL. */
SENTRY_API int sentry_verify(const uint8_t *root, const uint8_t *expected);

/* ------------------------------------------------------------------------ */
/* Lattice hash over dataset samples (section 2.2 Eq. (1); 4.2.2; 4.3)      */
/* ------------------------------------------------------------------------ */

/*
 * out_lanes[l] = sum over records i of h(record_i)[l] mod 2^16, l < 1024
 * (Eq. (1) with q = 2^16; one block per sample, section 4.3).  h(M) is
 * BLAKE2Xb(M) with 2048 output bytes read as little-endian uint16 lanes: a
 * BLAKE2b-512 root hash carrying the XOF length, expanded by 32 one-block
 * BLAKE2b calls.  Records with equal bytes count once each (multiset).
 * dev_records  device; record i = bytes [offsets[i], offsets[i+1]) of it; any
 *              alignment; may be NULL if every record is empty.  The kernels
 *              read whole aligned 4-byte words, so up to 3 bytes on either side
 *              of a record may be read (never past the word that holds a byte
 *              of the record).
 * dev_offsets  device, n+1 non-decreasing uint64 byte offsets (8-byte aligned);
 *              offsets[0] need not be 0.  Monotonicity is not checked: the
 *              result is undefined, and reads may fault, if it is violated.
 * n            number of records; 0 gives all-zero lanes (dev_offsets may be
 *              NULL then).
 * out_lanes    device-accessible, 1024 uint16 (2-byte aligned), overwritten.
 */
SENTRY_API int sentry_lthash(const void *dev_records, const uint64_t *dev_offsets, size_t n,
                  uint16_t *out_lanes, void *stream);

/*
 * The same for samples of one size laid back to back, which is how section 4.3
 * runs the dataset kernel (its block size is the size of one sample: 32x32x3
 * bytes for images, the padded length for text): record i = bytes
 * [i * record_bytes, (i + 1) * record_bytes) of dev_records, no offsets array.
 * The host then knows all about the batch and launches only the kernels that
 * have work.  out_lanes equals sentry_lthash (sentry_lthash32 for the second
 * call, 32 uint16) over the same records.
 * dev_records   device, any alignment; may be NULL when n or record_bytes is 0.
 * record_bytes  any size; 0 makes n empty records.
 * n             number of records (0 gives all-zero lanes).
 * Errors: SENTRY_ERR_INVALID_ARG for NULL or misaligned out_lanes, NULL records
 * with bytes to read, n > 2^30 - 65 or n * record_bytes beyond 2^64.
 */
SENTRY_API int sentry_lthash_fixed(const void *dev_records, size_t record_bytes, size_t n,
                                   uint16_t *out_lanes, void *stream);
SENTRY_API int sentry_lthash32_fixed(const void *dev_records, size_t record_bytes, size_t n,
                                     uint16_t *out_lanes, void *stream);

/*
 * Batches that mix data sources (section 4.1.2: shuffled batches hold samples of
 * several providers; section 4.3: a dictionary maps each source to its samples, one
 * reduction per source, each result added to that source's running sum):
 *   acc_lanes[k][l] += sum over records i with source_id[i] == k of h(record_i)[l]
 * mod 2^16, for every source k < n_sources, in one call per batch.  With one
 * source and acc zeroed this is sentry_lthash.
 * dev_records, dev_offsets, n   as for sentry_lthash.
 * dev_source_ids  device, n uint32 (4-byte aligned); a record whose id is not
 *                 below n_sources is left out of every sum.
 * n_sources       1 .. 4096.
 * acc_lanes       device-accessible, n_sources rows of 1024 uint16 (2-byte
 *                 aligned), read and updated: the caller zeroes it before the
 *                 first batch and carries it from batch to batch.
 */
SENTRY_API int sentry_lthash_sources(const void *dev_records, const uint64_t *dev_offsets,
                                     const uint32_t *dev_source_ids, size_t n, size_t n_sources,
                                     uint16_t *acc_lanes, void *stream);

/*
 * The digests of Eq. (1) one by one, and Eq. (1) over digests that are already
 * in memory.  A provider that keeps every sample's digest can take a sample out
 * of a dataset hash, or build the hash of any subset, without the samples' bytes
 * (section 2.2: add and remove by lattice addition).
 *   sentry_lthash_digests: out_digests[i][l] = h(record_i)[l], i < n, l < 1024
 *   sentry_lthash_sum:     out_lanes[l] = sum over i < n of dev_digests[i][l] mod 2^16
 * so that sum(digests(records)) == sentry_lthash(records).
 * dev_records, dev_offsets, n   as for sentry_lthash.
 * out_digests  device, n rows of 1024 uint16 (2048 bytes each, 16-byte aligned),
 *              overwritten; nothing is written for n == 0.
 * dev_digests  device, n rows of 1024 uint16, 16-byte aligned; not modified.  May
 *              be NULL when n == 0, which gives all-zero lanes.
 * out_lanes    device-accessible, 1024 uint16 (2-byte aligned), overwritten.
 */
SENTRY_API int sentry_lthash_digests(const void *dev_records, const uint64_t *dev_offsets, size_t n,
                                     uint16_t *out_digests, void *stream);
SENTRY_API int sentry_lthash_sum(const uint16_t *dev_digests, size_t n, uint16_t *out_lanes, void *stream);

/* acc[l] = (acc[l] + x[l]) mod 2^16 and (acc[l] - x[l]) mod 2^16 (section 2.2:
 * LtHash(S1)+LtHash(S2) = LtHash(S1 u S2), LtHash(S1 u S2)-LtHash(S1) =
 * LtHash(S2); the lattice addition of section 4.2.2).  Both device-accessible,
 * 1024 uint16, 2-byte aligned; x is not modified; acc == x is allowed. */
SENTRY_API int sentry_lthash_combine(uint16_t *acc, const uint16_t *x, void *stream);
SENTRY_API int sentry_lthash_remove(uint16_t *acc, const uint16_t *x, void *stream);

/*
 * The lattice hash at the digest width section 4.2.2 describes: every sample is
 * hashed by plain unkeyed BLAKE2b with a 64-byte digest, the digest is cut into
 * 32 partitions of 16 bits (little-endian, in digest order), and partition l of
 * all samples is summed mod 2^16:
 *   out_lanes[l] = sum_i BLAKE2b-512(record_i)[2l .. 2l+1] mod 2^16, l < 32.
 * (sentry_lthash is the same sum over 1024 lanes of the extended-output hash;
 * this one is the 64-byte form.)  Records, offsets and n as for sentry_lthash
 * (same alignment rules, same over-read of up to 3 bytes, n == 0 gives zeros).
 * out_lanes    device-accessible, 32 uint16 (2-byte aligned), overwritten.
 * sentry_lthash32_combine / _remove are the lattice addition and subtraction on
 * such 32-lane values (acc and x device-accessible, 32 uint16 each, 2-byte
 * aligned; x is not modified; acc == x is allowed).
 * sentry_lthash32_sources is sentry_lthash_sources at this width (section 4.3:
 * one running sum per data source): acc_lanes holds n_sources (1 .. 4096) rows
 * of 32 uint16, row k is increased by the digests of the records whose
 * dev_source_ids entry is k; ids not below n_sources are left out; arguments
 * otherwise as for sentry_lthash_sources.
 * Errors: SENTRY_ERR_INVALID_ARG for NULL or misaligned pointers or n > 2^30 - 65;
 * SENTRY_ERR_NOMEM / SENTRY_ERR_HIP from the scratch allocation or a launch.
 * Like sentry_lthash, the calls only launch kernels once the stream's scratch
 * is large enough.
 */
SENTRY_API int sentry_lthash32(const void *dev_records, const uint64_t *dev_offsets, size_t n,
                               uint16_t *out_lanes, void *stream);
SENTRY_API int sentry_lthash32_sources(const void *dev_records, const uint64_t *dev_offsets,
                                       const uint32_t *dev_source_ids, size_t n, size_t n_sources,
                                       uint16_t *acc_lanes, void *stream);
SENTRY_API int sentry_lthash32_combine(uint16_t *acc, const uint16_t *x, void *stream);
SENTRY_API int sentry_lthash32_remove(uint16_t *acc, const uint16_t *x, void *stream);

/*
 * Lattice hash of records that sit in host memory, loaded in batches on a side
 * stream (by the load kernel or hipMemcpyAsync, as for sentry_merkle_root_h2d)
 * while the previous batch is hashed, the running sum carried across
 * batches (section 4.3: per-batch digests added to a running sum).  Equal to
 * sentry_lthash over the same records.
 * host_records  host (pinned for overlap); host_offsets: host, n+1 offsets.
 * batch_bytes   upper bound on the record bytes copied per batch (> 0); a
 *               record longer than this is an error.  Batches are cut at record
 *               boundaries.  Up to three batches are in flight, each with a
 *               device buffer of its size (held in scratch) and a stream of
 *               its own, so that the hashing of one batch, which is bound
 *               by its longest record, overlaps the copies and hashes of the
 *               next ones.
 * out_lanes     device-accessible, overwritten with the sum over all n records.
 */
SENTRY_API int sentry_lthash_h2d(const void *host_records, const uint64_t *host_offsets, size_t n,
                      size_t batch_bytes, uint16_t *out_lanes, void *stream);

/*
 * The running sum over a dataset that arrives batch by batch from host memory
 * (section 4.3: the digest of every batch is added to a running sum; section 4.4:
 * while the data is loaded).  The same pipeline as sentry_lthash_h2d, fed one
 * batch per call, so that the host needs to hold only the batches in flight:
 * batch k is loaded on a side stream into one of three staging buffers (held per
 * caller stream, each as large as the largest batch fed so far) and hashed on
 * one of three streams while batches k+1 and k+2 load, each stream keeping its
 * own running sum.
 * begin       creates the state (an opaque handle owned by the library).
 * update_h2d  feeds n records: record i = host_records[host_offsets[i],
 *             host_offsets[i+1]), offsets as for sentry_lthash but in host memory
 *             (n+1 of them, 8-byte aligned).  Pinned memory is read by the load
 *             kernel at the PCIe rate; pageable memory goes through hipMemcpyAsync.
 *             Both host arrays must stay unchanged until `stream` has passed the
 *             call (it waits for the batch's load, not for its hash).  All batches
 *             of one state are fed on one stream.  n == 0 does nothing.  The call
 *             reads the offsets on the host: a batch whose records all have one
 *             size is hashed as sentry_lthash_fixed hashes it, and its offsets
 *             are not loaded to the device.
 * final       waits on `stream` for the hashes still running on the side streams,
 *             writes the sum over all records fed to out_lanes (device-accessible,
 *             1024 uint16; all zero if nothing was fed) and releases the state.
 * abort       releases a state without a result (synchronises the device).
 * The result equals sentry_lthash over all the records in any order.
 * sentry_lthash32_stream_begin creates a state for the 32-partition hash
 * instead: update_h2d and abort are the same calls, final writes 32 uint16 to
 * out_lanes, and the result equals sentry_lthash32 over all the records.
 */
SENTRY_API int sentry_lthash_stream_begin(void **state);
SENTRY_API int sentry_lthash32_stream_begin(void **state);
SENTRY_API int sentry_lthash_stream_update_h2d(void *state, const void *host_records, const uint64_t *host_offsets,
                                               size_t n, void *stream);
SENTRY_API int sentry_lthash_stream_final(void *state, uint16_t *out_lanes, void *stream);
SENTRY_API int sentry_lthash_stream_abort(void *state);

/*
 * Lattice hash of a model (section 4.2.2, Algorithm 4).  The blocks of all
 * tensors, in tensor order, are numbered 0, 1, 2, ... across the model; block k
 * (block_bytes bytes, the last block of a tensor may be short, a tensor of
 * length 0 has none) has the digest BLAKE2b-512(LE64(k) || block), read as 32
 * little-endian uint16 partitions (the 64-byte digest of section 4.2.2).
 *   out_layer_lanes[t][l] = sum of the digests of tensor t's blocks,
 *   out_lanes[l]          = sum over all blocks = sum of the tensor digests,
 * every partition mod 2^16.  The index in front of each block is what makes the
 * order-invariant sum sensitive to block order (section 2.2).
 * dev_ptrs, lens   host arrays as for sentry_merkle_segments (16-byte aligned
 *                  device pointers), read before the call returns.
 * block_bytes      > 0 and a multiple of 16 (the paper's default is 8192).
 * out_layer_lanes  device-accessible, n_seg rows of 32 uint16, or NULL.
 * out_lanes        device-accessible, 32 uint16.  Both overwritten.
 */
SENTRY_API int sentry_lthash_model(const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                                   size_t block_bytes, uint16_t *out_layer_lanes, uint16_t *out_lanes,
                                   void *stream);
/*
 * The same for a run of tensors out of a model: their blocks are numbered from
 * first_index (the number of blocks of the tensors in front of them) instead of
 * 0.  The digests of disjoint runs add up to the model's (section 2.2: the sum
 * over a union is the sum of the sums), so after a change to some tensors the
 * model digest is brought up to date from their digests alone:
 *   model' = model - digest(old tensor) + digest(new tensor)
 * with sentry_lthash32_remove and sentry_lthash32_combine on the 32 partitions.
 * Other arguments and errors as for sentry_lthash_model (which is this call with
 * first_index 0).
 */
SENTRY_API int sentry_lthash_model_from(const void *const *dev_ptrs, const size_t *lens, size_t n_seg,
                                        size_t block_bytes, uint64_t first_index,
                                        uint16_t *out_layer_lanes, uint16_t *out_lanes, void *stream);

/* ------------------------------------------------------------------------ */

/* Text for the calling thread's last failing call ("" if none). */
SENTRY_API const char *sentry_last_error(void);

/*
 * Take the scratch memory of later calls now (for callers that want those calls
 * to return without waiting and to be fit for graph capture from the first one;
 * not a step of the paper).  Grows, on `stream`, the scratch of
 *   - sentry_merkle_root, sentry_merkle_leaves and sentry_merkle_reduce for inputs
 *     of up to merkle_max_len bytes in leaves of merkle_leaf_bytes (0 = leave the
 *     Merkle scratch alone), and
 *   - sentry_lthash, sentry_lthash32, their _fixed forms, sentry_lthash_digests and
 *     sentry_lthash_sum for up to lthash_max_records records or digests (0 = leave
 *     it alone),
 * to what the largest such call needs; calls within those limits then only
 * launch kernels.  Growing a region waits for the stream (once, here).
 * Errors: SENTRY_ERR_INVALID_ARG for a leaf size that is not a multiple of 64 or
 * more than 2^30 - 65 records; SENTRY_ERR_NOMEM / SENTRY_ERR_HIP.
 */
SENTRY_API int sentry_reserve_scratch(size_t merkle_max_len, size_t merkle_leaf_bytes,
                                      size_t lthash_max_records, void *stream);

/*
 * The memory the library holds for calls on `stream` of the current device: the
 * extra GPU memory of a hashing scheme (section 5.2, "Memory Usage Evaluation";
 * Table 1 reports it per scheme and model).  *out_device_bytes = bytes of the
 * stream's scratch regions (digests of the tree levels, tables, partial sums,
 * staging buffers of the host-streaming calls, gathered blocks of the coalesced
 * scheme), *out_pinned_bytes = pinned host memory of its table staging; either
 * may be NULL.  Both are grow-only until sentry_release_scratch: after a call
 * they are what the largest call so far on that stream needed.  Not counted:
 * the state a sentry_*_stream_begin call holds until its final or abort, and
 * the 2 MiB array of sentry_merkle_root_noalloc.  Host-side bookkeeping only:
 * no wait, no GPU work.
 * Errors: SENTRY_ERR_INVALID_ARG if both outputs are NULL; SENTRY_ERR_HIP.
 */
SENTRY_API int sentry_scratch_bytes(void *stream, size_t *out_device_bytes, size_t *out_pinned_bytes);

/* Free all cached scratch memory of the current device (synchronises it). */
SENTRY_API int sentry_release_scratch(void);

#ifdef __cplusplus
}
#endif
#endif /* SENTRY_H */

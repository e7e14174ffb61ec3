// What the translation units of the lattice hash share: the launches of the per-record root
// hashes (blake2_lthash.hip) and a few limits.  Host declarations only.
#pragma once

#include "sentry_internal.h"

namespace sentry {

// most data sources one per-source call takes
constexpr uint32_t LT_MAX_SOURCES = 4096;
// a launch holds fewer than 2^32 work-items in all, four lanes per record at most
constexpr uint64_t LT_MAX_RECORDS = 0xffffffffull / 4 - 64;

// First two words of the BLAKE2b parameter block of the per-record hash (the other words are zero):
// the BLAKE2Xb root hash of the 1024-lane digest (digest 64, fanout 1, depth 1, XOF length 2048), and
// the plain unkeyed BLAKE2b-512 whose 64-byte digest is the per-sample digest of section 4.2.2.
constexpr uint64_t LT_ROOT_P0 = 0x0000000001010040ull;
constexpr uint64_t LT_ROOT_P1 = (uint64_t)(2 * SENTRY_LANES) << 32;
constexpr uint64_t LT_PLAIN_P0 = 0x0000000001010040ull;
constexpr uint64_t LT_PLAIN_P1 = 0;

// 64-byte hashes of n records into h0 (device, 64 * n bytes): records at dev_records with offsets
// relative to offset_base, or (the _fixed form) records of record_bytes bytes each, back to back.
int lthash_roots(const void *dev_records, const uint64_t *dev_offsets, uint64_t offset_base, uint64_t n, uint64_t *h0,
                 hipStream_t s, uint64_t p0 = LT_ROOT_P0, uint64_t p1 = LT_ROOT_P1);
int lthash_roots_fixed(const void *dev_records, uint64_t record_bytes, uint64_t n, uint64_t *h0, hipStream_t s,
                       uint64_t p0 = LT_ROOT_P0, uint64_t p1 = LT_ROOT_P1);

// compute units of the current device (cached)
int lthash_cu_count();

}  // namespace sentry

"""MI355X-native hashing of ML artifacts resident in GPU memory (Sentry, CCS '25):
a SHA-256 Merkle tree over weight bytes and a BLAKE2Xb lattice hash over dataset
samples.  All work happens in ``libsentry_hip.so`` (hand-written HIP for gfx950,
C ABI in ``include/sentry.h``); this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    LANES, HASH_SHA256, HASH_BLAKE2B, HASH_SHA3_256, SentryError, lib_path, load,
    OK, MISMATCH, ERR_INVALID_ARG, ERR_HIP, ERR_NOMEM,
    sentry_merkle_root, sentry_merkle_root_noalloc, sentry_merkle_root_h, sentry_merkle_segments, sentry_merkle_inplace, sentry_merkle_segments_h, sentry_merkle_inplace_h, sentry_merkle_coalesced, sentry_merkle_coalesced_h, sentry_merkle_coalesced_plan,
    sentry_merkle_leaves, sentry_merkle_reduce,
    sentry_merkle_stream_begin, sentry_merkle_stream_update, sentry_merkle_stream_update_h2d, sentry_merkle_stream_final,
    sentry_merkle_stream_abort, sentry_merkle_root_h2d, sentry_verify,
    sentry_lthash, sentry_lthash_digests, sentry_lthash_sum, sentry_lthash_sources, sentry_lthash_model, sentry_lthash_model_from, sentry_lthash_combine, sentry_lthash_remove, sentry_lthash32, sentry_lthash_fixed, sentry_lthash32_fixed, sentry_lthash32_sources, sentry_lthash32_combine, sentry_lthash32_remove, sentry_lthash_h2d,
    sentry_lthash_stream_begin, sentry_lthash32_stream_begin, sentry_lthash_stream_update_h2d, sentry_lthash_stream_final, sentry_lthash_stream_abort,
    sentry_last_error, sentry_reserve_scratch, sentry_scratch_bytes, sentry_release_scratch,
)

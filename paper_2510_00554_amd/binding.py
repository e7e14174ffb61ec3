"""ctypes binding of ``libsentry_hip.so``: same names as the C ABI, argument marshalling
only.  Pointers are passed as integers (``tensor.data_ptr()``), streams as the integer
``torch.cuda.Stream.cuda_stream`` (0 = default stream).  Nothing here computes: if the
library is missing the import of any entry point fails loudly; there is no fallback.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LANES = 1024
_LIB_NAME = "libsentry_hip.so"

OK, MISMATCH, ERR_INVALID_ARG, ERR_HIP, ERR_NOMEM = 0, 1, -1, -2, -3


class SentryError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("sentry error %d: %s" % (code, text))
        self.code = code


def lib_path():
    return os.path.join(HERE, _LIB_NAME)


_lib = None

# name -> (restype, argtypes); the single source for ctypes prototypes and for the
# "every declared symbol is exported" test
_vp, _sz, _int = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
PROTOTYPES = {
    "sentry_merkle_root": (_int, [_vp, _sz, _sz, _vp, _vp]),
    "sentry_merkle_root_noalloc": (_int, [_vp, _sz, _sz, _vp, _vp]),
    "sentry_merkle_root_h": (_int, [_int, _vp, _sz, _sz, _vp, _vp]),
    "sentry_merkle_segments": (_int, [_vp, _vp, _sz, _sz, _vp, _vp, _vp]),
    "sentry_merkle_inplace": (_int, [_vp, _vp, _sz, _sz, _vp, _vp]),
    "sentry_merkle_segments_h": (_int, [_int, _vp, _vp, _sz, _sz, _vp, _vp, _vp]),
    "sentry_merkle_inplace_h": (_int, [_int, _vp, _vp, _sz, _sz, _vp, _vp]),
    "sentry_merkle_coalesced": (_int, [_vp, _vp, _sz, _sz, _vp, _sz, _vp, _vp]),
    "sentry_merkle_coalesced_plan": (_int, [_vp, _vp, _sz, _sz, _vp, _vp, _vp]),
    "sentry_merkle_coalesced_h": (_int, [_int, _vp, _vp, _sz, _sz, _vp, _sz, _vp, _vp]),
    "sentry_merkle_leaves": (_int, [_vp, _sz, _sz, _vp, _vp]),
    "sentry_merkle_reduce": (_int, [_vp, _sz, _vp, _vp]),
    "sentry_merkle_stream_begin": (_int, [_sz, _sz, ctypes.POINTER(_vp)]),
    "sentry_merkle_stream_update": (_int, [_vp, _vp, _sz, _vp]),
    "sentry_merkle_stream_update_h2d": (_int, [_vp, _vp, _sz, _vp]),
    "sentry_merkle_stream_final": (_int, [_vp, _vp, _vp]),
    "sentry_merkle_stream_abort": (_int, [_vp]),
    "sentry_merkle_root_h2d": (_int, [_vp, _sz, _sz, _sz, _vp, _vp]),
    "sentry_verify": (_int, [ctypes.c_char_p, ctypes.c_char_p]),
    "sentry_lthash": (_int, [_vp, _vp, _sz, _vp, _vp]),
    "sentry_lthash_digests": (_int, [_vp, _vp, _sz, _vp, _vp]),
    "sentry_lthash_sum": (_int, [_vp, _sz, _vp, _vp]),
    "sentry_lthash_sources": (_int, [_vp, _vp, _vp, _sz, _sz, _vp, _vp]),
    "sentry_lthash_model": (_int, [_vp, _vp, _sz, _sz, _vp, _vp, _vp]),
    "sentry_lthash_model_from": (_int, [_vp, _vp, _sz, _sz, ctypes.c_uint64, _vp, _vp, _vp]),
    "sentry_lthash_combine": (_int, [_vp, _vp, _vp]),
    "sentry_lthash_remove": (_int, [_vp, _vp, _vp]),
    "sentry_lthash32": (_int, [_vp, _vp, _sz, _vp, _vp]),
    "sentry_lthash_fixed": (_int, [_vp, _sz, _sz, _vp, _vp]),
    "sentry_lthash32_fixed": (_int, [_vp, _sz, _sz, _vp, _vp]),
    "sentry_lthash32_sources": (_int, [_vp, _vp, _vp, _sz, _sz, _vp, _vp]),
    "sentry_lthash32_combine": (_int, [_vp, _vp, _vp]),
    "sentry_lthash32_remove": (_int, [_vp, _vp, _vp]),
    "sentry_lthash_h2d": (_int, [_vp, _vp, _sz, _sz, _vp, _vp]),
    "sentry_lthash_stream_begin": (_int, [ctypes.POINTER(_vp)]),
    "sentry_lthash32_stream_begin": (_int, [ctypes.POINTER(_vp)]),
    "sentry_lthash_stream_update_h2d": (_int, [_vp, _vp, _vp, _sz, _vp]),
    "sentry_lthash_stream_final": (_int, [_vp, _vp, _vp]),
    "sentry_lthash_stream_abort": (_int, [_vp]),
    "sentry_last_error": (ctypes.c_char_p, []),
    "sentry_reserve_scratch": (_int, [_sz, _sz, _sz, _vp]),
    "sentry_scratch_bytes": (_int, [_vp, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]),
    "sentry_release_scratch": (_int, []),
}


def load():
    """Load the built library (build it with ``python -m paper_2510_00554_amd.build``)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            # nothing built yet: build once (hipcc, gfx950); there is no CPU fallback
            try:
                from . import build as _build
                _build.build()
            except Exception as e:
                raise ImportError("%s is not built and building it failed (%s); run "
                                  "`python -m paper_2510_00554_amd.build`" % (path, e))
        L = ctypes.CDLL(path)
        for name, (res, args) in PROTOTYPES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(rc):
    if rc < 0:
        raise SentryError(rc, sentry_last_error())
    return rc


def sentry_last_error():
    return load().sentry_last_error().decode("utf-8", "replace")


def sentry_reserve_scratch(merkle_max_len, merkle_leaf_bytes, lthash_max_records, stream=0):
    return _check(load().sentry_reserve_scratch(merkle_max_len, merkle_leaf_bytes, lthash_max_records, stream))


def sentry_scratch_bytes(stream=0):
    """(device bytes, pinned host bytes) the library holds for `stream`."""
    d, h = _sz(0), _sz(0)
    _check(load().sentry_scratch_bytes(stream, ctypes.byref(d), ctypes.byref(h)))
    return d.value, h.value


def sentry_release_scratch():
    return _check(load().sentry_release_scratch())


def sentry_merkle_root(dev_buf, length, leaf_bytes, out_digest, stream=0):
    return _check(load().sentry_merkle_root(dev_buf, length, leaf_bytes, out_digest, stream))


def sentry_merkle_root_noalloc(dev_buf, length, leaf_bytes, out_digest, stream=0):
    return _check(load().sentry_merkle_root_noalloc(dev_buf, length, leaf_bytes, out_digest, stream))


HASH_SHA256, HASH_BLAKE2B, HASH_SHA3_256 = 0, 1, 2


def sentry_merkle_root_h(hash_id, dev_buf, length, leaf_bytes, out_digest, stream=0):
    return _check(load().sentry_merkle_root_h(hash_id, dev_buf, length, leaf_bytes, out_digest, stream))


def sentry_merkle_segments(dev_ptrs, lens, leaf_bytes, out_seg_roots, out_root, stream=0):
    """dev_ptrs, lens: Python sequences of ints (device addresses, byte lengths)."""
    n = len(dev_ptrs)
    if len(lens) != n:
        raise ValueError("dev_ptrs and lens differ in length")
    ptrs = (ctypes.c_void_p * max(n, 1))(*dev_ptrs)
    ls = (ctypes.c_size_t * max(n, 1))(*lens)
    return _check(load().sentry_merkle_segments(ptrs, ls, n, leaf_bytes, out_seg_roots, out_root, stream))


def sentry_merkle_inplace(dev_ptrs, lens, leaf_bytes, out_root, stream=0):
    """dev_ptrs, lens: Python sequences of ints (device addresses, byte lengths)."""
    n = len(dev_ptrs)
    if len(lens) != n:
        raise ValueError("dev_ptrs and lens differ in length")
    ptrs = (ctypes.c_void_p * max(n, 1))(*dev_ptrs)
    ls = (ctypes.c_size_t * max(n, 1))(*lens)
    return _check(load().sentry_merkle_inplace(ptrs, ls, n, leaf_bytes, out_root, stream))


def _segment_arrays(dev_ptrs, lens):
    n = len(dev_ptrs)
    if len(lens) != n:
        raise ValueError("dev_ptrs and lens differ in length")
    return (ctypes.c_void_p * max(n, 1))(*dev_ptrs), (ctypes.c_size_t * max(n, 1))(*lens), n


def sentry_merkle_segments_h(hash_id, dev_ptrs, lens, leaf_bytes, out_seg_roots, out_root, stream=0):
    """dev_ptrs, lens: Python sequences of ints (device addresses, byte lengths)."""
    ptrs, ls, n = _segment_arrays(dev_ptrs, lens)
    return _check(load().sentry_merkle_segments_h(hash_id, ptrs, ls, n, leaf_bytes, out_seg_roots, out_root, stream))


def sentry_merkle_inplace_h(hash_id, dev_ptrs, lens, leaf_bytes, out_root, stream=0):
    """dev_ptrs, lens: Python sequences of ints (device addresses, byte lengths)."""
    ptrs, ls, n = _segment_arrays(dev_ptrs, lens)
    return _check(load().sentry_merkle_inplace_h(hash_id, ptrs, ls, n, leaf_bytes, out_root, stream))


def sentry_merkle_coalesced(dev_ptrs, lens, leaf_bytes, dev_buffer, buffer_bytes, out_root, stream=0):
    """dev_ptrs, lens: Python sequences of ints; dev_buffer 0 = no coalesced copy is made."""
    ptrs, ls, n = _segment_arrays(dev_ptrs, lens)
    return _check(load().sentry_merkle_coalesced(ptrs, ls, n, leaf_bytes, dev_buffer, buffer_bytes, out_root, stream))


def sentry_merkle_coalesced_plan(dev_ptrs, lens, leaf_bytes):
    """(gathered bytes, copied bytes, runs) of the call without a buffer; no GPU work."""
    ptrs, ls, n = _segment_arrays(dev_ptrs, lens)
    g, c, r = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(load().sentry_merkle_coalesced_plan(ptrs, ls, n, leaf_bytes, ctypes.byref(g), ctypes.byref(c), ctypes.byref(r)))
    return g.value, c.value, r.value


def sentry_merkle_coalesced_h(hash_id, dev_ptrs, lens, leaf_bytes, dev_buffer, buffer_bytes, out_root, stream=0):
    ptrs, ls, n = _segment_arrays(dev_ptrs, lens)
    return _check(load().sentry_merkle_coalesced_h(hash_id, ptrs, ls, n, leaf_bytes, dev_buffer, buffer_bytes, out_root,
                                                   stream))


def sentry_merkle_leaves(dev_buf, length, leaf_bytes, out_leaf_digests, stream=0):
    return _check(load().sentry_merkle_leaves(dev_buf, length, leaf_bytes, out_leaf_digests, stream))


def sentry_merkle_reduce(dev_nodes, n, out_digest, stream=0):
    return _check(load().sentry_merkle_reduce(dev_nodes, n, out_digest, stream))


def sentry_merkle_stream_begin(total_len, leaf_bytes):
    state = ctypes.c_void_p()
    _check(load().sentry_merkle_stream_begin(total_len, leaf_bytes, ctypes.byref(state)))
    return state


def sentry_merkle_stream_update(state, dev_chunk, length, stream=0):
    return _check(load().sentry_merkle_stream_update(state, dev_chunk, length, stream))


def sentry_merkle_stream_update_h2d(state, host_chunk, length, stream=0):
    return _check(load().sentry_merkle_stream_update_h2d(state, host_chunk, length, stream))


def sentry_merkle_stream_final(state, out_digest, stream=0):
    return _check(load().sentry_merkle_stream_final(state, out_digest, stream))


def sentry_merkle_stream_abort(state):
    return _check(load().sentry_merkle_stream_abort(state))


def sentry_merkle_root_h2d(host_buf, length, leaf_bytes, chunk_bytes, out_digest, stream=0):
    return _check(load().sentry_merkle_root_h2d(host_buf, length, leaf_bytes, chunk_bytes, out_digest, stream))


def sentry_verify(root, expected):
    """root, expected: 32-byte ``bytes``.  Returns 0 (equal) or 1 (mismatch)."""
    if root is not None and len(root) != 32 or expected is not None and len(expected) != 32:
        raise ValueError("digests are 32 bytes")
    return _check(load().sentry_verify(root, expected))


def sentry_lthash(dev_records, dev_offsets, n, out_lanes, stream=0):
    return _check(load().sentry_lthash(dev_records, dev_offsets, n, out_lanes, stream))


def sentry_lthash_digests(dev_records, dev_offsets, n, out_digests, stream=0):
    return _check(load().sentry_lthash_digests(dev_records, dev_offsets, n, out_digests, stream))


def sentry_lthash_sum(dev_digests, n, out_lanes, stream=0):
    return _check(load().sentry_lthash_sum(dev_digests, n, out_lanes, stream))


def sentry_lthash_sources(dev_records, dev_offsets, dev_source_ids, n, n_sources, acc_lanes, stream=0):
    return _check(load().sentry_lthash_sources(dev_records, dev_offsets, dev_source_ids, n, n_sources,
                                               acc_lanes, stream))


def sentry_lthash_model(dev_ptrs, lens, block_bytes, out_layer_lanes, out_lanes, stream=0):
    """dev_ptrs, lens: Python sequences of ints (device addresses, byte lengths)."""
    n = len(dev_ptrs)
    if len(lens) != n:
        raise ValueError("dev_ptrs and lens differ in length")
    ptrs = (ctypes.c_void_p * max(n, 1))(*dev_ptrs)
    ls = (ctypes.c_size_t * max(n, 1))(*lens)
    return _check(load().sentry_lthash_model(ptrs, ls, n, block_bytes, out_layer_lanes, out_lanes, stream))


def sentry_lthash_model_from(dev_ptrs, lens, block_bytes, first_index, out_layer_lanes, out_lanes, stream=0):
    ptrs, ls, n = _segment_arrays(dev_ptrs, lens)
    return _check(load().sentry_lthash_model_from(ptrs, ls, n, block_bytes, first_index, out_layer_lanes, out_lanes, stream))


def sentry_lthash_combine(acc, x, stream=0):
    return _check(load().sentry_lthash_combine(acc, x, stream))


def sentry_lthash_remove(acc, x, stream=0):
    return _check(load().sentry_lthash_remove(acc, x, stream))


def sentry_lthash32(dev_records, dev_offsets, n, out_lanes, stream=0):
    return _check(load().sentry_lthash32(dev_records, dev_offsets, n, out_lanes, stream))


def sentry_lthash_fixed(dev_records, record_bytes, n, out_lanes, stream=0):
    return _check(load().sentry_lthash_fixed(dev_records, record_bytes, n, out_lanes, stream))


def sentry_lthash32_fixed(dev_records, record_bytes, n, out_lanes, stream=0):
    return _check(load().sentry_lthash32_fixed(dev_records, record_bytes, n, out_lanes, stream))


def sentry_lthash32_sources(dev_records, dev_offsets, dev_source_ids, n, n_sources, acc_lanes, stream=0):
    return _check(load().sentry_lthash32_sources(dev_records, dev_offsets, dev_source_ids, n, n_sources, acc_lanes, stream))


def sentry_lthash32_combine(acc, x, stream=0):
    return _check(load().sentry_lthash32_combine(acc, x, stream))


def sentry_lthash32_remove(acc, x, stream=0):
    return _check(load().sentry_lthash32_remove(acc, x, stream))


def sentry_lthash_h2d(host_records, host_offsets, n, batch_bytes, out_lanes, stream=0):
    return _check(load().sentry_lthash_h2d(host_records, host_offsets, n, batch_bytes, out_lanes, stream))


def sentry_lthash_stream_begin():
    state = ctypes.c_void_p()
    _check(load().sentry_lthash_stream_begin(ctypes.byref(state)))
    return state


def sentry_lthash32_stream_begin():
    state = ctypes.c_void_p()
    _check(load().sentry_lthash32_stream_begin(ctypes.byref(state)))
    return state


def sentry_lthash_stream_update_h2d(state, host_records, host_offsets, n, stream=0):
    return _check(load().sentry_lthash_stream_update_h2d(state, host_records, host_offsets, n, stream))


def sentry_lthash_stream_final(state, out_lanes, stream=0):
    return _check(load().sentry_lthash_stream_final(state, out_lanes, stream))


def sentry_lthash_stream_abort(state):
    return _check(load().sentry_lthash_stream_abort(state))

"""ctypes loader for the CPU oracle (``sentry_oracle.c``): TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The GPU library and its Python binding
never do.  The wrappers below only marshal numpy arrays into the C functions;
every piece of arithmetic is in the C file.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sentry_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
LANES = 1024


def build(force=False):
    """Compile the oracle with gcc (plain C99, -O2, no threads)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp.%d" % os.getpid()
    subprocess.run(["gcc", "-std=gnu99", "-O2", "-fPIC", "-shared", "-o", tmp, _SRC],
                   check=True)
    os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = _bind(ctypes.CDLL(build()))
    return _lib


def _bind(L):
    """Set the prototypes of every oracle function on a loaded library."""
    if True:
        vp, sz, u32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint32
        L.oracle_sha256.argtypes = [vp, sz, vp]
        L.oracle_sha256.restype = None
        L.oracle_sha256_constants.argtypes = [vp, vp]
        L.oracle_sha256_constants.restype = None
        L.oracle_merkle_reduce.argtypes = [vp, sz, vp]
        L.oracle_merkle_reduce.restype = None
        L.oracle_merkle_leaves.argtypes = [vp, sz, sz, vp]
        L.oracle_merkle_leaves.restype = sz
        L.oracle_merkle_root.argtypes = [vp, sz, sz, vp]
        L.oracle_merkle_root.restype = ctypes.c_int
        L.oracle_merkle_segments.argtypes = [vp, vp, sz, sz, vp, vp]
        L.oracle_merkle_segments.restype = ctypes.c_int
        L.oracle_merkle_inplace.argtypes = [vp, vp, sz, sz, vp]
        L.oracle_merkle_inplace.restype = ctypes.c_int
        L.oracle_sha3_256.argtypes = [vp, sz, vp]
        L.oracle_sha3_256.restype = None
        L.oracle_keccak_constants.argtypes = [vp, vp]
        L.oracle_keccak_constants.restype = None
        L.oracle_merkle_root_h.argtypes = [ctypes.c_int, vp, sz, sz, vp]
        L.oracle_merkle_root_h.restype = ctypes.c_int
        L.oracle_merkle_segments_h.argtypes = [ctypes.c_int, vp, vp, sz, sz, vp, vp]
        L.oracle_merkle_segments_h.restype = ctypes.c_int
        L.oracle_merkle_inplace_h.argtypes = [ctypes.c_int, vp, vp, sz, sz, vp]
        L.oracle_merkle_inplace_h.restype = ctypes.c_int
        L.oracle_merkle_coalesced_h.argtypes = [ctypes.c_int, vp, vp, sz, sz, vp]
        L.oracle_merkle_coalesced_h.restype = ctypes.c_int
        L.oracle_verify.argtypes = [vp, vp]
        L.oracle_verify.restype = ctypes.c_int
        L.oracle_blake2b_constants.argtypes = [vp, vp]
        L.oracle_blake2b_constants.restype = None
        L.oracle_blake2b_param.argtypes = [vp, vp, sz, vp, sz]
        L.oracle_blake2b_param.restype = None
        L.oracle_blake2xb_root.argtypes = [vp, sz, u32, vp]
        L.oracle_blake2xb_root.restype = None
        L.oracle_blake2xb.argtypes = [vp, sz, vp, u32]
        L.oracle_blake2xb.restype = None
        L.oracle_lthash_one.argtypes = [vp, sz, vp]
        L.oracle_lthash_one.restype = None
        L.oracle_lthash.argtypes = [vp, vp, sz, vp]
        L.oracle_lthash.restype = None
        L.oracle_lthash_digests.argtypes = [vp, vp, sz, vp]
        L.oracle_lthash_digests.restype = None
        L.oracle_lthash_sum.argtypes = [vp, sz, vp]
        L.oracle_lthash_sum.restype = None
        L.oracle_lthash_sources.argtypes = [vp, vp, vp, sz, sz, vp]
        L.oracle_lthash_sources.restype = None
        L.oracle_lthash_model.argtypes = [vp, vp, sz, sz, vp, vp]
        L.oracle_lthash_model.restype = None
        L.oracle_lthash_model_from.argtypes = [vp, vp, sz, sz, ctypes.c_uint64, vp, vp]
        L.oracle_lthash_model_from.restype = None
        L.oracle_lanes_add.argtypes = [vp, vp, sz]
        L.oracle_lanes_add.restype = None
        L.oracle_lanes_sub.argtypes = [vp, vp, sz]
        L.oracle_lanes_sub.restype = None
        L.oracle_lthash32.argtypes = [vp, vp, sz, vp]
        L.oracle_lthash32.restype = None
        L.oracle_lthash32_sources.argtypes = [vp, vp, vp, sz, sz, vp]
        L.oracle_lthash32_sources.restype = None
        L.oracle_lthash_combine.argtypes = [vp, vp]
        L.oracle_lthash_combine.restype = None
        L.oracle_lthash_remove.argtypes = [vp, vp]
        L.oracle_lthash_remove.restype = None
    return L


class use_library:
    """Context manager for tests of the pins themselves: inside it every wrapper of this module
    calls the library at `path` (a build of an edited copy of sentry_oracle.c) instead."""

    def __init__(self, path):
        self.path = path

    def __enter__(self):
        global _lib
        lib()
        self.saved = _lib
        _lib = _bind(ctypes.CDLL(self.path))
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = self.saved
        return False


def _u8(data):
    """Contiguous uint8 view of bytes / bytearray / ndarray (no arithmetic)."""
    if isinstance(data, np.ndarray):
        a = np.ascontiguousarray(data)
        return a.view(np.uint8).reshape(-1)
    return np.frombuffer(bytes(data), dtype=np.uint8)


def _ptr(a):
    return a.ctypes.data if a.size else None


def sha256(data):
    a = _u8(data)
    out = np.empty(32, np.uint8)
    lib().oracle_sha256(_ptr(a), a.size, out.ctypes.data)
    return out.tobytes()


def sha256_constants():
    k = np.empty(64, np.uint32)
    h0 = np.empty(8, np.uint32)
    lib().oracle_sha256_constants(k.ctypes.data, h0.ctypes.data)
    return k, h0


def merkle_leaves(data, leaf_bytes):
    a = _u8(data)
    n = max(1, -(-a.size // leaf_bytes))
    out = np.empty((n, 32), np.uint8)
    got = lib().oracle_merkle_leaves(_ptr(a), a.size, leaf_bytes, out.ctypes.data)
    assert got == n
    return out


def merkle_reduce(nodes):
    a = np.array(nodes, dtype=np.uint8, copy=True).reshape(-1, 32)   # reduced in place
    out = np.empty(32, np.uint8)
    lib().oracle_merkle_reduce(a.ctypes.data, a.shape[0], out.ctypes.data)
    return out.tobytes()


def merkle_root(data, leaf_bytes):
    a = _u8(data)
    out = np.empty(32, np.uint8)
    rc = lib().oracle_merkle_root(_ptr(a), a.size, leaf_bytes, out.ctypes.data)
    if rc:
        raise ValueError("oracle_merkle_root rc=%d" % rc)
    return out.tobytes()


def merkle_segments(segments, leaf_bytes):
    """segments: list of byte-like; returns (list of per-segment roots, global root)."""
    arrs = [_u8(s) for s in segments]
    n = len(arrs)
    ptrs = (ctypes.c_void_p * n)(*[_ptr(a) for a in arrs])
    lens = (ctypes.c_size_t * n)(*[a.size for a in arrs])
    seg = np.empty((max(n, 1), 32), np.uint8)
    out = np.empty(32, np.uint8)
    rc = lib().oracle_merkle_segments(ptrs, lens, n, leaf_bytes, seg.ctypes.data, out.ctypes.data)
    if rc:
        raise ValueError("oracle_merkle_segments rc=%d" % rc)
    return [seg[i].tobytes() for i in range(n)], out.tobytes()


def merkle_inplace(segments, leaf_bytes):
    """One flat tree over the blocks of all segments (Algorithm 3); returns the root."""
    arrs = [_u8(s) for s in segments]
    n = len(arrs)
    ptrs = (ctypes.c_void_p * max(n, 1))(*[_ptr(a) for a in arrs])
    lens = (ctypes.c_size_t * max(n, 1))(*[a.size for a in arrs])
    out = np.empty(32, np.uint8)
    rc = lib().oracle_merkle_inplace(ptrs, lens, n, leaf_bytes, out.ctypes.data)
    if rc:
        raise ValueError("oracle_merkle_inplace rc=%d" % rc)
    return out.tobytes()


HASH_SHA256, HASH_BLAKE2B, HASH_SHA3_256 = 0, 1, 2


def sha3_256(data):
    a = _u8(data)
    out = np.empty(32, np.uint8)
    lib().oracle_sha3_256(_ptr(a), a.size, out.ctypes.data)
    return out.tobytes()


def keccak_constants():
    rc = np.empty(24, np.uint64)
    rho = np.empty(25, np.int32)
    lib().oracle_keccak_constants(rc.ctypes.data, rho.ctypes.data)
    return rc, rho


def merkle_root_h(hash_id, data, leaf_bytes):
    a = _u8(data)
    out = np.empty(64, np.uint8)
    dl = lib().oracle_merkle_root_h(hash_id, _ptr(a), a.size, leaf_bytes, out.ctypes.data)
    if dl < 0:
        raise ValueError("oracle_merkle_root_h rc=%d" % dl)
    return out[:dl].tobytes()


def merkle_segments_h(hash_id, segments, leaf_bytes):
    """Algorithm 2 under hash ``hash_id``: (list of per-segment roots, root over them)."""
    arrs = [_u8(s) for s in segments]
    n = len(arrs)
    ptrs = (ctypes.c_void_p * max(n, 1))(*[_ptr(a) for a in arrs])
    lens = (ctypes.c_size_t * max(n, 1))(*[a.size for a in arrs])
    seg = np.empty((max(n, 1), 64), np.uint8)
    out = np.empty(64, np.uint8)
    dl = lib().oracle_merkle_segments_h(hash_id, ptrs, lens, n, leaf_bytes, seg.ctypes.data, out.ctypes.data)
    if dl < 0:
        raise ValueError("oracle_merkle_segments_h rc=%d" % dl)
    flat = seg.reshape(-1)
    return [flat[dl * i:dl * (i + 1)].tobytes() for i in range(n)], out[:dl].tobytes()


def merkle_inplace_h(hash_id, segments, leaf_bytes):
    """Algorithm 3 under hash ``hash_id``: the root of the flat tree over all segments' blocks."""
    arrs = [_u8(s) for s in segments]
    n = len(arrs)
    ptrs = (ctypes.c_void_p * max(n, 1))(*[_ptr(a) for a in arrs])
    lens = (ctypes.c_size_t * max(n, 1))(*[a.size for a in arrs])
    out = np.empty(64, np.uint8)
    dl = lib().oracle_merkle_inplace_h(hash_id, ptrs, lens, n, leaf_bytes, out.ctypes.data)
    if dl < 0:
        raise ValueError("oracle_merkle_inplace_h rc=%d" % dl)
    return out[:dl].tobytes()


def merkle_coalesced_h(hash_id, segments, leaf_bytes):
    """Algorithm 1 under hash ``hash_id``: the root of the tree over the zero-padded concatenation."""
    arrs = [_u8(s) for s in segments]
    n = len(arrs)
    ptrs = (ctypes.c_void_p * max(n, 1))(*[_ptr(a) for a in arrs])
    lens = (ctypes.c_size_t * max(n, 1))(*[a.size for a in arrs])
    out = np.empty(64, np.uint8)
    dl = lib().oracle_merkle_coalesced_h(hash_id, ptrs, lens, n, leaf_bytes, out.ctypes.data)
    if dl < 0:
        raise ValueError("oracle_merkle_coalesced_h rc=%d" % dl)
    return out[:dl].tobytes()


def verify(a, b):
    x, y = _u8(a), _u8(b)
    assert x.size == 32 and y.size == 32
    return lib().oracle_verify(x.ctypes.data, y.ctypes.data)


def blake2b_constants():
    iv = np.empty(8, np.uint64)
    sigma = np.empty(160, np.uint8)
    lib().oracle_blake2b_constants(iv.ctypes.data, sigma.ctypes.data)
    return iv, sigma.reshape(10, 16)


def blake2b_param(param, data, out_len=64):
    p = _u8(param)
    assert p.size == 64
    a = _u8(data)
    out = np.empty(out_len, np.uint8)
    lib().oracle_blake2b_param(p.ctypes.data, _ptr(a), a.size, out.ctypes.data, out_len)
    return out.tobytes()


def blake2xb_root(data, xof_len=2048):
    a = _u8(data)
    out = np.empty(64, np.uint8)
    lib().oracle_blake2xb_root(_ptr(a), a.size, xof_len, out.ctypes.data)
    return out.tobytes()


def blake2xb(data, xof_len=2048):
    a = _u8(data)
    out = np.empty(xof_len, np.uint8)
    lib().oracle_blake2xb(_ptr(a), a.size, out.ctypes.data, xof_len)
    return out.tobytes()


def lthash_one(data):
    a = _u8(data)
    out = np.empty(LANES, np.uint16)
    lib().oracle_lthash_one(_ptr(a), a.size, out.ctypes.data)
    return out


def lthash(records, offsets):
    """records: byte-like; offsets: n+1 uint64 byte offsets into records."""
    a = _u8(records)
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    n = max(off.size - 1, 0)
    out = np.full(LANES, 0xAAAA, np.uint16)      # the C function must overwrite every lane
    if n:
        assert int(off[-1]) <= a.size
    lib().oracle_lthash(_ptr(a), _ptr(off), n, out.ctypes.data)
    return out


def lthash_digests(records, offsets):
    """The digest of every record: n x 1024 uint16."""
    a = _u8(records)
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    n = max(off.size - 1, 0)
    out = np.full((n, LANES), 0xAAAA, np.uint16)
    if n:
        assert int(off[-1]) <= a.size
        lib().oracle_lthash_digests(_ptr(a), _ptr(off), n, out.ctypes.data)
    return out


def lthash_sum(digests):
    """Lane-wise sum mod 2^16 of n digests (n x 1024 uint16) that are already computed."""
    d = np.ascontiguousarray(digests, dtype=np.uint16).reshape(-1, LANES)
    out = np.full(LANES, 0xAAAA, np.uint16)
    lib().oracle_lthash_sum(d.ctypes.data if d.size else None, d.shape[0], out.ctypes.data)
    return out


def lthash_sources(records, offsets, sources, n_sources, acc=None):
    """Per-source running sums: returns acc (n_sources x 1024 uint16) updated with this batch."""
    a = _u8(records)
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    src = np.ascontiguousarray(sources, dtype=np.uint32)
    n = max(off.size - 1, 0)
    assert src.size == n
    out = np.zeros((n_sources, LANES), np.uint16) if acc is None else np.array(acc, dtype=np.uint16, copy=True)
    assert out.shape == (n_sources, LANES)
    lib().oracle_lthash_sources(_ptr(a), _ptr(off), _ptr(src), n, n_sources, out.ctypes.data)
    return out


def lanes_add(acc, x):
    r = np.array(acc, dtype=np.uint16, copy=True)
    xx = np.ascontiguousarray(x, dtype=np.uint16)
    assert r.shape == xx.shape
    lib().oracle_lanes_add(r.ctypes.data, xx.ctypes.data, r.size)
    return r


def lanes_sub(acc, x):
    r = np.array(acc, dtype=np.uint16, copy=True)
    xx = np.ascontiguousarray(x, dtype=np.uint16)
    assert r.shape == xx.shape
    lib().oracle_lanes_sub(r.ctypes.data, xx.ctypes.data, r.size)
    return r


def lthash32(records, offsets):
    """Dataset lattice hash at the paper's digest width: 32 uint16 partitions (section 4.2.2)."""
    rec = _u8(records)
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    n = max(off.size - 1, 0)
    out = np.full(32, 0xAAAA, np.uint16)          # the C function must overwrite every partition
    if n:
        assert int(off[-1]) <= rec.size
    lib().oracle_lthash32(_ptr(rec), _ptr(off), n, out.ctypes.data)
    return out


def lthash32_sources(records, offsets, sources, n_sources, acc=None):
    """Per-source running sums at the 32-partition width: acc (n_sources x 32 uint16) updated with this batch."""
    a = _u8(records)
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    src = np.ascontiguousarray(sources, dtype=np.uint32)
    n = max(off.size - 1, 0)
    assert src.size == n
    out = np.zeros((n_sources, 32), np.uint16) if acc is None else np.array(acc, dtype=np.uint16, copy=True)
    assert out.shape == (n_sources, 32)
    lib().oracle_lthash32_sources(_ptr(a), _ptr(off), _ptr(src), n, n_sources, out.ctypes.data)
    return out


def lthash_model(segments, block_bytes, first_index=0):
    """Model lattice hash (Algorithm 4): returns (per-layer lanes n_seg x 32, model lanes 32)."""
    arrs = [_u8(s) for s in segments]
    n = len(arrs)
    ptrs = (ctypes.c_void_p * max(n, 1))(*[_ptr(a) for a in arrs])
    lens = (ctypes.c_size_t * max(n, 1))(*[a.size for a in arrs])
    layer = np.zeros((max(n, 1), 32), np.uint16)
    total = np.zeros(32, np.uint16)
    lib().oracle_lthash_model_from(ptrs, lens, n, block_bytes, first_index, layer.ctypes.data, total.ctypes.data)
    return layer[:n], total


def lthash_combine(acc, x):
    r = np.array(acc, dtype=np.uint16, copy=True)
    xx = np.ascontiguousarray(x, dtype=np.uint16)
    lib().oracle_lthash_combine(r.ctypes.data, xx.ctypes.data)
    return r


def lthash_remove(acc, x):
    r = np.array(acc, dtype=np.uint16, copy=True)
    xx = np.ascontiguousarray(x, dtype=np.uint16)
    lib().oracle_lthash_remove(r.ctypes.data, xx.ctypes.data)
    return r

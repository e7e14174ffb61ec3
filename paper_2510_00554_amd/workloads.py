"""Seeded synthetic inputs with the shapes of the paper's workloads.

This module holds no hashing arithmetic.  It serves the GPU tests, ``bench.py`` and the
scripts that write golden values, so every generator exists twice with bit-identical
results: a numpy version (host, used with the CPU oracle) and a torch version (fills a
tensor on the GPU without a host copy).  Both are the same counter-based construction
in exact integer arithmetic, so a 138 GB checkpoint never has to exist in host memory to
be reproducible:

  word(seed, i)  = mix64(mix64(seed) + (i + 1) * GAMMA)        (the SplitMix64 sequence)
  uniform bytes  = the little-endian bytes of word(seed, 0), word(seed, 1), ...
  bf16 "normal"  = the sum of the four 16-bit fields of word(seed, i), centred, scaled to
                   standard deviation 0.02 in float32 (one exact multiply) and rounded to
                   bfloat16 (round to nearest even on the bit pattern).  The sum of four
                   uniforms is close to a Gaussian (bounded at 3.46 sigma); hashing cost
                   does not depend on the values.

Shapes stand in for the paper's artifacts: 32x32x3 uint8 images (section 5, "Datasets
and Models"), Llama-style checkpoints laid out tensor by tensor (a ``state_dict``,
section 4.2), variable-length records.
"""
import math

import numpy as np

GAMMA = 0x9E3779B97F4A7C15
M1 = 0xBF58476D1CE4E5B9
M2 = 0x94D049BB133111EB
MASK64 = (1 << 64) - 1
BASE_SEED = 20251000

_NP_BLOCK = 1 << 16   # words per numpy pass

# seeds of the five target configurations
SEED_C1 = BASE_SEED + 1          # 16 MiB of uniform bytes
SEED_C2 = BASE_SEED + 2          # 50,000 image-shaped samples
SEED_C3 = BASE_SEED + 3          # 7B checkpoint (per-tensor seeds derive from it)
SEED_C4_LEN = BASE_SEED + 4      # record lengths
SEED_C4_BYTES = BASE_SEED + 5    # record bytes: one uniform stream cut at record boundaries
SEED_C5 = BASE_SEED + 6          # 70B checkpoint
C4_RECORDS = 1_281_167
C4_BATCH_BYTES = 8_000_000_000

# float32 scale that maps the centred four-field sum to standard deviation 0.02
_SUM_STD = math.sqrt(4 * (65536.0 ** 2 - 1.0) / 12.0)
SCALE32 = float(np.float32(0.02 / _SUM_STD))


def _mix_int(z):
    z &= MASK64
    z = ((z ^ (z >> 30)) * M1) & MASK64
    z = ((z ^ (z >> 27)) * M2) & MASK64
    return z ^ (z >> 31)


def _signed(x):
    x &= MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


# ---------------------------------------------------------------------------
# numpy backend
# ---------------------------------------------------------------------------

def _words_np(seed, w0, w1):
    key = np.uint64(_mix_int(seed))
    with np.errstate(over="ignore"):
        z = (np.arange(w0 + 1, w1 + 1, dtype=np.uint64) * np.uint64(GAMMA)) + key
        z = (z ^ (z >> np.uint64(30))) * np.uint64(M1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(M2)
        z = z ^ (z >> np.uint64(31))
    return z


def _bf16_bits_np(words):
    s = ((words & np.uint64(0xFFFF)) + ((words >> np.uint64(16)) & np.uint64(0xFFFF))
         + ((words >> np.uint64(32)) & np.uint64(0xFFFF)) + (words >> np.uint64(48)))
    c = s.astype(np.int64) - 131070
    x = c.astype(np.float32) * np.float32(SCALE32)
    b = x.view(np.uint32).astype(np.uint64)
    r = (b + np.uint64(0x7FFF) + ((b >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    return r.astype(np.uint16)


# ---------------------------------------------------------------------------
# torch backend (any device)
# ---------------------------------------------------------------------------

def _lsr_t(z, k):
    import torch
    return torch.bitwise_and(torch.bitwise_right_shift(z, k), (1 << (64 - k)) - 1)


def _words_t(seed, w0, w1, device):
    import torch
    key = _signed(_mix_int(seed))
    z = torch.arange(w0 + 1, w1 + 1, dtype=torch.int64, device=device) * _signed(GAMMA) + key
    z = (z ^ _lsr_t(z, 30)) * _signed(M1)
    z = (z ^ _lsr_t(z, 27)) * _signed(M2)
    return z ^ _lsr_t(z, 31)


def _bf16_bits_t(words):
    import torch
    s = ((words & 0xFFFF) + (_lsr_t(words, 16) & 0xFFFF) + (_lsr_t(words, 32) & 0xFFFF) + _lsr_t(words, 48))
    x = (s - 131070).to(torch.float32) * SCALE32
    b = x.view(torch.int32).to(torch.int64) & 0xFFFFFFFF
    r = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16) & 0xFFFF
    return (((r + 0x8000) & 0xFFFF) - 0x8000).to(torch.int16)


# ---------------------------------------------------------------------------
# HIP backend: the same two generators as fill kernels (libsentry_workloads.so), used for
# CUDA tensors when the library is built; one launch per call instead of dozens of torch ops
# ---------------------------------------------------------------------------

_fill_lib = None


def _hip_fill():
    global _fill_lib
    if _fill_lib is None:
        import ctypes
        import os
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsentry_workloads.so")
        if not os.path.exists(path):
            _fill_lib = False
        else:
            L = ctypes.CDLL(path)
            u64, vp = ctypes.c_uint64, ctypes.c_void_p
            L.workloads_fill_uniform.argtypes = [vp, u64, u64, u64, vp]
            L.workloads_fill_uniform.restype = ctypes.c_int
            L.workloads_fill_normal_bf16.argtypes = [vp, u64, u64, u64, ctypes.c_float, vp]
            L.workloads_fill_normal_bf16.restype = ctypes.c_int
            _fill_lib = L
    return _fill_lib or None


def _is_cuda(device):
    return device is not None and str(device).startswith("cuda")


# ---------------------------------------------------------------------------
# public generators
# ---------------------------------------------------------------------------

def uniform_bytes(seed, start, nbytes, device=None, out=None, chunk=1 << 27, backend=None):
    """Bytes [start, start+nbytes) of the uniform stream `seed`.

    device None -> numpy uint8 array; otherwise a torch uint8 tensor on `device`
    (written into `out` if given, a 1-D uint8 tensor of nbytes elements)."""
    if device is None:
        # small blocks: the temporaries stay in cache and in the allocator's free lists
        w0, w1 = start // 8, -(-(start + nbytes) // 8)
        words = np.empty(w1 - w0, np.uint64)
        for p in range(w0, w1, _NP_BLOCK):
            q = min(p + _NP_BLOCK, w1)
            words[p - w0:q - w0] = _words_np(seed, p, q)
        b = words.view(np.uint8)
        return b[start - 8 * w0: start - 8 * w0 + nbytes].copy()
    import torch
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=device)
    if _is_cuda(device) and backend != "torch" and _hip_fill() is not None:
        rc = _hip_fill().workloads_fill_uniform(out.data_ptr(), _mix_int(seed), start, nbytes,
                                                torch.cuda.current_stream().cuda_stream)
        assert rc == 0
        return out
    pos = 0
    while pos < nbytes:
        n = min(chunk, nbytes - pos)
        s = start + pos
        w0, w1 = s // 8, -(-(s + n) // 8)
        b = _words_t(seed, w0, w1, device).view(torch.uint8)
        out[pos:pos + n] = b[s - 8 * w0: s - 8 * w0 + n]
        pos += n
    return out


def normal_bf16_bits(seed, start_elem, n, device=None, out=None, chunk=1 << 26, backend=None):
    """bf16 bit patterns of elements [start_elem, start_elem+n) of the weight stream `seed`.

    device None -> numpy uint16 array; otherwise a torch int16 tensor (same bits)."""
    if device is None:
        res = np.empty(n, np.uint16)
        for p in range(0, n, _NP_BLOCK):
            q = min(p + _NP_BLOCK, n)
            res[p:q] = _bf16_bits_np(_words_np(seed, start_elem + p, start_elem + q))
        return res
    import torch
    if out is None:
        out = torch.empty(n, dtype=torch.int16, device=device)
    if _is_cuda(device) and backend != "torch" and _hip_fill() is not None:
        rc = _hip_fill().workloads_fill_normal_bf16(out.data_ptr(), _mix_int(seed), start_elem, n, SCALE32,
                                                    torch.cuda.current_stream().cuda_stream)
        assert rc == 0
        return out
    pos = 0
    while pos < n:
        m = min(chunk, n - pos)
        out[pos:pos + m] = _bf16_bits_t(_words_t(seed, start_elem + pos, start_elem + pos + m, device))
        pos += m
    return out


# ---------------------------------------------------------------------------
# workload shapes
# ---------------------------------------------------------------------------

def llama_layout(layers, d, ffn, vocab, kv_dim=None):
    """(name, numel) of every tensor of a Llama-style checkpoint in state-dict order."""
    kv = d if kv_dim is None else kv_dim
    out = [("embed", vocab * d)]
    for i in range(layers):
        out += [("l%d.q" % i, d * d), ("l%d.k" % i, kv * d), ("l%d.v" % i, kv * d), ("l%d.o" % i, d * d),
                ("l%d.gate" % i, ffn * d), ("l%d.up" % i, ffn * d), ("l%d.down" % i, d * ffn),
                ("l%d.input_norm" % i, d), ("l%d.post_attn_norm" % i, d)]
    out += [("final_norm", d), ("lm_head", vocab * d)]
    return out


def layout_7b():
    """32 layers, d=4096, ffn=11008, vocab 32000: 291 tensors, 13,476,831,232 bytes in bf16."""
    return llama_layout(32, 4096, 11008, 32000)


def layout_70b():
    """80 layers, d=8192, ffn=28672, vocab 32000, 8 KV heads of 128: 723 tensors, 137,953,296,384 bytes."""
    return llama_layout(80, 8192, 28672, 32000, kv_dim=1024)


def layout_tiny():
    """A small model of the same structure for tests: 2 layers, d=256, ffn=704, vocab 1000."""
    return llama_layout(2, 256, 704, 1000, kv_dim=64)


def tensor_seed(base_seed, index):
    return base_seed + 1000 * (index + 1)


def checkpoint_tensor(layout, index, base_seed=BASE_SEED, device=None):
    """Tensor `index` of a checkpoint as bf16 bit patterns (numpy uint16 / torch int16)."""
    return normal_bf16_bits(tensor_seed(base_seed, index), 0, layout[index][1], device=device)


def checkpoint_bytes_np(layout, base_seed=BASE_SEED):
    """All tensors as a list of numpy uint8 arrays (small layouts only)."""
    return [checkpoint_tensor(layout, i, base_seed).view(np.uint8) for i in range(len(layout))]


def checkpoint_flat_torch(layout, device, base_seed=BASE_SEED):
    """The whole checkpoint as one uint8 tensor on `device`, tensors back to back, plus the
    byte offset of every tensor."""
    import torch
    offs = [0]
    for _, numel in layout:
        offs.append(offs[-1] + 2 * numel)
    buf = torch.empty(offs[-1], dtype=torch.uint8, device=device)
    as16 = buf.view(torch.int16)
    for i, (_, numel) in enumerate(layout):
        normal_bf16_bits(tensor_seed(base_seed, i), 0, numel, device=device,
                         out=as16[offs[i] // 2: offs[i] // 2 + numel])
    return buf, offs


def checkpoint_offsets(layout):
    offs = [0]
    for _, numel in layout:
        offs.append(offs[-1] + 2 * numel)
    return offs


def checkpoint_stream_np(layout, start, nbytes, base_seed=BASE_SEED, offs=None):
    """Bytes [start, start+nbytes) of the checkpoint laid out tensor by tensor (numpy uint8)."""
    import bisect
    offs = checkpoint_offsets(layout) if offs is None else offs
    out = np.empty(nbytes, np.uint8)
    pos = start
    end = start + nbytes
    i = bisect.bisect_right(offs, pos) - 1
    while pos < end:
        t_end = min(end, offs[i + 1])
        e0, e1 = (pos - offs[i]) // 2, -(-(t_end - offs[i]) // 2)
        piece = normal_bf16_bits(tensor_seed(base_seed, i), e0, e1 - e0).view(np.uint8)
        lo = (pos - offs[i]) - 2 * e0
        out[pos - start:t_end - start] = piece[lo:lo + (t_end - pos)]
        pos = t_end
        i += 1
    return out


def image_records(n, seed=SEED_C2, device=None):
    """n samples of 32x32x3 uint8 (3072 bytes each), packed; returns (bytes, offsets)."""
    data = uniform_bytes(seed, 0, 3072 * n, device=device)
    off = np.arange(n + 1, dtype=np.uint64) * np.uint64(3072)
    return data, off


def lognormal_record_lengths(n, seed=SEED_C4_LEN, median=110_000, sigma=0.5, lo=8_000, hi=1_000_000):
    """Record lengths in bytes: round(median * exp(sigma * z)) clipped to [lo, hi], z a
    12-uniform-sum standard normal drawn from the counter generator (host, float64)."""
    w = _words_np(seed, 0, 3 * n).reshape(n, 3)
    fields = np.stack([(w >> np.uint64(16 * k)) & np.uint64(0xFFFF) for k in range(4)], axis=-1)
    z = (fields.reshape(n, 12).astype(np.float64).sum(axis=1) - 6 * 65535.0) / math.sqrt(65536.0 ** 2 - 1.0)
    ln = np.rint(median * np.exp(sigma * z))
    return np.clip(ln, lo, hi).astype(np.uint64)


def dirichlet_source_ids(n, n_sources, seed, alpha_one=True):
    """Source id per sample for a dataset put together from n_sources providers whose shares
    are drawn from a Dirichlet distribution with concentration 1 (section 5.2, the run over 1 to
    128 sources): shares = normalised Exp(1) draws, every sample then picks its source by those
    shares.  Host, float64, from the counter generator; returns uint32[n]."""
    assert alpha_one
    w = _words_np(seed, 0, n_sources + n)
    u = ((w >> np.uint64(11)).astype(np.float64) + 1.0) / 9007199254740992.0          # (0, 1]
    e = -np.log(u[:n_sources])
    cdf = np.cumsum(e / e.sum())
    ids = np.searchsorted(cdf, u[n_sources:], side="left")
    return np.minimum(ids, n_sources - 1).astype(np.uint32)


def offsets_from_lengths(lengths):
    off = np.zeros(len(lengths) + 1, np.uint64)
    np.cumsum(lengths, out=off[1:])
    return off


def cut_batches(offsets, batch_bytes):
    """Record index ranges [(first, last_exclusive), ...] whose bytes fit batch_bytes each."""
    out, i, n = [], 0, len(offsets) - 1
    while i < n:
        j = int(np.searchsorted(offsets, offsets[i] + np.uint64(batch_bytes), side="right")) - 1
        j = min(max(j, i + 1), n)
        out.append((i, j))
        i = j
    return out

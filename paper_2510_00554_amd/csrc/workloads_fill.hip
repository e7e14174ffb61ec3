// Synthetic-input fill kernels (own shared library, libsentry_workloads.so): the GPU twin of
// the numpy generators in workloads.py, bit for bit.  Test and benchmark plumbing only: no
// hashing arithmetic lives here and the hashing library does not link to it.
//
//   word(key, i)  = mix64(key + (i + 1) * GAMMA)            (SplitMix64 sequence, key = mix64(seed))
//   uniform bytes = little-endian bytes of word(key, 0), word(key, 1), ...
//   bf16 element  = (sum of the four 16-bit fields of word(key, i) - 131070) * scale in float32
//                   (one IEEE multiply), rounded to bfloat16 by round-to-nearest-even on the bits
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ uint64_t word_at(uint64_t key, uint64_t i)
{
    return mix64(key + (i + 1) * 0x9E3779B97F4A7C15ull);
}

// out[0 .. n_words) = word(key, w0 + k); out is 8-byte aligned
__global__ void fill_words_kernel(uint64_t *out, uint64_t key, uint64_t w0, uint64_t n_words)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n_words; k += stride)
        out[k] = word_at(key, w0 + k);
}

// bytes [start, start + n) of the stream, for the unaligned head and tail of a range
__global__ void fill_bytes_kernel(uint8_t *out, uint64_t key, uint64_t start, uint64_t n)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += stride) {
        const uint64_t b = start + k;
        out[k] = (uint8_t)(word_at(key, b >> 3) >> (8 * (b & 7)));
    }
}

__device__ __forceinline__ uint32_t bf16_bits(uint64_t w, float scale)
{
    const int32_t s = (int32_t)((w & 0xFFFF) + ((w >> 16) & 0xFFFF) + ((w >> 32) & 0xFFFF) + (w >> 48)) - 131070;
    const float x = __fmul_rn((float)s, scale);
    const uint32_t b = __float_as_uint(x);
    return ((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16) & 0xFFFFu;
}

// out[k] = bf16 bits of element e0 + k; out is 2-byte aligned
__global__ void fill_bf16_kernel(uint16_t *out, uint64_t key, uint64_t e0, uint64_t n, float scale)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += stride)
        out[k] = (uint16_t)bf16_bits(word_at(key, e0 + k), scale);
}

uint32_t grid_for(uint64_t n)
{
    uint64_t g = (n + 255) / 256;
    return (uint32_t)(g > 65536 ? 65536 : (g ? g : 1));
}

}  // namespace

extern "C" {

// Fill dev_out[0 .. nbytes) with bytes [start, start + nbytes) of the uniform stream.
__attribute__((visibility("default")))
int workloads_fill_uniform(void *dev_out, uint64_t key, uint64_t start, uint64_t nbytes, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *out = static_cast<uint8_t *>(dev_out);
    if (nbytes == 0) return 0;
    // head up to the first position where both the stream offset and the address are 8-byte
    // aligned (possible only if they agree mod 8); otherwise everything goes byte by byte
    uint64_t head = (8 - (start & 7)) & 7;
    if (((reinterpret_cast<uintptr_t>(out) + head) & 7) != 0 || head > nbytes) head = nbytes;
    // a launch holds fewer than 2^32 work-items in all: every kernel here strides over its range
    if (head) hipLaunchKernelGGL(fill_bytes_kernel, dim3(grid_for(head)), dim3(256), 0, s, out, key, start, head);
    const uint64_t n_words = (nbytes - head) / 8;
    if (n_words)
        hipLaunchKernelGGL(fill_words_kernel, dim3(grid_for(n_words)), dim3(256), 0, s,
                           reinterpret_cast<uint64_t *>(out + head), key, (start + head) / 8, n_words);
    const uint64_t tail = nbytes - head - 8 * n_words;
    if (tail)
        hipLaunchKernelGGL(fill_bytes_kernel, dim3(1), dim3(256), 0, s, out + head + 8 * n_words, key,
                           start + head + 8 * n_words, tail);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

// Fill dev_out[0 .. n) (uint16) with the bf16 bit patterns of elements [e0, e0 + n).
__attribute__((visibility("default")))
int workloads_fill_normal_bf16(void *dev_out, uint64_t key, uint64_t e0, uint64_t n, float scale, void *stream)
{
    if (n == 0) return 0;
    hipLaunchKernelGGL(fill_bf16_kernel, dim3(grid_for(n)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint16_t *>(dev_out), key, e0, n, scale);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // extern "C"

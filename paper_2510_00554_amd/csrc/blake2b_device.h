// BLAKE2b (RFC 7693) compression for gfx950, shared by the lattice-hash translation units.
// Device code only; every function is inlined into the kernels that use it.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

// 64-bit values live in register pairs

// (as a vector cast, not shift-and-or: the compiler turns "x + (lo | hi << 32)" into two adds)
typedef uint32_t b2_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint64_t pack64(uint32_t lo, uint32_t hi)
{
    const b2_u32x2 v = {lo, hi};
    return __builtin_bit_cast(uint64_t, v);
}

// rotations as two 32-bit funnel shifts on the halves; by 32 it is a swap of the halves
__device__ __forceinline__ uint64_t rotr64_32(uint64_t x) { return pack64((uint32_t)(x >> 32), (uint32_t)x); }
template <int N>   // 0 < N < 32
__device__ __forceinline__ uint64_t rotr64_lt32(uint64_t x)
{
    const uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
    return pack64(__builtin_amdgcn_alignbit(hi, lo, N), __builtin_amdgcn_alignbit(lo, hi, N));
}
__device__ __forceinline__ uint64_t rotr64_63(uint64_t x)   // = rotate left by one
{
    const uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
    return pack64(__builtin_amdgcn_alignbit(lo, hi, 31), __builtin_amdgcn_alignbit(hi, lo, 31));
}

#define B2_G(a, b, c, d, x, y)                     \
    do {                                           \
        a = a + b + (x); d = rotr64_32(d ^ a);     \
        c = c + d;       b = rotr64_lt32<24>(b ^ c); \
        a = a + b + (y); d = rotr64_lt32<16>(d ^ a); \
        c = c + d;       b = rotr64_63(b ^ c);     \
    } while (0)

constexpr uint64_t b2_iv(int i)
{
    constexpr uint64_t iv[8] = {0x6a09e667f3bcc908ull, 0xbb67ae8584caa73bull, 0x3c6ef372fe94f82bull,
                                0xa54ff53a5f1d36f1ull, 0x510e527fade682d1ull, 0x9b05688c2b3e6c1full,
                                0x1f83d9abfb41bd6bull, 0x5be0cd19137e2179ull};
    return iv[i];
}

constexpr int b2_sigma(int r, int i)
{
    constexpr unsigned char S[10][16] = {
        {0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15}, {14, 10, 4, 8, 9, 15, 13, 6, 1, 12, 0, 2, 11, 7, 5, 3},
        {11, 8, 12, 0, 5, 2, 15, 13, 10, 14, 3, 6, 7, 1, 9, 4}, {7, 9, 3, 1, 13, 12, 11, 14, 2, 6, 5, 10, 4, 0, 15, 8},
        {9, 0, 5, 7, 2, 4, 10, 15, 14, 1, 11, 12, 6, 8, 3, 13}, {2, 12, 6, 10, 0, 11, 8, 3, 4, 13, 7, 5, 15, 14, 1, 9},
        {12, 5, 1, 15, 14, 13, 4, 10, 0, 7, 6, 3, 9, 2, 8, 11}, {13, 11, 7, 14, 12, 1, 3, 9, 5, 0, 15, 4, 8, 6, 2, 10},
        {6, 15, 14, 9, 11, 3, 0, 8, 12, 2, 13, 7, 1, 4, 10, 5}, {10, 2, 8, 4, 7, 6, 1, 5, 15, 11, 9, 14, 3, 12, 13, 0}};
    return S[r % 10][i];
}

// h <- F(h, m, t, last): twelve rounds, fully unrolled so that the message permutation
// becomes static register indexing.  t = message bytes so far (below 2^64).
__device__ __forceinline__ void blake2b_compress(uint64_t (&h)[8], const uint64_t (&m)[16], uint64_t t, bool last)
{
    uint64_t v[16];
#pragma unroll
    for (int i = 0; i < 8; i++) { v[i] = h[i]; v[8 + i] = b2_iv(i); }
    v[12] ^= t;
    if (last) v[14] = ~v[14];
#pragma unroll
    for (int r = 0; r < 12; r++) {
        B2_G(v[0], v[4], v[8], v[12], m[b2_sigma(r, 0)], m[b2_sigma(r, 1)]);
        B2_G(v[1], v[5], v[9], v[13], m[b2_sigma(r, 2)], m[b2_sigma(r, 3)]);
        B2_G(v[2], v[6], v[10], v[14], m[b2_sigma(r, 4)], m[b2_sigma(r, 5)]);
        B2_G(v[3], v[7], v[11], v[15], m[b2_sigma(r, 6)], m[b2_sigma(r, 7)]);
        B2_G(v[0], v[5], v[10], v[15], m[b2_sigma(r, 8)], m[b2_sigma(r, 9)]);
        B2_G(v[1], v[6], v[11], v[12], m[b2_sigma(r, 10)], m[b2_sigma(r, 11)]);
        B2_G(v[2], v[7], v[8], v[13], m[b2_sigma(r, 12)], m[b2_sigma(r, 13)]);
        B2_G(v[3], v[4], v[9], v[14], m[b2_sigma(r, 14)], m[b2_sigma(r, 15)]);
    }
#pragma unroll
    for (int i = 0; i < 8; i++) h[i] ^= v[i] ^ v[8 + i];
}

}  // namespace

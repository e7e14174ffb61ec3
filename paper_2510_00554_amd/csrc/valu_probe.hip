// Issue-rate probe for the VALU opcodes the hash kernels are made of (own shared library,
// libsentry_probe.so): measurement plumbing of bench.py, not part of the hashing library.
//
// The integer-ALU roofline of a hash kernel is "instructions of its mix over the rate at which
// the chip can issue them", and on gfx950 that rate is not one number: some opcodes issue at
// about twice the rate of others once a SIMD holds several waves.  Each probe launch runs one
// opcode (or one short mix) as four independent register chains per lane, 65,536 instructions
// per wave, on `waves_per_simd` waves for every SIMD of the chip, and reports lane-operations per
// second from HIP-event time plus the shader clock seen by the waves.  The kernels touch no
// memory except one result word per lane and two counters per workgroup.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <vector>

namespace {

constexpr int ITER = 1024;      // loop trips
constexpr int UNROLL = 16;      // groups of four instructions per trip
constexpr int WG = 256;         // four waves: one per SIMD of a CU

// The same with the registers named: a three-source instruction reads its operands from the four
// VGPR banks (register number mod 4), and how fast it issues depends on whether they collide.  The
// chains live in v40..v43, the other operands in v44..v51; the values do not matter for the timing.
#define FIXED(text) asm volatile(text ::: "v40", "v41", "v42", "v43", "v44", "v45", "v46", "v47", "v48", "v49", "v50", "v51")

// four independent chains a, b, c, d; e, f are read-only vector operands, sk a scalar one
#define OP32(text) asm volatile(text : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "v"(e), "v"(f), "s"(sk))
#define OP64(text) asm volatile(text : "+v"(a64), "+v"(b64), "+v"(c64), "+v"(d64) : "v"(e64))

enum Op {
    OP_ADD = 0, OP_SUB, OP_XOR, OP_AND, OP_OR, OP_LSHR, OP_LSHL, OP_MOV, OP_BITOP3, OP_ADD_LITERAL,
    OP_ADD3, OP_ALIGNBIT, OP_PERM, OP_LSHL_ADD_U64, OP_PK_ADD_U16, OP_BFI, OP_ADD_SGPR, OP_ADD3_SGPR,
    OP_MOV_DPP, OP_XOR_DPP, OP_CNDMASK, OP_MIX_SHA, OP_MIX_BLAKE2B, OP_MIX_KECCAK,
    OP_BITOP3_BANKS3, OP_BITOP3_BANKS1, OP_ADD3_BANKS3, OP_MIX_SHA_BANKS3, OP_COUNT
};

const char *const OP_NAME[OP_COUNT] = {
    "v_add_u32", "v_sub_u32", "v_xor_b32", "v_and_b32", "v_or_b32", "v_lshrrev_b32", "v_lshlrev_b32", "v_mov_b32",
    "v_bitop3_b32", "v_add_u32 (literal)", "v_add3_u32", "v_alignbit_b32", "v_perm_b32", "v_lshl_add_u64",
    "v_pk_add_u16", "v_bfi_b32", "v_add_u32 (sgpr)", "v_add3_u32 (sgpr)", "v_mov_b32_dpp quad_perm",
    "v_xor_b32_dpp quad_perm", "v_cndmask_b32", "mix: sha-256 block (per 16: 7 alignbit, 4 bitop3, 3 add3, 1 add, 1 lshr)",
    "mix: blake2b G (per 16: 6 xor, 5 alignbit, 5 lshl_add_u64)", "mix: keccak round (per 16: 6 bitop3, 5 xor, 5 alignbit)",
    "v_bitop3_b32, sources in three register banks", "v_bitop3_b32, sources in one register bank",
    "v_add3_u32, sources in three register banks", "mix: sha-256 block, three-source ops read three register banks"};

template <int OP>
__global__ void __launch_bounds__(WG) probe_kernel(uint32_t *out, uint64_t *clocks, uint32_t seed, uint32_t sk)
{
    uint32_t a = threadIdx.x + seed, b = a * 3 + 1, c = a ^ 0x55, d = a + 7, e = a * 5 + 3, f = a * 7 + 1;
    uint64_t a64 = ((uint64_t)a << 32) | b, b64 = ((uint64_t)c << 32) | d, c64 = a64 ^ 0x1234567ull, d64 = b64 + 99, e64 = ((uint64_t)e << 32) | f;
    const uint64_t t0 = clock64(), w0 = wall_clock64();
#pragma unroll 1
    for (int i = 0; i < ITER; i++) {
#pragma unroll
        for (int k = 0; k < UNROLL; k++) {
            if (OP == OP_ADD) OP32("v_add_u32 %0, %0, %4\n v_add_u32 %1, %1, %4\n v_add_u32 %2, %2, %4\n v_add_u32 %3, %3, %4");
            if (OP == OP_SUB) OP32("v_sub_u32 %0, %0, %4\n v_sub_u32 %1, %1, %4\n v_sub_u32 %2, %2, %4\n v_sub_u32 %3, %3, %4");
            if (OP == OP_XOR) OP32("v_xor_b32 %0, %0, %4\n v_xor_b32 %1, %1, %4\n v_xor_b32 %2, %2, %4\n v_xor_b32 %3, %3, %4");
            if (OP == OP_AND) OP32("v_and_b32 %0, %0, %4\n v_and_b32 %1, %1, %4\n v_and_b32 %2, %2, %4\n v_and_b32 %3, %3, %4");
            if (OP == OP_OR) OP32("v_or_b32 %0, %0, %4\n v_or_b32 %1, %1, %4\n v_or_b32 %2, %2, %4\n v_or_b32 %3, %3, %4");
            if (OP == OP_LSHR) OP32("v_lshrrev_b32 %0, 3, %0\n v_lshrrev_b32 %1, 3, %1\n v_lshrrev_b32 %2, 3, %2\n v_lshrrev_b32 %3, 3, %3");
            if (OP == OP_LSHL) OP32("v_lshlrev_b32 %0, 3, %0\n v_lshlrev_b32 %1, 3, %1\n v_lshlrev_b32 %2, 3, %2\n v_lshlrev_b32 %3, 3, %3");
            if (OP == OP_MOV) OP32("v_mov_b32 %0, %1\n v_mov_b32 %1, %2\n v_mov_b32 %2, %3\n v_mov_b32 %3, %4");
            if (OP == OP_BITOP3) OP32("v_bitop3_b32 %0, %0, %4, %5 bitop3:0x96\n v_bitop3_b32 %1, %1, %4, %5 bitop3:0x96\n v_bitop3_b32 %2, %2, %4, %5 bitop3:0x96\n v_bitop3_b32 %3, %3, %4, %5 bitop3:0x96");
            if (OP == OP_ADD_LITERAL) OP32("v_add_u32 %0, 0x428a2f98, %0\n v_add_u32 %1, 0x428a2f98, %1\n v_add_u32 %2, 0x428a2f98, %2\n v_add_u32 %3, 0x428a2f98, %3");
            if (OP == OP_ADD3) OP32("v_add3_u32 %0, %0, %4, %5\n v_add3_u32 %1, %1, %4, %5\n v_add3_u32 %2, %2, %4, %5\n v_add3_u32 %3, %3, %4, %5");
            if (OP == OP_ALIGNBIT) OP32("v_alignbit_b32 %0, %0, %0, 7\n v_alignbit_b32 %1, %1, %1, 7\n v_alignbit_b32 %2, %2, %2, 7\n v_alignbit_b32 %3, %3, %3, 7");
            if (OP == OP_PERM) OP32("v_perm_b32 %0, %0, %4, %5\n v_perm_b32 %1, %1, %4, %5\n v_perm_b32 %2, %2, %4, %5\n v_perm_b32 %3, %3, %4, %5");
            if (OP == OP_LSHL_ADD_U64) OP64("v_lshl_add_u64 %0, %0, 0, %4\n v_lshl_add_u64 %1, %1, 0, %4\n v_lshl_add_u64 %2, %2, 0, %4\n v_lshl_add_u64 %3, %3, 0, %4");
            if (OP == OP_PK_ADD_U16) OP32("v_pk_add_u16 %0, %0, %4\n v_pk_add_u16 %1, %1, %4\n v_pk_add_u16 %2, %2, %4\n v_pk_add_u16 %3, %3, %4");
            if (OP == OP_BFI) OP32("v_bfi_b32 %0, %0, %4, %5\n v_bfi_b32 %1, %1, %4, %5\n v_bfi_b32 %2, %2, %4, %5\n v_bfi_b32 %3, %3, %4, %5");
            if (OP == OP_ADD_SGPR) OP32("v_add_u32 %0, %0, %6\n v_add_u32 %1, %1, %6\n v_add_u32 %2, %2, %6\n v_add_u32 %3, %3, %6");
            if (OP == OP_ADD3_SGPR) OP32("v_add3_u32 %0, %0, %4, %6\n v_add3_u32 %1, %1, %4, %6\n v_add3_u32 %2, %2, %4, %6\n v_add3_u32 %3, %3, %4, %6");
            if (OP == OP_MOV_DPP) OP32("v_mov_b32_dpp %0, %1 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf\n v_mov_b32_dpp %1, %2 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf\n v_mov_b32_dpp %2, %3 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf\n v_mov_b32_dpp %3, %4 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf");
            if (OP == OP_XOR_DPP) OP32("v_xor_b32_dpp %0, %4, %0 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf\n v_xor_b32_dpp %1, %4, %1 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf\n v_xor_b32_dpp %2, %4, %2 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf\n v_xor_b32_dpp %3, %4, %3 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf");
            if (OP == OP_CNDMASK) OP32("v_cndmask_b32 %0, %0, %4, vcc\n v_cndmask_b32 %1, %1, %4, vcc\n v_cndmask_b32 %2, %2, %4, vcc\n v_cndmask_b32 %3, %3, %4, vcc");
            // Mixes in the proportions of the hash kernels' hot loops, four instructions per group and
            // a period of four groups, so that a trip of sixteen groups holds four periods.
            if (OP == OP_MIX_SHA) {   // of 16: 7 alignbit, 4 bitop3, 3 add3, 1 add, 1 lshr (the block mix is 576:352:240:120:96 of 1384)
                if ((k & 3) == 0) OP32("v_alignbit_b32 %0, %0, %0, 7\n v_bitop3_b32 %1, %1, %4, %5 bitop3:0x96\n v_alignbit_b32 %2, %2, %2, 13\n v_add3_u32 %3, %3, %4, %5");
                if ((k & 3) == 1) OP32("v_alignbit_b32 %0, %0, %0, 7\n v_bitop3_b32 %1, %1, %4, %5 bitop3:0xca\n v_alignbit_b32 %2, %2, %2, 13\n v_add3_u32 %3, %3, %4, %5");
                if ((k & 3) == 2) OP32("v_alignbit_b32 %0, %0, %0, 7\n v_bitop3_b32 %1, %1, %4, %5 bitop3:0xe8\n v_alignbit_b32 %2, %2, %2, 13\n v_add3_u32 %3, %3, %4, %5");
                if ((k & 3) == 3) OP32("v_alignbit_b32 %0, %0, %0, 7\n v_bitop3_b32 %1, %1, %4, %5 bitop3:0x96\n v_lshrrev_b32 %2, 3, %2\n v_add_u32 %3, %3, %4");
            }
            if (OP == OP_MIX_BLAKE2B) {   // of 16: 6 xor, 5 alignbit, 5 lshl_add_u64 (the compression mix is 800:576:576 of 1952)
                if ((k & 3) == 0) asm volatile("v_xor_b32 %0, %0, %4\n v_alignbit_b32 %1, %1, %0, 24\n v_lshl_add_u64 %2, %2, 0, %5\n v_xor_b32 %3, %3, %4" : "+v"(a), "+v"(b), "+v"(c64), "+v"(d) : "v"(e), "v"(e64));
                if ((k & 3) == 1) asm volatile("v_xor_b32 %0, %0, %4\n v_alignbit_b32 %1, %1, %0, 16\n v_lshl_add_u64 %2, %2, 0, %5\n v_alignbit_b32 %3, %3, %0, 31" : "+v"(a), "+v"(b), "+v"(c64), "+v"(d) : "v"(e), "v"(e64));
                if ((k & 3) == 2) asm volatile("v_xor_b32 %0, %0, %4\n v_alignbit_b32 %1, %1, %0, 24\n v_lshl_add_u64 %2, %2, 0, %5\n v_xor_b32 %3, %3, %4" : "+v"(a), "+v"(b), "+v"(c64), "+v"(d) : "v"(e), "v"(e64));
                if ((k & 3) == 3) asm volatile("v_xor_b32 %0, %0, %4\n v_alignbit_b32 %1, %1, %0, 16\n v_lshl_add_u64 %2, %2, 0, %5\n v_lshl_add_u64 %3, %3, 0, %5" : "+v"(a), "+v"(b), "+v"(c64), "+v"(d64) : "v"(e), "v"(e64));
            }
            if (OP == OP_BITOP3_BANKS3) FIXED("v_bitop3_b32 v40, v40, v45, v46 bitop3:0x96\n v_bitop3_b32 v41, v41, v46, v47 bitop3:0x96\n v_bitop3_b32 v42, v42, v47, v44 bitop3:0x96\n v_bitop3_b32 v43, v43, v44, v45 bitop3:0x96");
            if (OP == OP_BITOP3_BANKS1) FIXED("v_bitop3_b32 v40, v40, v44, v48 bitop3:0x96\n v_bitop3_b32 v41, v41, v45, v49 bitop3:0x96\n v_bitop3_b32 v42, v42, v46, v50 bitop3:0x96\n v_bitop3_b32 v43, v43, v47, v51 bitop3:0x96");
            if (OP == OP_ADD3_BANKS3) FIXED("v_add3_u32 v40, v40, v45, v46\n v_add3_u32 v41, v41, v46, v47\n v_add3_u32 v42, v42, v47, v44\n v_add3_u32 v43, v43, v44, v45");
            if (OP == OP_MIX_SHA_BANKS3) {
                if ((k & 3) != 3) FIXED("v_alignbit_b32 v40, v40, v40, 7\n v_bitop3_b32 v41, v41, v46, v47 bitop3:0x96\n v_alignbit_b32 v42, v42, v42, 13\n v_add3_u32 v43, v43, v44, v45");
                if ((k & 3) == 3) FIXED("v_alignbit_b32 v40, v40, v40, 7\n v_bitop3_b32 v41, v41, v46, v47 bitop3:0x96\n v_lshrrev_b32 v42, 3, v42\n v_add_u32 v43, v43, v44");
            }
            if (OP == OP_MIX_KECCAK) {   // of 16: 6 bitop3, 5 xor, 5 alignbit (the round mix is 70:62:58 of 190)
                if ((k & 3) == 0) OP32("v_bitop3_b32 %0, %0, %4, %5 bitop3:0x96\n v_xor_b32 %1, %1, %4\n v_alignbit_b32 %2, %2, %2, 7\n v_bitop3_b32 %3, %3, %4, %5 bitop3:0xd2");
                if ((k & 3) == 1) OP32("v_bitop3_b32 %0, %0, %4, %5 bitop3:0x96\n v_xor_b32 %1, %1, %4\n v_alignbit_b32 %2, %2, %2, 7\n v_xor_b32 %3, %3, %4");
                if ((k & 3) == 2) OP32("v_bitop3_b32 %0, %0, %4, %5 bitop3:0x96\n v_xor_b32 %1, %1, %4\n v_alignbit_b32 %2, %2, %2, 7\n v_bitop3_b32 %3, %3, %4, %5 bitop3:0xd2");
                if ((k & 3) == 3) OP32("v_bitop3_b32 %0, %0, %4, %5 bitop3:0x96\n v_xor_b32 %1, %1, %4\n v_alignbit_b32 %2, %2, %2, 7\n v_alignbit_b32 %3, %3, %3, 13");
            }
        }
    }
    const uint64_t t1 = clock64(), w1 = wall_clock64();
    out[blockIdx.x * WG + threadIdx.x] = a ^ b ^ c ^ d ^ (uint32_t)(a64 ^ b64 ^ c64 ^ d64) ^ (uint32_t)((a64 ^ b64 ^ c64 ^ d64) >> 32);
    if (threadIdx.x == 0) {
        clocks[2 * blockIdx.x] = t1 - t0;
        clocks[2 * blockIdx.x + 1] = w1 - w0;
    }
}

template <int OP>
hipError_t launch(int grid, uint32_t *out, uint64_t *clocks, uint32_t seed, hipStream_t s)
{
    hipLaunchKernelGGL(probe_kernel<OP>, dim3(grid), dim3(WG), 0, s, out, clocks, seed, 12345u);
    return hipGetLastError();
}

template <int OP>
hipError_t dispatch(int op, int grid, uint32_t *out, uint64_t *clocks, uint32_t seed, hipStream_t s)
{
    if (op == OP) return launch<OP>(grid, out, clocks, seed, s);
    if constexpr (OP + 1 < OP_COUNT) return dispatch<OP + 1>(op, grid, out, clocks, seed, s);
    return hipErrorInvalidValue;
}

}  // namespace

extern "C" {

__attribute__((visibility("default"))) int sentry_probe_op_count(void) { return OP_COUNT; }

__attribute__((visibility("default"))) const char *sentry_probe_op_name(int op)
{
    return (op >= 0 && op < OP_COUNT) ? OP_NAME[op] : "";
}

// One opcode at `waves_per_simd` (1 .. 8) waves on every SIMD of the current device.
//   tera_lane_ops  lane-operations per second / 1e12 (instructions x 64 lanes over HIP-event time)
//   sclk_mhz       shader clock seen by the waves (cycle counter over the 100 MHz wall counter)
//   clk_per_instr  cycles between two instructions of one wave
// Returns 0, or a hipError_t value.
__attribute__((visibility("default"))) int sentry_probe_valu(int op, int waves_per_simd, double *tera_lane_ops,
                                                             double *sclk_mhz, double *clk_per_instr)
{
    if (op < 0 || op >= OP_COUNT || waves_per_simd < 1 || waves_per_simd > 8) return (int)hipErrorInvalidValue;
    int dev = 0, cus = 0;
    hipError_t e;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return (int)e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return (int)e;
    const int grid = cus * waves_per_simd;
    uint32_t *out = nullptr;
    uint64_t *clocks = nullptr;
    if ((e = hipMalloc(&out, (size_t)grid * WG * 4)) != hipSuccess) return (int)e;
    if ((e = hipMalloc(&clocks, (size_t)grid * 16)) != hipSuccess) { (void)hipFree(out); return (int)e; }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    float ms = 0;
    std::vector<uint64_t> h(2 * (size_t)grid);
    do {
        if ((e = hipEventCreate(&e0)) != hipSuccess) break;
        if ((e = hipEventCreate(&e1)) != hipSuccess) break;
        if ((e = dispatch<0>(op, grid, out, clocks, 1, nullptr)) != hipSuccess) break;   // warm-up
        if ((e = hipDeviceSynchronize()) != hipSuccess) break;
        if ((e = hipEventRecord(e0, nullptr)) != hipSuccess) break;
        if ((e = dispatch<0>(op, grid, out, clocks, 2, nullptr)) != hipSuccess) break;
        if ((e = hipEventRecord(e1, nullptr)) != hipSuccess) break;
        if ((e = hipEventSynchronize(e1)) != hipSuccess) break;
        if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) break;
        e = hipMemcpy(h.data(), clocks, 16 * (size_t)grid, hipMemcpyDeviceToHost);
    } while (0);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(out);
    (void)hipFree(clocks);
    if (e != hipSuccess) return (int)e;
    double cyc = 0, wall = 0;
    for (int i = 0; i < grid; i++) { cyc += (double)h[2 * i]; wall += (double)h[2 * i + 1]; }
    const double instr_per_wave = (double)ITER * UNROLL * 4;
    const double lane_ops = instr_per_wave * 64.0 * grid * (WG / 64);
    *tera_lane_ops = lane_ops / (ms * 1e-3) / 1e12;
    *sclk_mhz = wall > 0 ? cyc / wall * 100.0 : 0.0;
    *clk_per_instr = cyc / grid / instr_per_wave;
    return 0;
}

}  // extern "C"

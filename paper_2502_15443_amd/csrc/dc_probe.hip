// Device side of libdc_mi355x: how fast the vector ALU issues single instructions (dc_issue_rate).  A measuring
// tool for the figures that say how close the decode kernels are to the instruction issue of the chip; not part
// of the method.  One kernel per instruction: a chain of 32 copies of it per loop turn on values that stay in
// registers, eight wavefronts resident on every SIMD, so that what is timed is the rate at which a SIMD issues
// the instruction, not its latency.
#include <hip/hip_runtime.h>

#include "dc.h"

namespace {

#define DC_REP4(x) x x x x
#define DC_REP32(x) DC_REP4(DC_REP4(x)) DC_REP4(DC_REP4(x))

// operands: %0 a, %1 d, %2 q (64 bits), %3 f, %4 b, %5 c (1..8), %6 g
#define DC_PROBE_KERNEL(NAME, ASM)                                                                          \
    __global__ __launch_bounds__(256) void NAME(uint32_t *sink, uint32_t seed, uint32_t turns)              \
    {                                                                                                       \
        uint32_t a = seed + threadIdx.x, b = seed * 3 + 1, c = (threadIdx.x & 7) + 1, d = a ^ 0x5555u;      \
        uint64_t q = ((uint64_t)a << 32) | b;                                                               \
        float f = (float)a, g = 1.0001f;                                                                    \
        for (uint32_t i = 0; i < turns; i++) {                                                              \
            DC_REP32(asm volatile(ASM : "+v"(a), "+v"(d), "+v"(q), "+v"(f) : "v"(b), "v"(c), "v"(g) : "vcc");) \
        }                                                                                                   \
        if (blockIdx.x == 0) sink[threadIdx.x] = a + d + (uint32_t)q + (uint32_t)(q >> 32) + (uint32_t)f;   \
    }

DC_PROBE_KERNEL(probe_and, "v_and_b32 %0, %0, %4")
DC_PROBE_KERNEL(probe_or, "v_or_b32 %0, %0, %4")
DC_PROBE_KERNEL(probe_xor, "v_xor_b32 %0, %0, %4")
DC_PROBE_KERNEL(probe_add, "v_add_u32 %0, %0, %4")
DC_PROBE_KERNEL(probe_sub, "v_sub_u32 %0, %0, %4")
DC_PROBE_KERNEL(probe_lshr, "v_lshrrev_b32 %0, %5, %0")
DC_PROBE_KERNEL(probe_lshl, "v_lshlrev_b32 %0, %5, %0")
DC_PROBE_KERNEL(probe_mov, "v_mov_b32 %0, %1")
DC_PROBE_KERNEL(probe_min, "v_min_u32 %0, %0, %4")
DC_PROBE_KERNEL(probe_alignbit, "v_alignbit_b32 %0, %1, %0, %5")
DC_PROBE_KERNEL(probe_bfe, "v_bfe_u32 %0, %0, %5, 11")
DC_PROBE_KERNEL(probe_perm, "v_perm_b32 %0, %0, %1, %4")
DC_PROBE_KERNEL(probe_add3, "v_add3_u32 %0, %0, %4, %5")
DC_PROBE_KERNEL(probe_lshl_add, "v_lshl_add_u32 %0, %0, 1, %4")
DC_PROBE_KERNEL(probe_and_or, "v_and_or_b32 %0, %0, %4, %5")
DC_PROBE_KERNEL(probe_lshl_or, "v_lshl_or_b32 %0, %0, 1, %4")
DC_PROBE_KERNEL(probe_mul_u24, "v_mul_u32_u24 %0, %0, %4")
DC_PROBE_KERNEL(probe_mad_u24, "v_mad_u32_u24 %0, %0, %4, %5")
DC_PROBE_KERNEL(probe_lshr_b64, "v_lshrrev_b64 %2, %5, %2")
DC_PROBE_KERNEL(probe_lshl_b64, "v_lshlrev_b64 %2, %5, %2")
DC_PROBE_KERNEL(probe_sub_sdwa, "v_sub_u32_sdwa %0, %0, %4 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0")
DC_PROBE_KERNEL(probe_cmp, "v_cmp_lt_u32 vcc, %0, %4")
DC_PROBE_KERNEL(probe_mbcnt, "v_mbcnt_lo_u32_b32 %0, %4, %0")
DC_PROBE_KERNEL(probe_mov_dpp, "v_mov_b32_dpp %0, %1 row_shr:1 row_mask:0xf bank_mask:0xf")
DC_PROBE_KERNEL(probe_mul_f32, "v_mul_f32 %3, %3, %6")
DC_PROBE_KERNEL(probe_add_f32, "v_add_f32 %3, %3, %6")
DC_PROBE_KERNEL(probe_fma_f32, "v_fma_f32 %3, %3, %6, %6")
DC_PROBE_KERNEL(probe_cvt_f32_i32, "v_cvt_f32_i32 %3, %0")
DC_PROBE_KERNEL(probe_cvt_pk_bf16, "v_cvt_pk_bf16_f32 %0, %3, %6")
DC_PROBE_KERNEL(probe_cvt_sdwa, "v_cvt_f32_i32_sdwa %3, sext(%0) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1")
DC_PROBE_KERNEL(probe_cvt_ubyte, "v_cvt_f32_ubyte1 %3, %0")
DC_PROBE_KERNEL(probe_dot2_bf16, "v_dot2_f32_bf16 %3, %0, %4, %3")
DC_PROBE_KERNEL(probe_dot2c_bf16, "v_dot2c_f32_bf16 %3, %0, %4")
DC_PROBE_KERNEL(probe_cmp_cndmask, "v_cmp_lt_u32 vcc, %1, %4\n\tv_cndmask_b32 %0, %0, %4, vcc")
DC_PROBE_KERNEL(probe_max, "v_max_u32 %0, %0, %4")
DC_PROBE_KERNEL(probe_bfi, "v_bfi_b32 %0, %4, %0, %1")
DC_PROBE_KERNEL(probe_lshr_b16, "v_lshrrev_b16 %0, %5, %0")
DC_PROBE_KERNEL(probe_add_u16, "v_add_u16 %0, %0, %4")

// LDS reads: every wavefront reads a 4 KiB table (the size of the decode table) at addresses of a given pattern,
// 32 reads a loop turn, the address of each read made to depend on the one before (by a value that is always 0).
//   PATTERN 0: every lane the same address; 1: lane l reads 16-bit entry l (two lanes a dword); 2: dword l;
//   3: dword 2 l; 4: dword 32 l mod 1024 (one bank if there are 32); 5: dword 64 l mod 1024; 6: a different
//   pseudo-random 11-bit entry per lane and read (what a table look-up of the decoder is)
template <int PATTERN, bool HALFWORD> __global__ __launch_bounds__(256) void probe_lds(uint32_t *sink, uint32_t seed, uint32_t turns)
{
    __shared__ uint32_t table[1024];
    for (uint32_t i = threadIdx.x; i < 1024; i += 256) table[i] = 0;
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t byte = PATTERN == 0 ? 64u : PATTERN == 1 ? 2 * lane : PATTERN == 2 ? 4 * lane : PATTERN == 3 ? 8 * lane
                  : PATTERN == 4 ? (128 * lane) & 4095u : PATTERN == 5 ? (256 * lane) & 4095u : 0u;
    uint32_t state = (seed + threadIdx.x + 1) * 2654435761u, sum = 0;
    const uint32_t base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)table;
    for (uint32_t i = 0; i < turns; i++) {
#pragma unroll
        for (int j = 0; j < 32; j++) {
            if (PATTERN == 6) {
                state = state * 1664525u + 1013904223u;
                byte = (state >> 20) & 0xFFEu;
            }
            uint32_t v;
            if (HALFWORD) v = *(const __attribute__((address_space(3))) uint16_t *)(uintptr_t)(base + (byte & ~1u) + sum);
            else v = *(const __attribute__((address_space(3))) uint32_t *)(uintptr_t)(base + (byte & ~3u) + sum);
            sum += v; // always 0: the next address waits for this read
        }
    }
    if (blockIdx.x == 0) sink[threadIdx.x] = sum + state;
}

typedef void (*probe_kernel)(uint32_t *, uint32_t, uint32_t);
struct Probe {
    const char *name;
    probe_kernel kernel;
};
const Probe kProbes[] = {
    {"v_and_b32", probe_and},           {"v_or_b32", probe_or},           {"v_xor_b32", probe_xor},
    {"v_add_u32", probe_add},           {"v_sub_u32", probe_sub},         {"v_lshrrev_b32", probe_lshr},
    {"v_lshlrev_b32", probe_lshl},      {"v_mov_b32", probe_mov},         {"v_min_u32", probe_min},
    {"v_alignbit_b32", probe_alignbit}, {"v_bfe_u32", probe_bfe},         {"v_perm_b32", probe_perm},
    {"v_add3_u32", probe_add3},         {"v_lshl_add_u32", probe_lshl_add}, {"v_and_or_b32", probe_and_or},
    {"v_lshl_or_b32", probe_lshl_or},   {"v_mul_u32_u24", probe_mul_u24}, {"v_mad_u32_u24", probe_mad_u24},
    {"v_lshrrev_b64", probe_lshr_b64},  {"v_lshlrev_b64", probe_lshl_b64}, {"v_sub_u32_sdwa", probe_sub_sdwa},
    {"v_cmp_lt_u32", probe_cmp},        {"v_mbcnt_lo_u32_b32", probe_mbcnt}, {"v_mov_b32_dpp", probe_mov_dpp},
    {"v_mul_f32", probe_mul_f32},       {"v_add_f32", probe_add_f32},     {"v_fma_f32", probe_fma_f32},
    {"v_cvt_f32_i32", probe_cvt_f32_i32}, {"v_cvt_pk_bf16_f32", probe_cvt_pk_bf16}, {"v_cvt_f32_i32_sdwa", probe_cvt_sdwa},
    {"v_cvt_f32_ubyte1", probe_cvt_ubyte}, {"v_dot2_f32_bf16", probe_dot2_bf16}, {"v_dot2c_f32_bf16", probe_dot2c_bf16},
    {"v_cmp_lt_u32 + v_cndmask_b32", probe_cmp_cndmask}, {"v_max_u32", probe_max},
    {"v_bfi_b32", probe_bfi}, {"v_lshrrev_b16", probe_lshr_b16}, {"v_add_u16", probe_add_u16},
    {"ds_read_u16, one address", probe_lds<0, true>}, {"ds_read_u16, entry l", probe_lds<1, true>},
    {"ds_read_b32, dword l", probe_lds<2, false>}, {"ds_read_b32, dword 2l", probe_lds<3, false>},
    {"ds_read_b32, dword 32l", probe_lds<4, false>}, {"ds_read_b32, dword 64l", probe_lds<5, false>},
    {"ds_read_u16, random entry of 2048", probe_lds<6, true>}, {"ds_read_b32, random dword of 1024", probe_lds<6, false>},
};
constexpr uint32_t kProbeCount = sizeof(kProbes) / sizeof(kProbes[0]);
constexpr uint32_t kTurns = 1000, kPerTurn = 32, kWavesPerSimd = 8;

} // namespace

extern "C" uint32_t dc_issue_rate_count() { return kProbeCount; }

extern "C" const char *dc_issue_rate_name(uint32_t which) { return which < kProbeCount ? kProbes[which].name : nullptr; }

extern "C" int dc_issue_rate(uint32_t which, uint32_t *sink_dev, uint64_t sink_bytes, void *hip_stream, double *ns_per_instruction)
{
    if (which >= kProbeCount || !sink_dev || sink_bytes < 1024 || !ns_per_instruction) return DC_E_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int device = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&device) != hipSuccess || hipGetDeviceProperties(&prop, device) != hipSuccess) return DC_E_HIP;
    // eight workgroups of four wavefronts on every compute unit: eight wavefronts on every SIMD
    const uint32_t blocks = (uint32_t)prop.multiProcessorCount * kWavesPerSimd;
    hipEvent_t t0, t1;
    if (hipEventCreate(&t0) != hipSuccess) return DC_E_HIP;
    if (hipEventCreate(&t1) != hipSuccess) {
        (void)hipEventDestroy(t0);
        return DC_E_HIP;
    }
    int rc = DC_OK;
    float ms = 0.0f;
    hipLaunchKernelGGL(kProbes[which].kernel, dim3(blocks), dim3(256), 0, stream, sink_dev, 1u, kTurns); // untimed
    if (hipEventRecord(t0, stream) != hipSuccess) rc = DC_E_HIP;
    hipLaunchKernelGGL(kProbes[which].kernel, dim3(blocks), dim3(256), 0, stream, sink_dev, 2u, kTurns);
    if (hipEventRecord(t1, stream) != hipSuccess || hipEventSynchronize(t1) != hipSuccess ||
        hipEventElapsedTime(&ms, t0, t1) != hipSuccess || hipGetLastError() != hipSuccess)
        rc = DC_E_HIP;
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    if (rc == DC_OK) *ns_per_instruction = (double)ms * 1e6 / ((double)kWavesPerSimd * kTurns * kPerTurn);
    return rc;
}

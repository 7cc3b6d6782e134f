// Device-side helpers shared by the kernels of libdc_mi355x (gfx950, wave64): 128-bit streaming
// accesses, LDS by integer address, cross-lane primitives.
#ifndef DC_DEVICE_H
#define DC_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dcdev {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 128-bit streaming accesses for data that is touched once.
__device__ __forceinline__ void store16_stream(void *p, uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    u32x4 v = {a, b, c, d};
    __builtin_nontemporal_store(v, static_cast<u32x4 *>(p));
}
__device__ __forceinline__ u32x4 load16_stream(const void *p)
{
    return __builtin_nontemporal_load(static_cast<const u32x4 *>(p));
}

// LDS accessed through 32-bit byte addresses, so that address arithmetic stays in one VALU operation.
typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(3))) uint16_t lds_u16;
__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
}
__device__ __forceinline__ uint32_t lds_load32(uint32_t addr) { return *(const lds_u32 *)(uintptr_t)addr; }
__device__ __forceinline__ uint32_t lds_load16(uint32_t addr) { return *(const lds_u16 *)(uintptr_t)addr; }

// Value of another lane through the data-parallel primitives; lanes without a source (and rows that
// the row mask leaves out) read 0.  0x110 + n: n lanes to the right inside a row of 16; 0x142 / 0x143:
// lane 15 of a row to the next row / lane 31 to rows 2 and 3; 0x138: one lane to the right over
// the whole wave.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}

// Inclusive prefix sum over the 64 lanes (HALVES: over each half of 32 lanes on its own).
template <bool HALVES> __device__ __forceinline__ uint32_t lanes_prefix_sum(uint32_t v)
{
    v += dpp_or_zero<0x111, 0xF>(v);
    v += dpp_or_zero<0x112, 0xF>(v);
    v += dpp_or_zero<0x114, 0xF>(v);
    v += dpp_or_zero<0x118, 0xF>(v);
    v += dpp_or_zero<0x142, 0xA>(v);
    if (!HALVES) v += dpp_or_zero<0x143, 0xC>(v);
    return v;
}

// For every lane the last non-zero value among the lanes below it (0 if none).
template <bool HALVES> __device__ __forceinline__ uint32_t lanes_last_nonzero_below(uint32_t v)
{
    uint32_t t;
    v = dpp_or_zero<0x138, 0xF>(v);
    t = dpp_or_zero<0x111, 0xF>(v); v = v ? v : t;
    t = dpp_or_zero<0x112, 0xF>(v); v = v ? v : t;
    t = dpp_or_zero<0x114, 0xF>(v); v = v ? v : t;
    t = dpp_or_zero<0x118, 0xF>(v); v = v ? v : t;
    t = dpp_or_zero<0x142, 0xA>(v); v = v ? v : t;
    if (!HALVES) { t = dpp_or_zero<0x143, 0xC>(v); v = v ? v : t; }
    return v;
}

// Sum over the 64 lanes, result in lane 63.
__device__ __forceinline__ float lanes_sum(float v)
{
#define DC_SUM_STEP(CTRL, MASK) v += __uint_as_float(dpp_or_zero<CTRL, MASK>(__float_as_uint(v)));
    DC_SUM_STEP(0x111, 0xF)
    DC_SUM_STEP(0x112, 0xF)
    DC_SUM_STEP(0x114, 0xF)
    DC_SUM_STEP(0x118, 0xF)
    DC_SUM_STEP(0x142, 0xA)
    DC_SUM_STEP(0x143, 0xC)
#undef DC_SUM_STEP
    return v;
}

} // namespace dcdev

// Records the launch status of the calling thread (dc_last_hip_error() reports it); DC_OK or DC_E_HIP.
int dc_launch_status();

#endif // DC_DEVICE_H

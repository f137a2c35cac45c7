// Device-side helpers shared by the HIP kernels (gfx950, wave64).
#ifndef HIKONV_DEVICE_H
#define HIKONV_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hikonv {

// Value held by the previous lane of the wavefront (lane i receives lane i-1); lane 0
// receives 0.  One DPP move (wave_shr:1 with bound_ctrl: a lane without a source reads 0, so
// the destination needs no preset), no LDS traffic.
__device__ __forceinline__ uint32_t lane_shr1(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x138 /* wave_shr:1 */, 0xf, 0xf, true);
}

__device__ __forceinline__ uint64_t lane_shr1(uint64_t v)
{
    uint32_t lo = lane_shr1((uint32_t)v);
    uint32_t hi = lane_shr1((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// 32 bits starting at bit `sh` (0..31) of the 64-bit value hi:lo.
__device__ __forceinline__ uint32_t funnel_shr(uint32_t hi, uint32_t lo, uint32_t sh)
{
    return __builtin_amdgcn_alignbit(hi, lo, sh);
}

// b-bit field at bit `pos` of w, zero- or sign-extended.
template <bool SIGNED>
__device__ __forceinline__ int32_t field(uint32_t w, uint32_t pos, uint32_t b)
{
    if (SIGNED) return __builtin_amdgcn_sbfe((int)w, pos, b);
    return (int32_t)__builtin_amdgcn_ubfe(w, pos, b);
}

// One packed multiply-accumulate, 32x32+64 -> 64 (Theorem 1's multiply fused with the
// accumulation of products before a split): v_mad_u64_u32 / v_mad_i64_i32.
template <bool SIGNED>
__device__ __forceinline__ uint64_t mad_wide(uint32_t a, uint32_t b, uint64_t acc)
{
    if (SIGNED) return (uint64_t)((int64_t)(int32_t)a * (int64_t)(int32_t)b + (int64_t)acc);
    return (uint64_t)a * (uint64_t)b + acc;
}

// 24x24+32 -> 32: v_mad_u32_u24 / v_mad_i32_i24 (full issue rate).
template <bool SIGNED>
__device__ __forceinline__ uint32_t mad_narrow(uint32_t a, uint32_t b, uint32_t acc)
{
    if (SIGNED) return (uint32_t)(__mul24((int)a, (int)b) + (int)acc);
    return __umul24(a, b) + acc;
}

// a*b + c on 24-bit signed operands, written as the instruction: left to itself the compiler
// turns a chain of these into separate multiplies and three-operand adds (4 instructions for 3
// products instead of 3).
__device__ __forceinline__ int32_t mad24(int32_t a, int32_t b, int32_t c)
{
    int32_t d;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// Segments N.. of an accumulated word (shift by S*N).  A shift that reaches the register
// width happens only for one-tap kernels, which have no high segments: the result is 0.
template <bool SIGNED>
__device__ __forceinline__ uint64_t shr_wide(uint64_t v, uint32_t sh)
{
    if (sh >= 64u) return 0;
    if (SIGNED) return (uint64_t)((int64_t)v >> sh);
    return v >> sh;
}

template <bool SIGNED>
__device__ __forceinline__ uint32_t shr_narrow(uint32_t v, uint32_t sh)
{
    if (sh >= 32u) return 0;
    if (SIGNED) return (uint32_t)((int32_t)v >> sh);
    return v >> sh;
}

} // namespace hikonv

#endif

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

// The TAPS (<= 8) filter taps at g, one byte each, sign- or zero-extended, fetched by scalar
// loads of the aligned dwords that hold them (an aligned dword that contains a valid byte lies
// in that byte's page, so nothing outside the buffer's pages is touched).  The taps arrive in
// scalar registers: no LDS staging and no workgroup barrier ahead of the kernel's first loads.
template <int TAPS>
__device__ __forceinline__ void load_taps_scalar(const uint8_t *g, bool is_signed, int32_t (&taps)[TAPS])
{
    static_assert(TAPS >= 1 && TAPS <= 8, "at most eight taps");
    const uintptr_t a = reinterpret_cast<uintptr_t>(g);
    const uint32_t *gp = reinterpret_cast<const uint32_t *>(a & ~static_cast<uintptr_t>(3));
    const uint32_t first = (uint32_t)(a & 3u);
    const uint32_t last = (first + TAPS - 1) >> 2; // index of the last dword with a tap: 0..2
    uint32_t d[4] = {0u, 0u, 0u, 0u};
    if (last == 0) {
        asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(d[0]) : "s"(gp) : "memory");
    } else if (last == 1) {
        asm volatile("s_load_dword %0, %2, 0x0\n\ts_load_dword %1, %2, 0x4\n\ts_waitcnt lgkmcnt(0)"
                     : "=&s"(d[0]), "=&s"(d[1])
                     : "s"(gp)
                     : "memory");
    } else {
        asm volatile("s_load_dword %0, %3, 0x0\n\ts_load_dword %1, %3, 0x4\n\ts_load_dword %2, %3, 0x8\n\ts_waitcnt lgkmcnt(0)"
                     : "=&s"(d[0]), "=&s"(d[1]), "=&s"(d[2])
                     : "s"(gp)
                     : "memory");
    }
#pragma unroll
    for (int k = 0; k < TAPS; ++k) {
        const uint32_t pos = first * 8u + 8u * k;
        // bytes never straddle a dword
        const uint32_t w = pos < 32u ? d[0] : pos < 64u ? d[1] : d[2];
        const uint32_t b = (w >> (pos & 31u)) & 0xffu;
        taps[k] = is_signed ? (int32_t)(int8_t)b : (int32_t)b;
    }
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

// Packed DNN-layer kernel (Theorem 3 of the paper): the layer is a sum over input channels
// and kernel rows of 1-D row convolutions, each computed block-wise by packed multiplies;
// block products with the same (co, h, x) are accumulated in the packed domain over M
// (ci, kh) pairs before one split (Section "DNN Convolution Extension").
//
// Mapping: one lane owns one packed block x of one output row (n, ho) and CO_T output
// channels.  Activation words A[chunk][n][ci][row][x] come pre-packed from k_pack_act (one
// coalesced dword load per multiply group); weight words B[co][ci][kh][chunk] are wave
// uniform and are fetched with scalar loads, so a multiply-accumulate is one VALU
// instruction with an SGPR operand:
//   WIDE   v_mad_u64_u32 / v_mad_i64_i32   (32x32+64 -> 64)
//   narrow v_mad_u32_u24 / v_mad_i32_i24   (24x24+32 -> 32, full issue rate)
// Split (every M pairs): Comb = Acc + (Acc of lane-1 >> S N) via DPP wave_shr:1, then N
// fields are read and added to int32 accumulators.  For signed data each of the N low
// fields carries a bias of 2^(S-1) (the accumulator starts from it), so every field is
// non-negative when read; the biases are subtracted once at the end.
//
// Each packed row starts with one all-zero word (block -1): the lane that owns it gives
// the row's first real block a zero carry-in.  Rows longer than 63 blocks are cut into
// segments of 63 blocks whose lane 0 recomputes the preceding block.
#ifndef HIKONV_CONV2D_KERNEL_H
#define HIKONV_CONV2D_KERNEL_H

#include "hikonv_device.h"
#include "hikonv_launch.h"

namespace hikonv {

template <int N, int CO_T, bool ANY_SIGNED, bool WIDE>
__global__ __launch_bounds__(256) void k_conv2d_packed(Conv2dArgs p)
{
    typedef typename std::conditional<WIDE, uint64_t, uint32_t>::type acc_t;
    const uint32_t *__restrict__ apk = p.apk;
    const uint32_t *__restrict__ wp = p.wp;

    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int S = p.S;

    // lane -> (output row, packed word index xi); block x = xi - 1
    int64_t row;
    int xi;
    bool halo, active;
    if (p.segs == 0) { // several whole rows per wave
        const int rw = lane / p.Xs;
        xi = lane - rw * p.Xs;
        row = wave * p.rows_per_wave + rw;
        active = rw < p.rows_per_wave && row < p.wave_rows;
        halo = xi == 0;
    } else { // one 63-block segment of a long row per wave
        row = wave / p.segs;
        const int seg = (int)(wave - row * p.segs);
        xi = seg * 63 + lane;
        active = row < p.wave_rows && xi < p.Xs;
        halo = lane == 0;
    }
    if (!active) {
        row = 0;
        xi = 0;
    }
    const int n = (int)(row / p.Ho), ho = (int)(row - (int64_t)n * p.Ho);

    const int co0 = blockIdx.y * CO_T;
    const int64_t row_words = p.Xs;
    const int64_t ci_words = (int64_t)p.Hp * row_words;
    const uint32_t *a_base = apk + ((int64_t)n * p.C * p.Hp + (int64_t)ho * p.stride) * row_words + xi;
    const uint32_t *w_ptr = wp + ((int64_t)(p.cog0 + co0 / 8) * p.terms) * 8 + (co0 & 7);

    acc_t bias = 0;
    if (ANY_SIGNED)
        for (int m = 0; m < N; ++m) bias += (acc_t)1 << (S * m + S - 1);
    const uint32_t fmask = (1u << S) - 1u;
    const uint32_t SN = (uint32_t)(S * N);

    acc_t acc[CO_T];
    int32_t out[CO_T][N];
#pragma unroll
    for (int c = 0; c < CO_T; ++c) {
        acc[c] = bias;
#pragma unroll
        for (int j = 0; j < N; ++j) out[c][j] = 0;
    }

    auto split = [&]() {
#pragma unroll
        for (int c = 0; c < CO_T; ++c) {
            acc_t comb;
            if (WIDE) {
                uint64_t hi = shr_wide<ANY_SIGNED>((uint64_t)acc[c], SN);
                comb = (acc_t)((uint64_t)acc[c] + lane_shr1(hi));
            } else {
                uint32_t hi = shr_narrow<ANY_SIGNED>((uint32_t)acc[c], SN);
                comb = (acc_t)((uint32_t)acc[c] + lane_shr1(hi));
            }
#pragma unroll
            for (int j = 0; j < N; ++j) out[c][j] += (int32_t)((uint32_t)(comb >> (S * j)) & fmask);
            acc[c] = bias;
        }
    };

    int since = 0, nsplit = 0;
    for (int ci = 0; ci < p.C; ++ci) {
        const uint32_t *a_ci = a_base + ci * ci_words;
        for (int kh = 0; kh < p.Kh; ++kh) {
            for (int ch = 0; ch < p.chunks; ++ch) {
                const uint32_t a = a_ci[ch * p.chunk_stride + kh * row_words];
#pragma unroll
                for (int c = 0; c < CO_T; ++c) {
                    const uint32_t b = w_ptr[c];
                    if (WIDE)
                        acc[c] = (acc_t)mad_wide<ANY_SIGNED>(a, b, (uint64_t)acc[c]);
                    else
                        acc[c] = (acc_t)mad_narrow<ANY_SIGNED>(a, b, (uint32_t)acc[c]);
                }
                w_ptr += 8;
            }
            if (++since == p.M) {
                split();
                since = 0;
                ++nsplit;
            }
        }
    }
    if (since) {
        split();
        ++nsplit;
    }

    if (!active || halo) return;
    const int32_t unbias = ANY_SIGNED ? nsplit * (1 << (S - 1)) : 0;
    const int x = xi - 1;
#pragma unroll
    for (int c = 0; c < CO_T; ++c) {
        if (co0 + c >= p.Co) break;
        int32_t *yrow = p.y + (((int64_t)n * p.Co + co0 + c) * p.Ho + ho) * p.Wo;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const int w1 = x * N + j - p.off; // stride-1 output column
            if (w1 >= 0 && w1 < p.Wo1) {
                if (p.stride == 1)
                    yrow[w1] = out[c][j] - unbias;
                else if (w1 % p.stride == 0)
                    yrow[w1 / p.stride] = out[c][j] - unbias;
            }
        }
    }
}

template <int N, bool ANY_SIGNED, bool WIDE>
inline void launch_conv2d_n(const Conv2dArgs &a, int co_tile, dim3 g, hipStream_t stream)
{
    if (co_tile == 8)
        hipLaunchKernelGGL((k_conv2d_packed<N, 8, ANY_SIGNED, WIDE>), g, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((k_conv2d_packed<N, 2, ANY_SIGNED, WIDE>), g, dim3(256), 0, stream, a);
}

template <bool ANY_SIGNED, bool WIDE>
inline hipError_t launch_conv2d_sw(const Conv2dArgs &a, int co_tile, dim3 g, hipStream_t stream)
{
    switch (a.N) {
    case 1: launch_conv2d_n<1, ANY_SIGNED, WIDE>(a, co_tile, g, stream); break;
    case 2: launch_conv2d_n<2, ANY_SIGNED, WIDE>(a, co_tile, g, stream); break;
    case 3: launch_conv2d_n<3, ANY_SIGNED, WIDE>(a, co_tile, g, stream); break;
    case 4: launch_conv2d_n<4, ANY_SIGNED, WIDE>(a, co_tile, g, stream); break;
    case 5: launch_conv2d_n<5, ANY_SIGNED, WIDE>(a, co_tile, g, stream); break;
    case 6: launch_conv2d_n<6, ANY_SIGNED, WIDE>(a, co_tile, g, stream); break;
    case 7: launch_conv2d_n<7, ANY_SIGNED, WIDE>(a, co_tile, g, stream); break;
    case 8: launch_conv2d_n<8, ANY_SIGNED, WIDE>(a, co_tile, g, stream); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_conv2d_wide(const Conv2dArgs &a, bool any_signed, int co_tile, dim3 g, hipStream_t stream);
hipError_t launch_conv2d_narrow(const Conv2dArgs &a, bool any_signed, int co_tile, dim3 g, hipStream_t stream);

} // namespace hikonv
#endif

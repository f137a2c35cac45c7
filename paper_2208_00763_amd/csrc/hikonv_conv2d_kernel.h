// Packed DNN-layer kernels (Theorem 3 of the paper): the layer is a sum over input channels
// and kernel rows of 1-D row convolutions, each computed block-wise by packed multiplies;
// block products with the same (co, h, x) are accumulated in the packed domain over M
// (ci, kh) pairs before one split (Section "DNN Convolution Extension").
//
// Mapping: one lane owns one packed block x of one output row (n, ho) and CO_T output
// channels.  Activation words A[chunk][n][ci][row][x] come pre-packed from k_pack_act (one
// coalesced dword load per term); weight words B[co][term] are wave uniform and are fetched
// with scalar loads, so a multiply-accumulate is one VALU instruction with an SGPR operand:
//   WIDE   v_mad_u64_u32 / v_mad_i64_i32   (32x32+64 -> 64)
//   narrow v_mad_u32_u24 / v_mad_i32_i24   (24x24+32 -> 32)
// Split (every M pairs): Comb = Acc + (Acc of lane-1 >> S N) via DPP wave_shr:1, then N
// fields are read and added to int32 accumulators.  For signed data each of the N low
// fields carries a bias of 2^(S-1) (the accumulator starts from it), so every field is
// non-negative when read; the biases are subtracted once at the end.
//
// Each packed row starts with one all-zero word (block -1): the lane that owns it gives
// the row's first real block a zero carry-in.  Rows longer than 63 blocks are cut into
// segments of 63 blocks whose lane 0 recomputes the preceding block.
//
// k_conv2d_packed is the plain loop (any M).  k_conv2d_pipe is the production kernel: terms
// are walked in groups of four through a table of activation offsets, the loads of the next
// group are issued before the multiplies of the current one, and the term range of a row
// group can be divided among the 2 or 4 waves of a workgroup (partial int32 sums are
// reduced through LDS), which supplies enough waves for layers with few output rows.
#ifndef HIKONV_CONV2D_KERNEL_H
#define HIKONV_CONV2D_KERNEL_H

#include "hikonv_device.h"
#include "hikonv_launch.h"

namespace hikonv {

template <bool WIDE>
struct acc_type {
    typedef uint64_t type;
};
template <>
struct acc_type<false> {
    typedef uint32_t type;
};

// lane -> (output row, packed word index xi); block x = xi - 1
struct LaneMap {
    int n, ho, xi;
    bool active, halo;
};

__device__ __forceinline__ LaneMap map_lane(const Conv2dArgs &p, int64_t row_group, int lane)
{
    LaneMap m;
    int64_t row;
    if (p.segs == 0) { // several whole rows per wave
        const int rw = lane / p.Xs;
        m.xi = lane - rw * p.Xs;
        row = row_group * p.rows_per_wave + rw;
        m.active = rw < p.rows_per_wave && row < p.wave_rows;
        m.halo = m.xi == 0;
    } else { // one 63-block segment of a long row per wave
        row = row_group / p.segs;
        const int seg = (int)(row_group - row * p.segs);
        m.xi = seg * 63 + lane;
        m.active = row < p.wave_rows && m.xi < p.Xs;
        m.halo = lane == 0;
    }
    if (!m.active) {
        row = 0;
        m.xi = 0;
    }
    m.n = (int)(row / p.Ho);
    m.ho = (int)(row - (int64_t)m.n * p.Ho);
    return m;
}

template <int N, int CO_T, bool ANY_SIGNED, bool WIDE>
struct SplitState {
    typedef typename acc_type<WIDE>::type acc_t;
    acc_t acc[CO_T];
    int32_t out[CO_T][N];
    acc_t bias;
    uint32_t fmask, SN;
    int S;

    __device__ __forceinline__ void init(int s)
    {
        S = s;
        bias = 0;
        if (ANY_SIGNED) {
#pragma unroll
            for (int m = 0; m < N; ++m) bias += (acc_t)1 << (S * m + S - 1);
        }
        fmask = (1u << S) - 1u;
        SN = (uint32_t)(S * N);
#pragma unroll
        for (int c = 0; c < CO_T; ++c) {
            acc[c] = bias;
#pragma unroll
            for (int j = 0; j < N; ++j) out[c][j] = 0;
        }
    }

    __device__ __forceinline__ void mad(int c, uint32_t a, uint32_t b)
    {
        if (WIDE)
            acc[c] = (acc_t)mad_wide<ANY_SIGNED>(a, b, (uint64_t)acc[c]);
        else
            acc[c] = (acc_t)mad_narrow<ANY_SIGNED>(a, b, (uint32_t)acc[c]);
    }

    // Theorem 2 in the packed domain, then Eq. output_split in bias form
    __device__ __forceinline__ void split()
    {
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
    }
};

template <int N, int CO_T>
__device__ __forceinline__ void store_outputs(const Conv2dArgs &p, const LaneMap &m, int co0, const int32_t (&out)[CO_T][N],
                                              int32_t unbias)
{
    if (!m.active || m.halo) return;
    const int x = m.xi - 1;
#pragma unroll
    for (int c = 0; c < CO_T; ++c) {
        if (co0 + c >= p.Co) break;
        int32_t *yrow = p.y + (((int64_t)m.n * p.Co + co0 + c) * p.Ho + m.ho) * p.Wo;
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

template <int N, int CO_T, bool ANY_SIGNED, bool WIDE>
__global__ __launch_bounds__(256) void k_conv2d_packed(Conv2dArgs p)
{
    const uint32_t *__restrict__ apk = p.apk;
    const uint32_t *__restrict__ wp = p.wp;
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const LaneMap m = map_lane(p, wave, lane);
    const int co0 = blockIdx.y * CO_T;
    const int64_t row_words = p.Xs;
    const int64_t ci_words = (int64_t)p.Hp * row_words;
    const uint32_t *a_base = apk + ((int64_t)m.n * p.C * p.Hp + (int64_t)m.ho * p.stride) * row_words + m.xi;
    const uint32_t *w_ptr = wp + ((int64_t)(p.cog0 + co0 / 8) * p.terms_pad) * 8 + (co0 & 7);

    SplitState<N, CO_T, ANY_SIGNED, WIDE> st;
    st.init(p.S);
    int since = 0, nsplit = 0;
    for (int ci = 0; ci < p.C; ++ci) {
        const uint32_t *a_ci = a_base + ci * ci_words;
        for (int kh = 0; kh < p.Kh; ++kh) {
            for (int ch = 0; ch < p.chunks; ++ch) {
                const uint32_t a = a_ci[ch * p.chunk_stride + kh * row_words];
#pragma unroll
                for (int c = 0; c < CO_T; ++c) st.mad(c, a, w_ptr[c]);
                w_ptr += 8;
            }
            if (++since == p.M) {
                st.split();
                since = 0;
                ++nsplit;
            }
        }
    }
    if (since) {
        st.split();
        ++nsplit;
    }
    store_outputs<N, CO_T>(p, m, co0, st.out, ANY_SIGNED ? nsplit * (1 << (p.S - 1)) : 0);
}

constexpr int kTermGroup = 4; // terms per pipelined group; packed weights are zero-padded to it

template <int N, int CO_T, bool ANY_SIGNED, bool WIDE>
__global__ __launch_bounds__(256) void k_conv2d_pipe(Conv2dArgs p)
{
    constexpr int U = kTermGroup;
    extern __shared__ int32_t s_red[]; // (4 - 4/ksplit) * CO_T * N * 64 partial sums

    const uint32_t *__restrict__ apk = p.apk;
    const uint32_t *__restrict__ wp = p.wp;
    const int32_t *__restrict__ toff = p.toff;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ks = wave % p.ksplit;                  // which slice of the term range
    const int64_t row_group = (int64_t)blockIdx.x * (4 / p.ksplit) + wave / p.ksplit;
    const LaneMap m = map_lane(p, row_group, lane);
    const int co0 = blockIdx.y * CO_T;
    const uint32_t lane_off =
        (uint32_t)(((int64_t)m.n * p.C * p.Hp + (int64_t)m.ho * p.stride) * p.Xs + m.xi); // words, < 2^31 (host check)

    const int t_begin = ks * p.slice_terms;
    int t_end = t_begin + p.slice_terms;
    if (t_end > p.terms_pad) t_end = p.terms_pad;
    const uint32_t *w_ptr = wp + ((int64_t)(p.cog0 + co0 / 8) * p.terms_pad + t_begin) * 8 + (co0 & 7);

    SplitState<N, CO_T, ANY_SIGNED, WIDE> st;
    st.init(p.S);
    int since = 0, nsplit = 0;

    // two-stage software pipeline: activation offsets are fetched two groups ahead (scalar),
    // activation words and weight words one group ahead; the table has 2U spare zero entries
    int32_t off_n[U];
    uint32_t a_n[U], w_n[U][CO_T];
#pragma unroll
    for (int u = 0; u < U; ++u) off_n[u] = toff[t_begin + u];
    if (t_begin < t_end) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a_n[u] = (apk + off_n[u])[lane_off];
#pragma unroll
            for (int c = 0; c < CO_T; ++c) w_n[u][c] = w_ptr[u * 8 + c];
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) off_n[u] = toff[t_begin + U + u];
    for (int t = t_begin; t < t_end; t += U) {
        uint32_t a_c[U], w_c[U][CO_T];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a_c[u] = a_n[u];
#pragma unroll
            for (int c = 0; c < CO_T; ++c) w_c[u][c] = w_n[u][c];
        }
        w_ptr += U * 8;
        if (t + U < t_end) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                a_n[u] = (apk + off_n[u])[lane_off];
#pragma unroll
                for (int c = 0; c < CO_T; ++c) w_n[u][c] = w_ptr[u * 8 + c];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) off_n[u] = toff[t + 2 * U + u];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int c = 0; c < CO_T; ++c) st.mad(c, a_c[u], w_c[u][c]);
        }
        since += U;
        if (since >= p.split_terms) { // split_terms is a multiple of U
            st.split();
            since = 0;
            ++nsplit;
        }
    }
    if (since) {
        st.split();
        ++nsplit;
    }
    const int32_t unbias = ANY_SIGNED ? nsplit * (1 << (p.S - 1)) : 0;

    if (p.ksplit > 1) {
        // reduce the partial sums of the slices through LDS; the wave with ks == 0 stores
        if (ks > 0) {
            int32_t *dst = s_red + ((wave - wave / p.ksplit - 1) * CO_T * N) * 64 + lane;
#pragma unroll
            for (int c = 0; c < CO_T; ++c)
#pragma unroll
                for (int j = 0; j < N; ++j) dst[(c * N + j) * 64] = st.out[c][j] - unbias;
        }
        __syncthreads();
        if (ks > 0) return;
        for (int k2 = 1; k2 < p.ksplit; ++k2) {
            const int w2 = wave + k2;
            const int32_t *src = s_red + ((w2 - w2 / p.ksplit - 1) * CO_T * N) * 64 + lane;
#pragma unroll
            for (int c = 0; c < CO_T; ++c)
#pragma unroll
                for (int j = 0; j < N; ++j) st.out[c][j] += src[(c * N + j) * 64];
        }
    }
    store_outputs<N, CO_T>(p, m, co0, st.out, unbias);
}

template <int N, bool ANY_SIGNED, bool WIDE>
inline void launch_conv2d_n(const Conv2dArgs &a, int co_tile, dim3 g, hipStream_t stream)
{
    if (a.pipelined) {
        // one slot per wave that hands its partial sums over (4 waves, 4/ksplit of them keep theirs)
        const size_t lds = (size_t)(4 - 4 / a.ksplit) * co_tile * N * 64 * sizeof(int32_t);
        if (co_tile == 8)
            hipLaunchKernelGGL((k_conv2d_pipe<N, 8, ANY_SIGNED, WIDE>), g, dim3(256), lds, stream, a);
        else
            hipLaunchKernelGGL((k_conv2d_pipe<N, 2, ANY_SIGNED, WIDE>), g, dim3(256), lds, stream, a);
    } else {
        if (co_tile == 8)
            hipLaunchKernelGGL((k_conv2d_packed<N, 8, ANY_SIGNED, WIDE>), g, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((k_conv2d_packed<N, 2, ANY_SIGNED, WIDE>), g, dim3(256), 0, stream, a);
    }
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

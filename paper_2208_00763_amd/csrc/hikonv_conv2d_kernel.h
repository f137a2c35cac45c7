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

// {-1,+1} layers (x = 2a - m, w = 2 beta - 1; a, beta in {0,1}; m = 1 inside the image):
//   sum x w = 4 sum a beta - 2 sum a - 2 sum m beta + sum m
// sum m beta is a rectangle sum over the per-channel prefix table of beta, sum m = C * (valid taps).
__device__ __forceinline__ int32_t bipolar_value(const Conv2dArgs &p, int co, int ho, int wo, int32_t sum_ab, int32_t sum_a)
{
    int kh_lo = p.pad - ho * p.stride, kh_hi = p.H + p.pad - ho * p.stride;
    int kw_lo = p.pad - wo * p.stride, kw_hi = p.W + p.pad - wo * p.stride;
    kh_lo = kh_lo < 0 ? 0 : kh_lo;
    kw_lo = kw_lo < 0 ? 0 : kw_lo;
    kh_hi = kh_hi > p.Kh ? p.Kh : kh_hi;
    kw_hi = kw_hi > p.Kw ? p.Kw : kw_hi;
    const int st = p.Kw + 1;
    const int32_t *ps = p.ps + (int64_t)co * (p.Kh + 1) * st;
    const int32_t rect = ps[kh_hi * st + kw_hi] - ps[kh_lo * st + kw_hi] - ps[kh_hi * st + kw_lo] + ps[kh_lo * st + kw_lo];
    return 4 * sum_ab - 2 * sum_a - 2 * rect + p.C * (kh_hi - kh_lo) * (kw_hi - kw_lo);
}

constexpr int kTermTile = 2048; // terms whose weights are staged in LDS at a time (72 KB at most)

template <int N, int CO_T, bool ANY_SIGNED, bool WIDE, bool BIP>
__global__ __launch_bounds__(256) void k_conv2d_pipe(Conv2dArgs p)
{
    constexpr int U = kTermGroup;
    constexpr int CE = CO_T + (BIP ? 1 : 0); // BIP: one more accumulator collects sum a (all-ones weights)
    // LDS: weight words of the current term tile [tile][CO_T] (+ [tile] all-ones words), the
    // activation offsets of its terms [tile + U]; reused at the end for the slice reduction
    extern __shared__ __attribute__((aligned(16))) uint32_t s_mem[];

    const uint32_t *__restrict__ apk = p.apk;
    const uint32_t *__restrict__ wp = p.wp;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ks = wave % p.ksplit;                  // which slice of every term tile
    const int64_t row_group = (int64_t)blockIdx.x * (4 / p.ksplit) + wave / p.ksplit;
    const LaneMap m = map_lane(p, row_group, lane);
    const int co0 = blockIdx.y * CO_T;
    const uint32_t *a_lane = apk + ((int64_t)m.n * p.C * p.Hp + (int64_t)m.ho * p.stride) * p.Xs + m.xi;
    const uint32_t *w_tile = wp + ((int64_t)(p.cog0 + co0 / 8) * p.terms_pad) * 8 + (co0 & 7);
    const uint32_t *w_ones = wp + ((int64_t)p.ones_cog * p.terms_pad) * 8;

    const int tile_cap = p.terms_pad < kTermTile ? p.terms_pad : kTermTile;
    uint32_t *s_w = s_mem;                                   // [tile_cap][CO_T]
    uint32_t *s_w1 = s_w + tile_cap * CO_T;                  // [tile_cap] (BIP)
    int32_t *s_off = reinterpret_cast<int32_t *>(s_w1 + (BIP ? tile_cap : 0)); // [tile_cap + U]

    SplitState<N, CE, ANY_SIGNED, WIDE> st;
    st.init(p.S);
    int since = 0, nsplit = 0;

    for (int tile0 = 0; tile0 < p.terms_pad; tile0 += tile_cap) {
        const int tile_n = p.terms_pad - tile0 < tile_cap ? p.terms_pad - tile0 : tile_cap; // multiple of U
        if (tile0 > 0) __syncthreads();
        // stage the tile: weights (zero beyond the real terms), all-ones words, activation offsets
        for (int i = tid; i < tile_n * CO_T; i += 256) {
            const int t = i / CO_T, c = i - t * CO_T;
            s_w[i] = w_tile[(int64_t)(tile0 + t) * 8 + c];
        }
        for (int t = tid; t < tile_n + U; t += 256) {
            const int term = tile0 + t;
            int32_t off = 0;
            if (term < p.terms) {
                const int ch = term % p.chunks, kh = (term / p.chunks) % p.Kh, ci = term / (p.chunks * p.Kh);
                off = (int32_t)(ch * p.chunk_stride + ((int64_t)ci * p.Hp + kh) * p.Xs);
            }
            s_off[t] = off;
            if (BIP && t < tile_n) s_w1[t] = w_ones[(int64_t)term * 8];
        }
        __syncthreads();

        // this wave's slice of the tile, in groups of U terms, two register buffers for the
        // activation words: the next group's loads are in flight during the multiplies
        const int slice = ((tile_n / U + p.ksplit - 1) / p.ksplit) * U;
        const int t_begin = ks * slice;
        int t_end = t_begin + slice;
        if (t_end > tile_n) t_end = tile_n;
        if (t_begin >= t_end) continue; // wave-uniform; barriers are outside this part

        uint32_t a0[U], a1[U];
        auto request = [&](uint32_t (&a)[U], int t) {
#pragma unroll
            for (int u = 0; u < U; ++u) a[u] = a_lane[s_off[t + u]];
        };
        auto multiply = [&](const uint32_t (&a)[U], int t) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t w[CE];
                if (CO_T % 4 == 0) {
#pragma unroll
                    for (int c4 = 0; c4 < CO_T / 4; ++c4) {
                        const uint4 q = *reinterpret_cast<const uint4 *>(&s_w[(t + u) * CO_T + 4 * c4]);
                        w[4 * c4] = q.x;
                        w[4 * c4 + 1] = q.y;
                        w[4 * c4 + 2] = q.z;
                        w[4 * c4 + 3] = q.w;
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < CO_T; ++c) w[c] = s_w[(t + u) * CO_T + c];
                }
                if (BIP) w[CO_T] = s_w1[t + u];
#pragma unroll
                for (int c = 0; c < CE; ++c) st.mad(c, a[u], w[c]);
            }
            since += U;
            if (since >= p.split_terms) { // split_terms is a multiple of U
                st.split();
                since = 0;
                ++nsplit;
            }
        };

        request(a0, t_begin);
        for (int t = t_begin; t < t_end; t += 2 * U) {
            request(a1, t + U < t_end ? t + U : t); // past the end: re-read this group
            multiply(a0, t);
            if (t + U >= t_end) break;
            request(a0, t + 2 * U < t_end ? t + 2 * U : t);
            multiply(a1, t + U);
        }
    }
    if (since) {
        st.split();
        ++nsplit;
    }
    const int32_t unbias = ANY_SIGNED ? nsplit * (1 << (p.S - 1)) : 0;

    if (p.ksplit > 1) {
        // reduce the partial sums of the slices through LDS; the wave with ks == 0 stores
        int32_t *s_red = reinterpret_cast<int32_t *>(s_mem);
        __syncthreads(); // the weight tile is no longer read
        if (ks > 0) {
            int32_t *dst = s_red + ((wave - wave / p.ksplit - 1) * CE * N) * 64 + lane;
#pragma unroll
            for (int c = 0; c < CE; ++c)
#pragma unroll
                for (int j = 0; j < N; ++j) dst[(c * N + j) * 64] = st.out[c][j] - unbias;
        }
        __syncthreads();
        if (ks > 0) return;
        for (int k2 = 1; k2 < p.ksplit; ++k2) {
            const int w2 = wave + k2;
            const int32_t *src = s_red + ((w2 - w2 / p.ksplit - 1) * CE * N) * 64 + lane;
#pragma unroll
            for (int c = 0; c < CE; ++c)
#pragma unroll
                for (int j = 0; j < N; ++j) st.out[c][j] += src[(c * N + j) * 64];
        }
    }

    if (!BIP) {
        store_outputs<N, CE>(p, m, co0, st.out, unbias);
    } else {
        if (!m.active || m.halo) return;
        const int x = m.xi - 1;
#pragma unroll
        for (int c = 0; c < CO_T; ++c) {
            if (co0 + c >= p.Co) break;
            int32_t *yrow = p.y + (((int64_t)m.n * p.Co + co0 + c) * p.Ho + m.ho) * p.Wo;
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const int w1 = x * N + j - p.off;
                if (w1 >= 0 && w1 < p.Wo1 && w1 % p.stride == 0) {
                    const int wo = w1 / p.stride;
                    yrow[wo] = bipolar_value(p, co0 + c, m.ho, wo, st.out[c][j], st.out[CO_T][j]);
                }
            }
        }
    }
}

// dynamic LDS bytes of k_conv2d_pipe
inline size_t conv2d_pipe_lds(const Conv2dArgs &a, int co_tile, int n)
{
    const int ce = co_tile + (a.fused_bipolar ? 1 : 0);
    const size_t tile_cap = a.terms_pad < kTermTile ? a.terms_pad : kTermTile;
    const size_t stage = (tile_cap * ce + tile_cap + kTermGroup) * 4;
    const size_t reduce = (size_t)(4 - 4 / a.ksplit) * ce * n * 64 * 4;
    return stage > reduce ? stage : reduce;
}

template <int N, bool ANY_SIGNED, bool WIDE>
inline void launch_conv2d_n(const Conv2dArgs &a, int co_tile, dim3 g, hipStream_t stream)
{
    if (a.pipelined) {
        const size_t lds = conv2d_pipe_lds(a, co_tile, N);
        if (a.fused_bipolar) {
            if (ANY_SIGNED) return; // bipolar layers are packed as unsigned bits
            if (co_tile == 8)
                hipLaunchKernelGGL((k_conv2d_pipe<N, 8, false, WIDE, true>), g, dim3(256), lds, stream, a);
            else
                hipLaunchKernelGGL((k_conv2d_pipe<N, 2, false, WIDE, true>), g, dim3(256), lds, stream, a);
        } else if (co_tile == 8)
            hipLaunchKernelGGL((k_conv2d_pipe<N, 8, ANY_SIGNED, WIDE, false>), g, dim3(256), lds, stream, a);
        else
            hipLaunchKernelGGL((k_conv2d_pipe<N, 2, ANY_SIGNED, WIDE, false>), g, dim3(256), lds, stream, a);
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

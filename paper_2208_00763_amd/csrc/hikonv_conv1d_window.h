// Packed 1-D convolution, one lane = one aligned group of G outputs (the form the
// int32-output path takes wherever it applies).  G = 8 with containers of 1, 2 or 4 bits,
// G = 4 with 8-bit containers.
//
// Theorem 2 cuts a long convolution into F_{N,K} blocks whose products overlap by K - 1
// segments.  Here a lane walks the few blocks that cover its own G outputs one after the
// other and carries the high part of a product into the next block in a register, as the
// paper's processor loop does with its `prev` and `this` words (Section "General purpose
// processors"), instead of handing it to the neighbour lane:
//   window  the T = TAPS + G - 1 consecutive elements the group needs, read straight from
//           global memory as three (four) dwords and funnel-shifted to bit 0;
//   pack    A_j = sum_n e[jN + n] 2^(S n), j = 0 .. ceil(T/N) - 1                (Eq. inpack)
//   mul     Acc_j = bias + Hi(Acc_(j-1)) + sum_c A_(j-c) B_c    (v_mad_u64_u32 / v_mad_i64_i32;
//           B_c holds taps cK .. cK+K-1, K = min(TAPS, N); a kernel wider than one B word
//           multiplies the packed word of the block c places back, which is the input
//           delayed by cK = cN elements)
//   align   Hi(Acc) = Acc >> S N, added through the multiply-add's addend (Eq. 1dnx in the
//           packed domain)
//   split   y[.] = field_i(Acc_j) - 2^(S-1) for the G segments jN + i = TAPS-1 .. TAPS+G-2
//           (Eq. output_split in bias form)
//   store   aligned int32x4 stores with the streaming hint; every store instruction of a wave
//           covers whole 128-byte lines of y (see hikonv_quad_stream.h).
// No lane exchange, and no barrier that the arithmetic needs (the skeleton has the workgroup's waves
// meet once, for the timing of their stores); each lane packs T elements for G outputs (the lane-exchange
// kernel packs every element once), which is the cheaper side of the trade on this chip
// because the path is bound by the bytes it writes.
// Groups at a row's ends, or whose loads would leave the buffer, assemble the same window from
// checked element loads (zero outside the row, Eq. pad_f0) and run the same arithmetic.
#ifndef HIKONV_CONV1D_WINDOW_H
#define HIKONV_CONV1D_WINDOW_H

#include <type_traits>

#include "hikonv_quad_stream.h"

namespace hikonv {

// G: outputs per window (8 with containers of up to 4 bits, else 4).
// WIDE: the window needs more than 64 bits, which happens only with 8-bit containers
template <int N, int TAPS, bool A_SIGNED, bool ANY_SIGNED, bool WIDE, int G>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_conv1d_window(Conv1dArgs p)
{
    constexpr int T = TAPS + G - 1;                // elements of a group's window
    constexpr int NB = (T + N - 1) / N;            // blocks that cover them
    constexpr int K = TAPS < N ? TAPS : N;         // taps per B word
    constexpr int CH = (TAPS + K - 1) / K;         // B words (CH > 1 only with K == N)
    static_assert(CH == 1 || K == N, "a delayed block is the packed word of an earlier block only when K == N");

    int32_t s_g[TAPS];
    load_taps_scalar<TAPS>(p.g, p.w_signed != 0, s_g);
    const int S = p.S, b = p.b;
    // B words (Eq. inpack), wave-uniform
    uint32_t bw[CH];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        uint32_t v = 0;
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (ch * K + k < TAPS) v += (uint32_t)s_g[ch * K + k] << (S * k);
        bw[ch] = __builtin_amdgcn_readfirstlane(v);
    }
    const uint32_t fmask = (1u << S) - 1u;
    const uint32_t SN = (uint32_t)(S * N);
    uint64_t bias_low = 0;
    int32_t bias_f = 0;
    if (ANY_SIGNED) {
#pragma unroll
        for (int m = 0; m < N; ++m) bias_low += 1ull << (S * m + S - 1);
        bias_f = 1 << (S - 1);
    }

    // the G outputs of a group from its window (elements at bits t*C of win_hi:win).  The container
    // width is a compile-time constant inside, so an element's dword and bit are known and a
    // container is one bit-field extract (containers never straddle a dword).
    auto group_c = [&](auto cc, uint64_t win, uint32_t win_hi, int32_t (&out)[G]) {
        constexpr int C = decltype(cc)::value;
        const uint32_t dw[3] = {(uint32_t)win, (uint32_t)(win >> 32), win_hi};
        uint32_t a[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            // Eq. inpack from the top element down: one shift-and-add per element
            uint32_t w = 0;
#pragma unroll
            for (int n = N - 1; n >= 0; --n) {
                const int e = j * N + n;
                if (e < T) w = (w << S) + (uint32_t)field<A_SIGNED>(dw[(e * C) >> 5], (uint32_t)((e * C) & 31), (uint32_t)b);
            }
            a[j] = w;
        }
        uint64_t hi = 0;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            uint64_t acc = bias_low + hi;
#pragma unroll
            for (int ch = 0; ch < CH; ++ch)
                if (j - ch >= 0) acc = mad_wide<ANY_SIGNED>(a[j - ch], bw[ch], acc);
            hi = ANY_SIGNED ? (uint64_t)((int64_t)acc >> SN) : acc >> SN;
#pragma unroll
            for (int i = 0; i < N; ++i) {
                constexpr int first = TAPS - 1;
                const int m = j * N + i;
                if (m >= first && m < first + G) {
                    // a packed word fits 32 bits, so S (N - 1) < 32: every segment but the last lies
                    // inside the low dword (one bit-field extract); the last may straddle the dwords
                    const uint32_t f = i < N - 1 ? __builtin_amdgcn_ubfe((uint32_t)acc, (uint32_t)(S * i), (uint32_t)S)
                                                 : (uint32_t)(acc >> (S * i)) & fmask;
                    out[m - first] = (int32_t)f - bias_f;
                }
            }
        }
    };
    // wave-uniform choice of the container width, outside the loops
    __shared__ stream_v4i s_turn[stream_turn_quads(G)];
    auto run = [&](auto cc) {
        for_each_output_group<G, T, WIDE, decltype(cc)::value>(p, p.shift_m - (TAPS - 1), s_turn,
                                          [&](uint64_t win, uint32_t win_hi, int32_t (&out)[G]) { group_c(cc, win, win_hi, out); });
    };
    if constexpr (G == 4) {
        run(std::integral_constant<int, 8>{});
    } else {
        if (p.c == 4)
            run(std::integral_constant<int, 4>{});
        else if (p.c == 2)
            run(std::integral_constant<int, 2>{});
        else
            run(std::integral_constant<int, 1>{});
    }
}

// instantiations live in one translation unit per tap count
template <int TAPS>
hipError_t launch_conv1d_window_taps(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream);

// outputs per window for this call
inline int conv1d_window_group(const Conv1dArgs &a) { return stream_group(a.c); }

// containers of 1, 2 or 4 bits: eight outputs per window (taps + 7 containers within 64 bits);
// 8-bit containers: four, from a window of up to 96 bits
template <int N, int TAPS>
hipError_t launch_window_nt(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream)
{
    const bool octets = conv1d_window_group(a) == 8;
    const bool wide = !octets && (TAPS + 3) * a.c > 64;
    const dim3 g = quad_stream_grid(a, octets ? 8 : 4), b(kStreamThreads);
#define HIKONV_WIN(AS, ANY)                                                                              \
    do {                                                                                                 \
        if (octets) {                                                                                    \
            hipLaunchKernelGGL((k_conv1d_window<N, TAPS, AS, ANY, false, 8>), g, b, 0, stream, a);       \
            return hipGetLastError();                                                                    \
        }                                                                                                \
        if constexpr ((TAPS + 3) * 8 > 64 && N <= 3) {                                                   \
            if (wide) {                                                                                  \
                hipLaunchKernelGGL((k_conv1d_window<N, TAPS, AS, ANY, true, 4>), g, b, 0, stream, a);    \
                return hipGetLastError();                                                                \
            }                                                                                            \
        }                                                                                                \
        if constexpr (N <= 4) { /* groups of 4: 8-bit containers, so N <= 4 */                           \
            if (!wide) {                                                                                 \
                hipLaunchKernelGGL((k_conv1d_window<N, TAPS, AS, ANY, false, 4>), g, b, 0, stream, a);   \
                return hipGetLastError();                                                                \
            }                                                                                            \
        }                                                                                                \
        return hipErrorNotSupported;                                                                     \
    } while (0)
    if (a_signed) HIKONV_WIN(true, true);
    if (any_signed) HIKONV_WIN(false, true);
    HIKONV_WIN(false, false);
#undef HIKONV_WIN
}

template <int TAPS>
hipError_t launch_conv1d_window_taps(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream)
{
    switch (a.N) {
    case 2: return launch_window_nt<2, TAPS>(a, a_signed, any_signed, stream);
    case 3: return launch_window_nt<3, TAPS>(a, a_signed, any_signed, stream);
    case 4: return launch_window_nt<4, TAPS>(a, a_signed, any_signed, stream);
    case 5: return launch_window_nt<5, TAPS>(a, a_signed, any_signed, stream);
    case 6: return launch_window_nt<6, TAPS>(a, a_signed, any_signed, stream);
    case 8: return launch_window_nt<8, TAPS>(a, a_signed, any_signed, stream);
    case 11: return launch_window_nt<11, TAPS>(a, a_signed, any_signed, stream);
    default: return hipErrorNotSupported;
    }
}

} // namespace hikonv
#endif

// 1-D convolution kernels for gfx950.
//
// k_conv1d_packed: Theorem 2 of the paper (a long 1-D convolution as overlap-added
// F_{N,K} blocks) with every block product computed by one 32x32->64 multiply of packed
// words (Theorem 1).  One lane owns one block of N inputs:
//   load   bit-dense row segment (+ halo) staged in LDS by the workgroup, coalesced
//   pack   A = sum_n f[xN+n] 2^(S n)  (Eq. inpack; for signed data plain two's-complement
//          shift-add, which is Eq. signpackslice)
//   mul    Acc = bias + sum_chunk A_chunk * B_chunk        (v_mad_u64_u32 / v_mad_i64_i32)
//   align  Comb = Acc + (Acc of the previous lane >> S N)  (DPP wave_shr:1; Eq. 1dnx in the
//          packed domain)
//   split  y[xN+j] = field_j(Comb) - 2^(S-1)               (Eq. output_split via a bias:
//          adding 2^(S-1) to each low field makes every field non-negative, so the carried
//          sign never arises)
//   store  through an LDS staging tile, 16-byte aligned coalesced int32x4 stores
// k_conv1d_unpacked: the baseline, one v_mad_i32_i24 per low-bit product.
#include <type_traits>

#include "hikonv_quad_stream.h"

namespace hikonv {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kBlocksPerWaveChunk = 63;          // 64 lanes: one halo block + 63 owned blocks
constexpr int kStageMax = 4 * 63 * 32;           // outputs per tile, upper bound (N <= 32)
constexpr int kInMax = 2176;                     // staged input dwords, upper bound

// dword d of the input buffer; the buffer's last bytes may not fill a dword
__device__ __forceinline__ uint32_t load_dword_safe(const uint32_t *x, int64_t d, int64_t total_dwords,
                                                    int64_t total_bytes)
{
    if (d < 0) return 0;
    if (d < total_dwords) return x[d];
    uint32_t v = 0;
    const uint8_t *xb = reinterpret_cast<const uint8_t *>(x);
    for (int t = 0; t < 4; ++t) {
        int64_t byte = d * 4 + t;
        if (byte < total_bytes) v |= (uint32_t)xb[byte] << (8 * t);
    }
    return v;
}

// bits of absolute dword d that belong to elements [0, len) of the row starting at row_bit0
__device__ __forceinline__ uint32_t row_mask(int64_t d, int64_t row_bit0, int64_t row_bit_end)
{
    int64_t lo = row_bit0 - d * 32, hi = row_bit_end - d * 32;
    if (lo < 0) lo = 0;
    if (hi > 32) hi = 32;
    if (hi <= lo) return 0;
    uint32_t m_hi = hi == 32 ? 0xffffffffu : ((1u << hi) - 1u);
    uint32_t m_lo = (1u << lo) - 1u;
    return m_hi & ~m_lo;
}

template <bool A_SIGNED, bool ANY_SIGNED>
__global__ __launch_bounds__(kThreads) void k_conv1d_packed(Conv1dArgs p)
{
    __shared__ uint32_t s_in[kInMax];
    __shared__ __attribute__((aligned(16))) int32_t s_out[kStageMax + 8];
    __shared__ uint32_t s_b[8];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t tile = blockIdx.x % p.tiles_per_row;
    const int64_t r = blockIdx.x / p.tiles_per_row;
    const int N = p.N, S = p.S, c = p.c, b = p.b;
    const int bpt = kWaves * p.CH * kBlocksPerWaveChunk;
    const int64_t xb0 = tile * bpt;

    // B words: chunk ch holds taps [ch*K, ch*K+K) of g (Eq. inpack)
    if (tid < p.chunks) {
        uint32_t bw = 0;
        for (int k = 0; k < p.Kp; ++k) {
            int t = tid * p.Kp + k;
            if (t < p.taps) {
                int32_t gv = p.w_signed ? (int32_t)(int8_t)p.g[t] : (int32_t)p.g[t];
                bw += (uint32_t)gv << (S * k);
            }
        }
        s_b[tid] = bw;
    }

    // stage the row segment this tile reads: elements [e_first, e_end), zero outside [0, len)
    const int64_t row_bit0 = r * p.row_stride_bits;
    const int64_t row_bit_end = row_bit0 + p.len * c;
    const int64_t e_first = (xb0 - 1) * N - (int64_t)(p.chunks - 1) * p.Kp;
    const int64_t e_end = (xb0 + bpt) * N;
    const int64_t d_first = (row_bit0 + e_first * c) >> 5;
    const int n_in = (int)(((row_bit0 + e_end * c + 31) >> 5) - d_first) + 1;
    for (int i = tid; i < n_in; i += kThreads) {
        int64_t d = d_first + i;
        uint32_t m = row_mask(d, row_bit0, row_bit_end);
        s_in[i] = m ? (load_dword_safe(p.x, d, p.total_dwords, p.total_bytes) & m) : 0u;
    }

    // staging offset so that LDS index == global int32 index (mod 4)
    const int64_t o_tile0 = xb0 * N - p.shift_m;
    const int64_t gflat0 = r * p.out_len + o_tile0;
    const int a_off = (int)(((gflat0 % 4) + 4) % 4);
    __syncthreads();

    const uint32_t fmask = (1u << S) - 1u;
    const uint32_t SN = (uint32_t)(S * N);
    uint64_t bias_low = 0;
    int32_t bias_f = 0;
    if (ANY_SIGNED) {
        for (int m = 0; m < N; ++m) bias_low += 1ull << (S * m + S - 1);
        bias_f = 1 << (S - 1);
    }
    const int per = 32 / c;                          // elements per 32-bit window
    // bit position, inside the staged region, of the first element of block xb0
    const int base_bit = (int)(row_bit0 + xb0 * N * c - d_first * 32);

    for (int cc = 0; cc < p.CH; ++cc) {
        const int xl = (wave * p.CH + cc) * kBlocksPerWaveChunk + lane - 1; // block - xb0
        uint64_t acc = bias_low;
        for (int ch = 0; ch < p.chunks; ++ch) {
            // chunk ch multiplies the input delayed by ch*K positions
            int bit = base_bit + (xl * N - ch * p.Kp) * c;
            uint32_t a = 0;
            for (int n0 = 0; n0 < N; n0 += per) {
                uint32_t raw = funnel_shr(s_in[(bit >> 5) + 1], s_in[bit >> 5], (uint32_t)bit & 31u);
                int cnt = N - n0 < per ? N - n0 : per;
                for (int t = 0; t < cnt; ++t)
                    a += (uint32_t)field<A_SIGNED>(raw, (uint32_t)(t * c), (uint32_t)b) << (S * (n0 + t));
                bit += cnt * c;
            }
            acc = mad_wide<ANY_SIGNED>(a, s_b[ch], acc);
        }
        const uint64_t hi = shr_wide<ANY_SIGNED>(acc, SN);
        const uint64_t comb = acc + lane_shr1(hi);
        if (lane > 0) {
            const int idx0 = xl * N + a_off;
            for (int j = 0; j < N; ++j)
                s_out[idx0 + j] = (int32_t)((uint32_t)(comb >> (S * j)) & fmask) - bias_f;
        }
    }
    __syncthreads();

    // coalesced stores: LDS quad q <-> outputs o_tile0 - a_off + 4q .. +3
    const int64_t o_lo = o_tile0 > 0 ? o_tile0 : 0;
    int64_t o_hi = o_tile0 + (int64_t)bpt * N;
    if (o_hi > p.out_len) o_hi = p.out_len;
    const int nquads = (bpt * N + a_off + 3) >> 2;
    int32_t *yrow = p.y + r * p.out_len;
    for (int q = tid; q < nquads; q += kThreads) {
        const int64_t o = o_tile0 - a_off + 4 * (int64_t)q;
        if (o >= o_lo && o + 4 <= o_hi) {
            const int4 v = *reinterpret_cast<const int4 *>(&s_out[4 * q]);
            *reinterpret_cast<int4 *>(&yrow[o]) = v;
        } else {
            for (int t = 0; t < 4; ++t)
                if (o + t >= o_lo && o + t < o_hi) yrow[o + t] = s_out[4 * q + t];
        }
    }
}

template <bool A_SIGNED>
__global__ __launch_bounds__(kThreads) void k_conv1d_unpacked(Conv1dArgs p)
{
    __shared__ int32_t s_g[64];
    if (threadIdx.x < p.taps)
        s_g[threadIdx.x] = p.w_signed ? (int32_t)(int8_t)p.g[threadIdx.x] : (int32_t)p.g[threadIdx.x];
    __syncthreads();
    const int64_t nquads = (p.out_len + 3 + 3) / 4;
    for (int64_t r = blockIdx.y; r < p.rows; r += gridDim.y) {
        const int a_off = (int)((r * p.out_len) & 3);
        // the quads of a wave start on a 128-byte line of y, as in the packed kernel: the row's
        // quad 0 sits `lead` quads into its line, so the lanes are shifted back by that much
        const int lead = (int)(((p.y_phase + r * p.out_len - a_off) >> 2) & 7);
        const int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x - lead;
        if (q < 0 || q >= nquads) continue;
        const int64_t row_bit0 = r * p.row_stride_bits;
        const int64_t o0 = 4 * q - a_off; // first output of this thread's aligned quad
        // elements f[m - taps + 1 .. m + 3], m = o0 + shift_m; element t feeds output u through tap
        // k = u + taps - 1 - t
        int32_t out[4] = {0, 0, 0, 0};
        const int64_t i0 = o0 + p.shift_m - (p.taps - 1);
        for (int t = 0; t < p.taps + 3; ++t) {
            int64_t i = i0 + t;
            int32_t v = 0;
            if (i >= 0 && i < p.len) {
                int64_t bit = row_bit0 + i * p.c;
                uint32_t w = load_dword_safe(p.x, bit >> 5, p.total_dwords, p.total_bytes);
                v = field<A_SIGNED>(w, (uint32_t)(bit & 31), (uint32_t)p.b);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int k = u + p.taps - 1 - t;
                if (k >= 0 && k < p.taps) out[u] = __mul24(v, s_g[k]) + out[u];
            }
        }
        int32_t *yrow = p.y + r * p.out_len;
        if (o0 >= 0 && o0 + 4 <= p.out_len) {
            typedef int32_t v4i __attribute__((ext_vector_type(4)));
            const v4i v4 = {out[0], out[1], out[2], out[3]};
            __builtin_nontemporal_store(v4, reinterpret_cast<v4i *>(&yrow[o0])); // streaming hint, whole lines per wave
        } else {
            for (int u = 0; u < 4; ++u)
                if (o0 + u >= 0 && o0 + u < p.out_len) yrow[o0 + u] = out[u];
        }
    }
}

// Streaming form of the baseline: one lane produces aligned groups of G outputs, each from a
// window of TAPS + G - 1 elements, on the same skeleton as the packed window kernel (same
// loads, same stores, same row handling, the same group size for the same containers); the
// arithmetic is one v_mad_i32_i24 per low-bit product.  Needs the window within 64 bits (three
// dwords) or, WIDE, 96 bits (four).
template <bool A_SIGNED, int TAPS, bool WIDE, int G>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_conv1d_unpacked_fast(Conv1dArgs p)
{
    int32_t gk[TAPS];
    load_taps_scalar<TAPS>(p.g, p.w_signed != 0, gk);
    const int b = p.b;
    // the container width is a compile-time constant inside, so an element is one bit-field
    // extract from the dword that holds it (containers never straddle a dword)
    auto direct_c = [&](auto cc, uint64_t win, uint32_t win_hi, int32_t (&out)[G]) {
        constexpr int C = decltype(cc)::value;
        const uint32_t dw[3] = {(uint32_t)win, (uint32_t)(win >> 32), win_hi};
        bool started[G];
#pragma unroll
        for (int u = 0; u < G; ++u) started[u] = false, out[u] = 0;
#pragma unroll
        for (int t = 0; t < TAPS + G - 1; ++t) {
            const int32_t v = field<A_SIGNED>(dw[(t * C) >> 5], (uint32_t)((t * C) & 31), (uint32_t)b);
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const int k = u + TAPS - 1 - t;
                if (k < 0 || k >= TAPS) continue;
                // the first product of an output is a multiply, every further one a multiply-add
                out[u] = started[u] ? mad24(v, gk[k], out[u]) : __mul24(v, gk[k]);
                started[u] = true;
            }
        }
    };
    // wave-uniform choice of the container width, outside the loops
    __shared__ stream_v4i s_turn[stream_turn_quads(G)];
    auto run = [&](auto cc) {
        for_each_output_group<G, TAPS + G - 1, WIDE, decltype(cc)::value>(p, p.shift_m - (TAPS - 1), s_turn,
                                                     [&](uint64_t win, uint32_t win_hi, int32_t (&out)[G]) { direct_c(cc, win, win_hi, out); });
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

} // namespace

int conv1d_tile_chunks(int N, int64_t n_blocks)
{
    int ch = kStageMax / (kWaves * kBlocksPerWaveChunk * N);
    if (ch > 8) ch = 8;
    int64_t need = ceil_div(n_blocks, kWaves * kBlocksPerWaveChunk);
    if (ch > need) ch = (int)need;
    return ch < 1 ? 1 : ch;
}

hipError_t launch_conv1d_packed(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream)
{
    const int bpt = kWaves * a.CH * kBlocksPerWaveChunk;
    if ((int64_t)bpt * a.N > kStageMax) return hipErrorNotSupported;
    // staged input dwords: ((bpt+1)*N + (chunks-1)*Kp) elements of c bits, plus alignment slack
    const int64_t in_bits = ((int64_t)(bpt + 1) * a.N + (int64_t)(a.chunks - 1) * a.Kp) * a.c;
    if (in_bits / 32 + 4 > kInMax) return hipErrorNotSupported;
    const int64_t grid = a.tiles_per_row * a.rows;
    if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorNotSupported;
    dim3 g((unsigned)grid), b(kThreads);
    if (a_signed)
        hipLaunchKernelGGL((k_conv1d_packed<true, true>), g, b, 0, stream, a);
    else if (any_signed)
        hipLaunchKernelGGL((k_conv1d_packed<false, true>), g, b, 0, stream, a);
    else
        hipLaunchKernelGGL((k_conv1d_packed<false, false>), g, b, 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_conv1d_unpacked(const Conv1dArgs &a, bool a_signed, hipStream_t stream)
{
    if (a.taps > 64) return hipErrorNotSupported;
    const int64_t nquads = (a.out_len + 6) / 4;
    const int64_t gx = ceil_div(nquads + 7, kThreads); // the lanes are shifted by up to 7 quads
    if (gx <= 0 || gx > 0x7fffffffLL) return hipErrorNotSupported;
    dim3 g((unsigned)gx, (unsigned)(a.rows < 65535 ? a.rows : 65535)), b(kThreads);
    const bool octets = stream_group(a.c) == 8; // eight outputs per window, by the packed window kernel's rule
    if (a.taps <= 7 && quad_stream_applicable(a, a.taps + (octets ? 7 : 3)) && ((a.taps + 3) * a.c <= 64 || a.c == 8)) {
        const bool wide_window = !octets && (a.taps + 3) * a.c > 64;
        g = quad_stream_grid(a, octets ? 8 : 4);
        b = dim3(kStreamThreads);
#define HIKONV_UNP(T)                                                                               \
    case T:                                                                                         \
        if (octets && a_signed)                                                                     \
            hipLaunchKernelGGL((k_conv1d_unpacked_fast<true, T, false, 8>), g, b, 0, stream, a);    \
        else if (octets)                                                                            \
            hipLaunchKernelGGL((k_conv1d_unpacked_fast<false, T, false, 8>), g, b, 0, stream, a);   \
        else if (a_signed && wide_window)                                                           \
            hipLaunchKernelGGL((k_conv1d_unpacked_fast<true, T, true, 4>), g, b, 0, stream, a);     \
        else if (a_signed)                                                                          \
            hipLaunchKernelGGL((k_conv1d_unpacked_fast<true, T, false, 4>), g, b, 0, stream, a);    \
        else if (wide_window)                                                                       \
            hipLaunchKernelGGL((k_conv1d_unpacked_fast<false, T, true, 4>), g, b, 0, stream, a);    \
        else                                                                                        \
            hipLaunchKernelGGL((k_conv1d_unpacked_fast<false, T, false, 4>), g, b, 0, stream, a);   \
        break;
        switch (a.taps) {
            HIKONV_UNP(1) HIKONV_UNP(2) HIKONV_UNP(3) HIKONV_UNP(4) HIKONV_UNP(5) HIKONV_UNP(6) HIKONV_UNP(7)
        }
#undef HIKONV_UNP
    } else if (a_signed)
        hipLaunchKernelGGL((k_conv1d_unpacked<true>), g, b, 0, stream, a);
    else
        hipLaunchKernelGGL((k_conv1d_unpacked<false>), g, b, 0, stream, a);
    return hipGetLastError();
}

} // namespace hikonv

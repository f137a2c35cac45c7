// Streaming variant of the packed 1-D convolution (Theorem 2 with Theorem 1 blocks) for the
// common plans (N <= 12, one 32-bit window holds a block's N containers).
//
// Every wavefront works alone, so the kernel has no workgroup barrier: a wave owns a run of
// CH chunks of 63 consecutive blocks.  Per chunk, lane l > 0 owns block x0 + l - 1 and lane 0
// recomputes block x0 - 1, whose high segments lane 1 needs.  A lane
//   reads the two dwords around its block's first container straight from global memory
//   (neighbouring lanes hit the same cache lines), funnel-shifts them into one window,
//   packs A (Eq. inpack), multiplies by the wave-uniform B held in an SGPR
//   (v_mad_u64_u32 / v_mad_i64_i32 with the bias as addend),
//   adds the previous lane's high part (DPP wave_shr:1; Eq. 1dnx in the packed domain),
//   reads the N fields (Eq. output_split in bias form) into the wave's LDS staging run.
// After its CH chunks the wave copies the run to global memory with 16-byte aligned,
// fully coalesced int32x4 stores.  Row edges (zero extension of Eq. pad_f0, and the end of
// the buffer) take a masked path that only the first and last chunk of a row enter.
#include <cstdlib>

#include "hikonv_device.h"
#include "hikonv_launch.h"

namespace hikonv {
namespace {

constexpr int kWavesPerGroup = 4;

// Lanes of a wave chunk that own no block.  Ordinary kernels: lane 0 recomputes the block
// before the chunk (its high segments feed lane 1).  Kernels whose taps are cut into SHARE
// B words of N taps each (K = N): chunk j of a block multiplies the input delayed by j*N
// values, which is the packed word of the block j places back, so a lane packs only its own
// block and takes the delayed words from the lanes before it (DPP); SHARE - 1 more leading
// lanes supply those words and own nothing.
__host__ __device__ constexpr int halo_lanes(int share) { return share > 1 ? share : 1; }
__host__ __device__ constexpr int chunk_blocks(int share) { return 64 - halo_lanes(share); }
// Wave chunks per run: about 1500 outputs.  A run owns an output interval whose ends fall on
// 128-byte lines of y (kAlignOutputs values).  Measured on MI355X: shorter runs are slower, and
// so are coarser alignments once the outputs they leave outside the interval exceed a few percent.
constexpr int kAlignOutputs = 32;
__host__ __device__ constexpr int run_chunks(int n, int /*share*/) { return 24 / n > 0 ? 24 / n : 1; }
// LDS dwords per wave: outputs of a run + alignment slack, rounded to 16 bytes
__host__ __device__ constexpr int run_stage_dwords(int n, int share)
{
    return ((run_chunks(n, share) * chunk_blocks(share) * n + 8 + 3) / 4) * 4;
}

__device__ __forceinline__ uint32_t load_dword_checked(const uint32_t *x, int64_t d, int64_t total_dwords,
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

// MULTI: the taps need several B words.  SHARE = 0: every chunk's delayed window is cut out of
// one 64-bit window and packed again; SHARE = 2..4 (plans with K = N and SHARE chunks): the
// delayed words come from the preceding lanes.
template <int N, bool A_SIGNED, bool ANY_SIGNED, bool MULTI, int SHARE>
__global__ __launch_bounds__(256) void k_conv1d_fast(Conv1dArgs p)
{
    constexpr int HALO = halo_lanes(SHARE);
    constexpr int kChunkBlocks = chunk_blocks(SHARE);
    constexpr int CH = run_chunks(N, SHARE);
    constexpr int STAGE = run_stage_dwords(N, SHARE);
    static_assert(SHARE == 0 || (MULTI && SHARE >= 2 && SHARE <= 4), "shared packing is for 2..4 B words");
    __shared__ __attribute__((aligned(16))) int32_t s_out[kWavesPerGroup * STAGE];
    __shared__ uint32_t s_bw[kWavesPerGroup * 8];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t run = (int64_t)blockIdx.x * kWavesPerGroup + wave; // global run index
    if (run >= p.rows * p.tiles_per_row) return;                      // wave-uniform
    const int64_t r = run / p.tiles_per_row;
    const int64_t t_run = run - r * p.tiles_per_row;
    // Block-aligned runs: the run owns CH*63 consecutive blocks.  Line-aligned runs (staged
    // stores only): the run owns the outputs [o_own0, o_own1) whose ends fall on 128-byte lines
    // of y, starts at the block that holds o_own0 and computes CH*63 blocks from there; the few
    // outputs beyond o_own1 belong to the next run, which recomputes them.
    int64_t xr0 = t_run * (CH * kChunkBlocks); // first owned block of the run
    int64_t o_own0 = 0, o_own1 = 0;
    const bool line_runs = p.aligned_runs != 0;
    if (line_runs) {
        const int phase = (int)((p.y_phase + r * p.out_len) & (p.align_outputs - 1)); // position of this row's output 0 inside its aligned unit
        o_own0 = t_run == 0 ? 0 : t_run * p.run_outputs - phase;
        o_own1 = (t_run + 1) * p.run_outputs - phase;
        if (o_own1 > p.out_len) o_own1 = p.out_len;
        if (o_own0 >= o_own1) return; // wave-uniform: the last interval of this row is empty
        xr0 = (o_own0 + p.shift_m) / N;
    }
    int32_t *stage = s_out + wave * STAGE;

    const int S = p.S, c = p.c, b = p.b;
    const uint32_t fmask = (1u << S) - 1u;
    const uint32_t SN = (uint32_t)(S * N);
    uint64_t bias_low = 0;
    int32_t bias_f = 0;
    if (ANY_SIGNED) {
#pragma unroll
        for (int m = 0; m < N; ++m) bias_low += 1ull << (S * m + S - 1);
        bias_f = 1 << (S - 1);
    }

    // B words (Eq. inpack).  Lane t holds tap t shifted to its slice; the taps of a chunk are
    // summed with lane reads, so B ends up wave-uniform (an SGPR in the single-chunk case).
    // The tap load is issued here and first used after the window loads have been issued.
    const uint8_t g_byte = p.g[lane < p.taps ? lane : p.taps - 1]; // in bounds for every lane
    auto tap_word = [&]() {
        int32_t gv = p.w_signed ? (int32_t)(int8_t)g_byte : (int32_t)g_byte;
        return lane < p.taps ? (uint32_t)gv << (S * (lane % p.Kp)) : 0u;
    };
    auto make_b0 = [&]() {
        const uint32_t my_tap = tap_word();
        uint32_t v = 0;
        for (int k = 0; k < p.taps; ++k) v += __builtin_amdgcn_readlane(my_tap, k);
        return v;
    };
    if (MULTI) {
        const uint32_t my_tap = tap_word();
        for (int ch = 0; ch < p.chunks; ++ch) {
            uint32_t bw = 0;
            for (int k = 0; k < p.Kp; ++k) {
                int t = ch * p.Kp + k;
                if (t < p.taps) bw += __builtin_amdgcn_readlane(my_tap, t);
            }
            if (lane == 0) s_bw[wave * 8 + ch] = bw;
        }
        __builtin_amdgcn_wave_barrier();
    }

    const int64_t row_bit0 = r * p.row_stride_bits;     // bit of element 0 of this row in the buffer
    const int64_t total_bits = p.total_bytes * 8;
    const int64_t o_run0 = xr0 * N - p.shift_m;          // output index of the run's first value
    const int a_off = (int)(((r * p.out_len + o_run0) % 4 + 4) % 4);

    // one block: pack A from a 32-bit window, multiply-accumulate over the chunks' B words
    auto pack = [&](uint32_t raw) {
        uint32_t a = 0;
#pragma unroll
        for (int n = 0; n < N; ++n) a += (uint32_t)field<A_SIGNED>(raw, (uint32_t)(n * c), (uint32_t)b) << (S * n);
        return a;
    };
    // overlap-add with the previous lane, split, stage in the wave's LDS run
    int32_t *yrow = p.y + r * p.out_len;
    auto finish = [&](uint64_t acc, int xl) {
        uint64_t comb = acc;
        if (SN < 64u) // wave-uniform; a one-tap kernel whose slices fill the word has no high part
            comb += lane_shr1(ANY_SIGNED ? (uint64_t)((int64_t)acc >> SN) : acc >> SN);
        if (lane >= HALO) {
            int32_t v[N];
#pragma unroll
            for (int j = 0; j < N; ++j) v[j] = (int32_t)((uint32_t)(comb >> (S * j)) & fmask) - bias_f;
            int32_t *dst = stage + xl * N + a_off;
#pragma unroll
            for (int j = 0; j < N; ++j) dst[j] = v[j];
        }
    };

    // wave-uniform test: every element the run reads lies inside the row, and both dwords of
    // every window lie inside the buffer
    const int64_t e_min = (xr0 - HALO) * N - (MULTI && !SHARE ? (int64_t)(p.chunks - 1) * p.Kp : 0);
    const int64_t e_end = (xr0 + CH * kChunkBlocks) * N;
    const bool interior = e_min >= 0 && e_end <= p.len && row_bit0 + e_end * c + 96 <= total_bits;

    // MULTI: one aligned 64-bit window per block covers every chunk's (delayed) window
    const int span_elems = MULTI && !SHARE ? (p.chunks - 1) * p.Kp + N : N;
    // Runs at a row edge stay on the streaming path as long as the buffer is a whole number
    // of dwords: their loads use clamped dword indices (the clamped dwords only hold
    // containers of elements outside [0, len), which the mask below removes).
    const bool whole_dwords = (p.total_bytes & 3) == 0;
    if ((interior || whole_dwords) && (!MULTI || SHARE || span_elems * c <= 64)) {
        // all loads of the run are issued before the first one is used
        const int delay = MULTI && !SHARE ? (p.chunks - 1) * p.Kp : 0; // elements the last chunk lags
        const int64_t e_lane0 = (xr0 + lane - HALO) * N - delay;       // first element of chunk 0's window
        const int64_t bit0 = row_bit0 + e_lane0 * c;
        const uint32_t sh0 = (uint32_t)bit0 & 31u;
        constexpr int kChunkStep = kChunkBlocks * N;                  // elements between chunks
        uint32_t d0[CH], d1[CH], d2[CH], shv[CH];
        if (interior) {
            const uint32_t *wp0 = p.x + (bit0 >> 5);
#pragma unroll
            for (int cc = 0; cc < CH; ++cc) {
                const uint32_t bitc = sh0 + (uint32_t)(cc * kChunkStep * c); // relative to wp0's dword
                const uint32_t *wp = wp0 + (bitc >> 5);
                d0[cc] = wp[0];
                d1[cc] = wp[1];
                d2[cc] = MULTI && !SHARE ? wp[2] : 0u;
                shv[cc] = bitc & 31u;
            }
        } else {
            const int64_t dbase = bit0 >> 5, dlast = p.total_dwords - 1;
#pragma unroll
            for (int cc = 0; cc < CH; ++cc) {
                const uint32_t bitc = sh0 + (uint32_t)(cc * kChunkStep * c);
                const int64_t d = dbase + (bitc >> 5);
                const int64_t i0 = d < 0 ? 0 : (d > dlast ? dlast : d);
                const int64_t i1 = d + 1 < 0 ? 0 : (d + 1 > dlast ? dlast : d + 1);
                const int64_t i2 = d + 2 < 0 ? 0 : (d + 2 > dlast ? dlast : d + 2);
                d0[cc] = p.x[i0];
                d1[cc] = p.x[i1];
                d2[cc] = MULTI && !SHARE ? p.x[i2] : 0u;
                shv[cc] = bitc & 31u;
            }
        }
        // containers of elements outside [0, len) are cleared (zero extension of Eq. pad_f0)
        auto keep_valid = [&](uint32_t raw, int64_t e0) {
            int64_t lo = e0 < 0 ? -e0 : 0, hi = p.len - e0;
            if (hi > N) hi = N;
            if (hi <= lo) return 0u;
            const uint32_t hi_bits = (uint32_t)(hi * c), lo_bits = (uint32_t)(lo * c);
            const uint32_t m_hi = hi_bits >= 32 ? 0xffffffffu : ((1u << hi_bits) - 1u);
            return raw & m_hi & ~((1u << lo_bits) - 1u);
        };
        const uint32_t b0 = MULTI ? 0u : make_b0();
        uint32_t bsh[SHARE > 0 ? SHARE : 1];
        if (SHARE) {
#pragma unroll
            for (int j = 0; j < SHARE; ++j) bsh[j] = s_bw[wave * 8 + j];
        }
#pragma unroll
        for (int cc = 0; cc < CH; ++cc) {
            const uint32_t w_lo = funnel_shr(d1[cc], d0[cc], shv[cc]);
            const int64_t e_cc = e_lane0 + (int64_t)cc * kChunkStep; // first element of this 64-bit window
            uint64_t acc = bias_low;
            if (!MULTI) {
                const uint32_t raw = interior ? w_lo : keep_valid(w_lo, e_cc);
                acc = mad_wide<ANY_SIGNED>(pack(raw), b0, acc);
            } else if (SHARE) {
                // one packed word per block; chunk j multiplies the word of the block j places back
                uint32_t a = pack(interior ? w_lo : keep_valid(w_lo, e_cc));
                acc = mad_wide<ANY_SIGNED>(a, bsh[0], acc);
#pragma unroll
                for (int j = 1; j < SHARE; ++j) {
                    a = lane_shr1(a);
                    acc = mad_wide<ANY_SIGNED>(a, bsh[j], acc);
                }
            } else {
                const uint64_t win = ((uint64_t)funnel_shr(d2[cc], d1[cc], shv[cc]) << 32) | w_lo;
                for (int ch = 0; ch < p.chunks; ++ch) {
                    const int lag = delay - ch * p.Kp;        // elements between the window start and chunk ch
                    uint32_t raw = (uint32_t)(win >> (lag * c));
                    if (!interior) raw = keep_valid(raw, e_cc + lag);
                    acc = mad_wide<ANY_SIGNED>(pack(raw), s_bw[wave * 8 + ch], acc);
                }
            }
            finish(acc, cc * kChunkBlocks + lane - HALO);
        }
    } else {
        const uint32_t b0 = MULTI ? 0u : make_b0();
#pragma unroll 1
        for (int cc = 0; cc < CH; ++cc) {
            const int xl = cc * kChunkBlocks + lane - HALO; // this lane's block, relative to xr0
            uint64_t acc = bias_low;
            const int nchunks = MULTI ? p.chunks : 1;
            for (int ch = 0; ch < nchunks; ++ch) {
                const int64_t e0 = (xr0 + xl) * N - (int64_t)ch * p.Kp; // first element of the window
                const int64_t bit = row_bit0 + e0 * c;
                uint32_t raw;
                if (interior) {
                    const uint32_t *wp = p.x + (bit >> 5);
                    raw = funnel_shr(wp[1], wp[0], (uint32_t)bit & 31u);
                } else {
                    // masked path: keep only the containers of elements in [0, len)
                    int64_t lo = e0 < 0 ? -e0 : 0, hi = p.len - e0;
                    if (hi > N) hi = N;
                    if (hi <= lo) {
                        raw = 0;
                    } else {
                        const int64_t d = bit >> 5; // arithmetic shift: floors for negative positions
                        uint32_t w0 = load_dword_checked(p.x, d, p.total_dwords, p.total_bytes);
                        uint32_t w1 = load_dword_checked(p.x, d + 1, p.total_dwords, p.total_bytes);
                        raw = funnel_shr(w1, w0, (uint32_t)(bit & 31));
                        const uint32_t hi_bits = (uint32_t)(hi * c), lo_bits = (uint32_t)(lo * c);
                        const uint32_t m_hi = hi_bits >= 32 ? 0xffffffffu : ((1u << hi_bits) - 1u);
                        raw &= m_hi & ~((1u << lo_bits) - 1u);
                    }
                }
                const uint32_t bw = MULTI ? s_bw[wave * 8 + ch] : b0;
                acc = mad_wide<ANY_SIGNED>(pack(raw), bw, acc);
            }
            finish(acc, xl);
        }
    }
    __builtin_amdgcn_wave_barrier();

    // copy the run to global memory: LDS quad q <-> outputs o_run0 - a_off + 4q .. +3
    int64_t o_lo = o_run0 > 0 ? o_run0 : 0;
    int64_t o_hi = o_run0 + CH * kChunkBlocks * N;
    if (o_hi > p.out_len) o_hi = p.out_len;
    if (line_runs) {
        o_lo = o_own0;
        o_hi = o_own1;
    }
    constexpr int NQ = (CH * kChunkBlocks * N + 3 + 3) / 4;
    // The first quad of every store instruction sits on a 128-byte line of y (the row's first
    // run aside), so that no line is split between two instructions.
    int q_first = 0;
    if (line_runs && t_run > 0) q_first = (int)((o_own0 - (o_run0 - a_off)) >> 2);
#pragma unroll 1
    for (int q = q_first + lane; q < NQ; q += 64) {
        const int64_t o = o_run0 - a_off + 4 * (int64_t)q;
        if (o >= o_lo && o + 4 <= o_hi) {
            typedef int32_t v4i __attribute__((ext_vector_type(4)));
            const v4i v4 = *reinterpret_cast<const v4i *>(&stage[4 * q]);
// streaming hint: the outputs are not read again, and every store instruction writes
            // whole 128-byte lines (measured: 0.22 -> 0.18 ms on the 4-bit case; no gain for N = 11)
            if (N <= 10)
                __builtin_nontemporal_store(v4, reinterpret_cast<v4i *>(&yrow[o]));
            else
                *reinterpret_cast<v4i *>(&yrow[o]) = v4;
        } else {
            for (int t = 0; t < 4; ++t)
                if (o + t >= o_lo && o + t < o_hi) yrow[o + t] = stage[4 * q + t];
        }
    }
}

// number of B words whose delayed inputs come from the preceding lanes (0: not this form)
inline int share_of(const Conv1dArgs &a)
{
    return a.chunks >= 2 && a.chunks <= 4 && a.Kp == a.N && a.N >= 2 && a.N <= 5 ? a.chunks : 0;
}

template <int N, bool AS, bool ANY>
hipError_t launch_signs(const Conv1dArgs &a, dim3 g, hipStream_t stream)
{
    const int share = share_of(a);
    if (a.chunks == 1) {
        hipLaunchKernelGGL((k_conv1d_fast<N, AS, ANY, false, 0>), g, dim3(256), 0, stream, a);
    } else if constexpr (N >= 2 && N <= 5) {
        switch (share) {
        case 2: hipLaunchKernelGGL((k_conv1d_fast<N, AS, ANY, true, 2>), g, dim3(256), 0, stream, a); break;
        case 3: hipLaunchKernelGGL((k_conv1d_fast<N, AS, ANY, true, 3>), g, dim3(256), 0, stream, a); break;
        case 4: hipLaunchKernelGGL((k_conv1d_fast<N, AS, ANY, true, 4>), g, dim3(256), 0, stream, a); break;
        default: hipLaunchKernelGGL((k_conv1d_fast<N, AS, ANY, true, 0>), g, dim3(256), 0, stream, a); break;
        }
    } else {
        hipLaunchKernelGGL((k_conv1d_fast<N, AS, ANY, true, 0>), g, dim3(256), 0, stream, a);
    }
    return hipGetLastError();
}

template <int N>
hipError_t launch_n(const Conv1dArgs &a, bool a_signed, bool any_signed, dim3 g, hipStream_t stream)
{
    if (a_signed) return launch_signs<N, true, true>(a, g, stream);
    if (any_signed) return launch_signs<N, false, true>(a, g, stream);
    return launch_signs<N, false, false>(a, g, stream);
}

} // namespace

bool conv1d_fast_applicable(const Conv1dArgs &a)
{
    return a.N >= 1 && a.N <= 12 && a.N * a.c <= 32 && a.chunks <= 8 && a.taps <= 64;
}

static int chunks_per_run(int N, int share)
{
    switch (N * 8 + share) {
#define HIKONV_CASE(n) case n * 8: return run_chunks(n, 0); case n * 8 + 2: return run_chunks(n, 2); \
                       case n * 8 + 3: return run_chunks(n, 3); case n * 8 + 4: return run_chunks(n, 4);
        HIKONV_CASE(1) HIKONV_CASE(2) HIKONV_CASE(3) HIKONV_CASE(4) HIKONV_CASE(5) HIKONV_CASE(6)
        HIKONV_CASE(7) HIKONV_CASE(8) HIKONV_CASE(9) HIKONV_CASE(10) HIKONV_CASE(11) HIKONV_CASE(12)
#undef HIKONV_CASE
    default: return 1;
    }
}

// blocks a wave run owns
static int64_t run_blocks(const Conv1dArgs &a)
{
    return (int64_t)chunks_per_run(a.N, share_of(a)) * chunk_blocks(share_of(a));
}

int64_t conv1d_fast_runs_per_row(const Conv1dArgs &a) { return ceil_div(a.n_blocks, run_blocks(a)); }

// Outputs per line-aligned interval: the run's blocks hold run_blocks*N outputs, the run may
// start up to N-1 outputs before its interval, and the interval is a whole number of 128-byte lines.
int64_t conv1d_fast_run_outputs(const Conv1dArgs &a)
{
    return (run_blocks(a) * a.N - a.N + 1) / a.align_outputs * a.align_outputs;
}

// a.tiles_per_row must hold conv1d_fast_runs_per_row(a), or the number of line-aligned intervals
hipError_t launch_conv1d_fast(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream)
{
    if (!conv1d_fast_applicable(a)) return hipErrorNotSupported;
    const int64_t runs = a.tiles_per_row * a.rows;
    const int64_t grid = ceil_div(runs, kWavesPerGroup);
    if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorNotSupported;
    dim3 g((unsigned)grid);
    switch (a.N) {
#define HIKONV_CASE(n) case n: return launch_n<n>(a, a_signed, any_signed, g, stream);
        HIKONV_CASE(1) HIKONV_CASE(2) HIKONV_CASE(3) HIKONV_CASE(4) HIKONV_CASE(5) HIKONV_CASE(6)
        HIKONV_CASE(7) HIKONV_CASE(8) HIKONV_CASE(9) HIKONV_CASE(10) HIKONV_CASE(11) HIKONV_CASE(12)
#undef HIKONV_CASE
    default: return hipErrorNotSupported;
    }
}

} // namespace hikonv

// 1-D convolution with the outputs requantised in the kernel and written bit-dense
// (Section "Single convolver architecture": quantised feature data can be kept compressed at
// run time): q = min(qmax, max(y, 0) >> shift) in out_bits-bit containers.  With 4 bytes per
// output gone the path is bound by the integer VALUs instead of by HBM writes.
//
// k_conv1d_requant: the packed path (Theorem 2 with Theorem 1 blocks).  A wave owns a run of
// whole output dwords; it computes the CH x 63 packed blocks that cover them (one block per
// lane and chunk, lane 0 recomputing the block before the chunk), exactly as the streaming
// int32 kernel does, clamps and shifts every field, stages the values in its LDS run and
// packs `32/c_out` of them into each output dword.  Blocks that straddle a run boundary are
// computed by both neighbouring waves, so no two waves ever write the same dword.
// k_conv1d_requant_unpacked: the baseline, one v_mad_i32_i24 per low-bit product; one lane
// produces one output dword from a 64-bit window of the row.
#include "hikonv_device.h"
#include "hikonv_launch.h"

namespace hikonv {
namespace {

constexpr int kWavesPerGroup = 4;
constexpr int kChunkBlocks = 63;

__host__ __device__ constexpr int rq_chunks(int n) { return 24 / n > 0 ? 24 / n : 1; }
// LDS run of a wave: slot kStagePad + s - head holds the value at full-convolution index xr0*N + s,
// so that the first output of the run sits on a 16-byte boundary
constexpr int kStagePad = 16;
__host__ __device__ constexpr int rq_stage_dwords(int n) { return ((rq_chunks(n) * kChunkBlocks * n + kStagePad + 3) / 4) * 4; }

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

template <int N, bool A_SIGNED, bool ANY_SIGNED, bool MULTI>
__global__ __launch_bounds__(256) void k_conv1d_requant(Conv1dArgs p)
{
    constexpr int CH = rq_chunks(N);
    constexpr int STAGE = rq_stage_dwords(N);
    __shared__ __align__(16) int32_t s_out[kWavesPerGroup * STAGE];
    __shared__ uint32_t s_bw[kWavesPerGroup * 8];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t run = (int64_t)blockIdx.x * kWavesPerGroup + wave;
    if (run >= p.rows * p.tiles_per_row) return; // wave-uniform
    const int64_t r = run / p.tiles_per_row;
    const int64_t o_first = (run - r * p.tiles_per_row) * p.rq_run_outputs; // first output of the run (dword aligned)
    const int64_t m_first = o_first + p.shift_m;                             // its index in the full convolution
    const int64_t xr0 = m_first / N;                                         // first block that is needed
    const int head = (int)(m_first - xr0 * N);                               // outputs of that block before o_first
    int32_t *stage = s_out + wave * STAGE;

    const int S = p.S, c = p.c, b = p.b;
    const uint32_t SN = (uint32_t)(S * N);
    uint64_t bias_low = 0;
    if (ANY_SIGNED) {
#pragma unroll
        for (int m = 0; m < N; ++m) bias_low += 1ull << (S * m + S - 1);
    }
    // Requantisation on the biased field F = y + 2^(S-1) (signed) or F = y (unsigned): with
    // s = min(shift, S-1), y >> shift clamps to the same value as (F >> s) - (2^(S-1) >> s).
    const int rsh = p.rq_shift < S - 1 ? p.rq_shift : S - 1;
    const uint32_t rmask = (1u << (S - rsh)) - 1u;
    const int32_t rbias = ANY_SIGNED ? (1 << (S - 1)) >> rsh : 0;
    // unsigned fields reach 2^S - 1: a shift of S or more leaves nothing
    const int32_t qmax = (!ANY_SIGNED && p.rq_shift >= S) ? 0 : p.rq_qmax;

    // B words (Eq. inpack): lane t holds tap t shifted to its slice, chunk sums by lane reads
    const uint8_t g_byte = p.g[lane < p.taps ? lane : p.taps - 1];
    auto tap_word = [&]() {
        int32_t gv = p.w_signed ? (int32_t)(int8_t)g_byte : (int32_t)g_byte;
        return lane < p.taps ? (uint32_t)gv << (S * (lane % p.Kp)) : 0u;
    };

    const int64_t row_bit0 = r * p.row_stride_bits;
    const int64_t total_bits = p.total_bytes * 8;
    const int delay = MULTI ? (p.chunks - 1) * p.Kp : 0;
    const int64_t e_min = (xr0 - 1) * N - delay;
    const int64_t e_end = (xr0 + CH * kChunkBlocks) * N;
    const bool interior = e_min >= 0 && e_end <= p.len && row_bit0 + e_end * c + 96 <= total_bits;
    const bool fits64 = !MULTI || (delay + N) * c <= 64; // one 64-bit window holds every chunk's window

    // all window loads of the run first (three dwords cover every chunk's delayed window)
    const int64_t e_lane0 = (xr0 + lane - 1) * N - delay;
    const int64_t bit0 = row_bit0 + e_lane0 * c;
    const uint32_t sh0 = (uint32_t)bit0 & 31u;
    constexpr int kChunkStep = kChunkBlocks * N;
    uint32_t d0[CH], d1[CH], d2[CH], shv[CH];
    if (interior) {
        const uint32_t *wp0 = p.x + (bit0 >> 5);
#pragma unroll
        for (int cc = 0; cc < CH; ++cc) {
            const uint32_t bitc = sh0 + (uint32_t)(cc * kChunkStep * c);
            const uint32_t *wp = wp0 + (bitc >> 5);
            d0[cc] = wp[0];
            d1[cc] = wp[1];
            d2[cc] = MULTI ? wp[2] : 0u;
            shv[cc] = bitc & 31u;
        }
    } else {
        const int64_t dbase = bit0 >> 5;
#pragma unroll
        for (int cc = 0; cc < CH; ++cc) {
            const uint32_t bitc = sh0 + (uint32_t)(cc * kChunkStep * c);
            const int64_t d = dbase + (bitc >> 5);
            d0[cc] = load_dword_checked(p.x, d, p.total_dwords, p.total_bytes);
            d1[cc] = load_dword_checked(p.x, d + 1, p.total_dwords, p.total_bytes);
            d2[cc] = MULTI ? load_dword_checked(p.x, d + 2, p.total_dwords, p.total_bytes) : 0u;
            shv[cc] = bitc & 31u;
        }
    }
    auto keep_valid = [&](uint32_t raw, int64_t e0) { // zero extension of Eq. pad_f0
        int64_t lo = e0 < 0 ? -e0 : 0, hi = p.len - e0;
        if (hi > N) hi = N;
        if (hi <= lo) return 0u;
        const uint32_t hi_bits = (uint32_t)(hi * c), lo_bits = (uint32_t)(lo * c);
        const uint32_t m_hi = hi_bits >= 32 ? 0xffffffffu : ((1u << hi_bits) - 1u);
        return raw & m_hi & ~((1u << lo_bits) - 1u);
    };
    auto pack = [&](uint32_t raw) {
        uint32_t a = 0;
#pragma unroll
        for (int n = 0; n < N; ++n) a += (uint32_t)field<A_SIGNED>(raw, (uint32_t)(n * c), (uint32_t)b) << (S * n);
        return a;
    };

    const uint32_t my_tap = tap_word();
    uint32_t b0 = 0;
    if (!MULTI) {
        for (int k = 0; k < p.taps; ++k) b0 += __builtin_amdgcn_readlane(my_tap, k);
    } else {
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

#pragma unroll
    for (int cc = 0; cc < CH; ++cc) {
        const uint32_t w_lo = funnel_shr(d1[cc], d0[cc], shv[cc]);
        const int64_t e_cc = e_lane0 + (int64_t)cc * kChunkStep;
        uint64_t acc = bias_low;
        if (!MULTI) {
            acc = mad_wide<ANY_SIGNED>(pack(interior ? w_lo : keep_valid(w_lo, e_cc)), b0, acc);
        } else {
            const uint64_t win = ((uint64_t)funnel_shr(d2[cc], d1[cc], shv[cc]) << 32) | w_lo;
            for (int ch = 0; ch < p.chunks; ++ch) {
                const int lag = delay - ch * p.Kp;
                uint32_t raw;
                if (fits64) {
                    raw = (uint32_t)(win >> (lag * c));
                    if (!interior) raw = keep_valid(raw, e_cc + lag);
                } else { // rare: the delayed windows of a block span more than 64 bits
                    const int64_t bit = row_bit0 + (e_cc + lag) * c;
                    const int64_t d = bit >> 5;
                    raw = funnel_shr(load_dword_checked(p.x, d + 1, p.total_dwords, p.total_bytes),
                                     load_dword_checked(p.x, d, p.total_dwords, p.total_bytes), (uint32_t)bit & 31u);
                    raw = keep_valid(raw, e_cc + lag);
                }
                acc = mad_wide<ANY_SIGNED>(pack(raw), s_bw[wave * 8 + ch], acc);
            }
        }
        uint64_t comb = acc;
        if (SN < 64u) comb += lane_shr1(ANY_SIGNED ? (uint64_t)((int64_t)acc >> SN) : acc >> SN);
        if (lane > 0) {
            int32_t *dst = stage + kStagePad - head + (cc * kChunkBlocks + lane - 1) * N;
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const int32_t y = (int32_t)((uint32_t)(comb >> (S * j + rsh)) & rmask) - rbias;
                dst[j] = ANY_SIGNED ? min(max(y, 0), qmax) : (int32_t)min((uint32_t)y, (uint32_t)qmax);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();

    // pack the run's values into output dwords: dword k holds outputs o_first + k*per .. +per-1
    const int per = 32 / p.rq_c_out, c_out = p.rq_c_out;
    int64_t n_out = p.out_len - o_first;
    if (n_out > p.rq_run_outputs) n_out = p.rq_run_outputs;
    const int n_dwords = (int)((n_out + per - 1) / per);
    uint32_t *qrow = p.rq_out + r * p.rq_row_dwords + o_first / per;
    const int4 *src = reinterpret_cast<const int4 *>(stage + kStagePad);
#pragma unroll 1
    for (int k = lane; k < n_dwords; k += 64) {
        uint32_t word = 0;
        const int4 *s4 = src + k * (per >> 2);
        for (int t4 = 0; t4 < (per >> 2); ++t4) {
            const int4 v = s4[t4];
            const int sh = 4 * t4 * c_out;
            word |= (uint32_t)v.x << sh;
            word |= (uint32_t)v.y << (sh + c_out);
            word |= (uint32_t)v.z << (sh + 2 * c_out);
            word |= (uint32_t)v.w << (sh + 3 * c_out);
        }
        const int64_t valid = n_out - (int64_t)k * per; // values past the row's end are not output
        if (valid < per) word &= (1u << (uint32_t)(valid * c_out)) - 1u;
        qrow[k] = word;
    }
}

// Plans outside the streaming kernel's domain (more than 12 slices per word, or a block's
// containers wider than one dword): run-time N, one checked load per element, one chunk of 63
// blocks per wave.  Same run partition and output packing as above.
constexpr int kAnyMaxN = 32;
constexpr int kAnyStage = kChunkBlocks * kAnyMaxN;

template <bool ANY_SIGNED>
__global__ __launch_bounds__(256) void k_conv1d_requant_any(Conv1dArgs p, int a_signed)
{
    __shared__ int32_t s_out[kWavesPerGroup * kAnyStage];
    __shared__ uint32_t s_bw[kWavesPerGroup * 8];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t run = (int64_t)blockIdx.x * kWavesPerGroup + wave;
    if (run >= p.rows * p.tiles_per_row) return; // wave-uniform
    const int N = p.N, S = p.S, c = p.c, b = p.b;
    const int64_t r = run / p.tiles_per_row;
    const int64_t o_first = (run - r * p.tiles_per_row) * p.rq_run_outputs;
    const int64_t m_first = o_first + p.shift_m;
    const int64_t xr0 = m_first / N;
    const int head = (int)(m_first - xr0 * N);
    int32_t *stage = s_out + wave * kAnyStage;
    const uint32_t fmask = (1u << S) - 1u;
    const uint32_t SN = (uint32_t)(S * N);
    uint64_t bias_low = 0;
    int32_t bias_f = 0;
    if (ANY_SIGNED) {
        for (int m = 0; m < N; ++m) bias_low += 1ull << (S * m + S - 1);
        bias_f = 1 << (S - 1);
    }
    const uint8_t g_byte = p.g[lane < p.taps ? lane : p.taps - 1];
    const int32_t gv = p.w_signed ? (int32_t)(int8_t)g_byte : (int32_t)g_byte;
    const uint32_t my_tap = lane < p.taps ? (uint32_t)gv << (S * (lane % p.Kp)) : 0u;
    for (int ch = 0; ch < p.chunks; ++ch) {
        uint32_t bw = 0;
        for (int k = 0; k < p.Kp; ++k) {
            int t = ch * p.Kp + k;
            if (t < p.taps) bw += __builtin_amdgcn_readlane(my_tap, t);
        }
        if (lane == 0) s_bw[wave * 8 + ch] = bw;
    }
    __builtin_amdgcn_wave_barrier();

    const int64_t row_bit0 = r * p.row_stride_bits;
    const int64_t X = xr0 + lane - 1; // this lane's block; lane 0 only supplies the overlap
    uint64_t acc = bias_low;
    for (int ch = 0; ch < p.chunks; ++ch) {
        const int64_t e0 = X * N - (int64_t)ch * p.Kp;
        uint32_t a = 0;
        for (int n = 0; n < N; ++n) {
            const int64_t e = e0 + n;
            if (e < 0 || e >= p.len) continue;
            const int64_t eb = row_bit0 + e * c;
            const uint32_t w = load_dword_checked(p.x, eb >> 5, p.total_dwords, p.total_bytes);
            const int32_t v = a_signed ? field<true>(w, (uint32_t)(eb & 31), (uint32_t)b)
                                       : field<false>(w, (uint32_t)(eb & 31), (uint32_t)b);
            a += (uint32_t)v << (S * n);
        }
        acc = mad_wide<ANY_SIGNED>(a, s_bw[wave * 8 + ch], acc);
    }
    uint64_t comb = acc;
    if (SN < 64u) comb += lane_shr1(ANY_SIGNED ? (uint64_t)((int64_t)acc >> SN) : acc >> SN);
    if (lane > 0) {
        int32_t *dst = stage + (lane - 1) * N;
        for (int j = 0; j < N; ++j) {
            int32_t y = (int32_t)((uint32_t)(comb >> (S * j)) & fmask) - bias_f;
            y = y < 0 ? 0 : y;
            y >>= p.rq_shift;
            dst[j] = y > p.rq_qmax ? p.rq_qmax : y;
        }
    }
    __builtin_amdgcn_wave_barrier();
    const int per = 32 / p.rq_c_out;
    int64_t n_out = p.out_len - o_first;
    if (n_out > p.rq_run_outputs) n_out = p.rq_run_outputs;
    const int n_dwords = (int)((n_out + per - 1) / per);
    uint32_t *qrow = p.rq_out + r * p.rq_row_dwords + o_first / per;
    for (int k = lane; k < n_dwords; k += 64) {
        uint32_t word = 0;
        const int s0 = head + k * per;
        for (int t = 0; t < per; ++t)
            if ((int64_t)k * per + t < n_out) word |= (uint32_t)stage[s0 + t] << (t * p.rq_c_out);
        qrow[k] = word;
    }
}

// Baseline with the same output format: a lane produces unpacked_unroll(PER) output dwords (PER
// values each), 256 dwords apart, from 64-bit windows of the row whose loads are all issued first
// (W96: windows of up to 96 bits from four dwords, for 8-bit containers with 6 or 7 taps).
__host__ __device__ constexpr int unpacked_unroll(int per) { return per <= 8 ? 4 : 1; }

template <bool A_SIGNED, int TAPS, int PER, bool W96 = false>
__global__ __launch_bounds__(256) void k_conv1d_requant_unpacked(Conv1dArgs p)
{
    constexpr int U = unpacked_unroll(PER);
    __shared__ int32_t s_g[64];
    if (threadIdx.x < p.taps)
        s_g[threadIdx.x] = p.w_signed ? (int32_t)(int8_t)p.g[threadIdx.x] : (int32_t)p.g[threadIdx.x];
    __syncthreads();
    int32_t gk[TAPS];
#pragma unroll
    for (int k = 0; k < TAPS; ++k) gk[k] = s_g[k];
    const int64_t total_bits = p.total_bytes * 8;
    const int c = p.c, b = p.b;
    const int64_t row_out_dwords = (p.out_len + PER - 1) / PER;
    const int rsh = p.rq_shift, qmax = p.rq_qmax;

    auto emit = [&](int64_t r, int64_t k, const int32_t (&out)[PER]) {
        uint32_t word = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int32_t y = min(max(out[u], 0) >> rsh, qmax);
            word |= (uint32_t)y << (u * (32 / PER));
        }
        const int64_t valid = p.out_len - k * PER; // values past the row's end are not output
        if (valid < PER) word &= (1u << (uint32_t)(valid * (32 / PER))) - 1u;
        p.rq_out[r * p.rq_row_dwords + k] = word;
    };
    auto accumulate = [&](int32_t (&out)[PER], int t, int32_t v) {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int kk = u + TAPS - 1 - t;
            if (kk >= 0 && kk < TAPS) out[u] = __mul24(v, gk[kk]) + out[u];
        }
    };

    // the PER outputs of a window.  With the same container width in and out (the usual case) the
    // position of an element is a compile-time constant: one bit-field extract from the dword that
    // holds it (a container never straddles a dword).  Taken for containers of 4 and 8 bits, where
    // it is faster (measured at 4096 x 65536, 3 taps: 0.100 against 0.112 ms at 4 bit; at 2 and 1
    // bit the shifted form below is the faster one, 0.094 against 0.131 and 0.234 against 0.264 ms)
    auto window_outputs = [&](uint64_t win, uint32_t win_hi, int32_t (&out)[PER]) {
#pragma unroll
        for (int u = 0; u < PER; ++u) out[u] = 0;
        if (PER <= 8 && c == 32 / PER) { // wave-uniform
            constexpr int CC = 32 / PER;
            const uint32_t dw[3] = {(uint32_t)win, (uint32_t)(win >> 32), win_hi};
#pragma unroll
            for (int t = 0; t < TAPS + PER - 1; ++t)
                accumulate(out, t, field<A_SIGNED>(dw[(t * CC) >> 5], (uint32_t)((t * CC) & 31), (uint32_t)b));
        } else {
#pragma unroll
            for (int t = 0; t < TAPS + PER - 1; ++t) {
                // a container never straddles bit 64 (its width divides 64)
                const uint32_t bits_t = W96 && t * c >= 64 ? win_hi >> (t * c - 64) : (uint32_t)(win >> (t * c));
                accumulate(out, t, field<A_SIGNED>(bits_t, 0u, (uint32_t)b));
            }
        }
    };

    for (int64_t r = blockIdx.y; r < p.rows; r += gridDim.y) {
        const int64_t row_bit0 = r * p.row_stride_bits;
        const int64_t k0 = (int64_t)blockIdx.x * (256 * U) + threadIdx.x;
        // first element read for dword k: k*PER + shift_m - (TAPS-1)
        const int64_t i_first = k0 * PER + p.shift_m - (TAPS - 1);
        const int64_t i_last = (k0 + (U - 1) * 256) * PER + p.shift_m - (TAPS - 1);
        const bool fast = k0 + (U - 1) * 256 < row_out_dwords && i_first >= 0 && i_last + TAPS + PER - 1 <= p.len &&
                          row_bit0 + i_last * c + 128 <= total_bits;
        if (fast) {
            uint32_t w0[U], w1[U], w2[U], w3[U], sh[U];
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const int64_t bit = row_bit0 + (i_first + (int64_t)q * 256 * PER) * c;
                const uint32_t *wp = p.x + (bit >> 5);
                w0[q] = wp[0];
                w1[q] = wp[1];
                w2[q] = wp[2];
                w3[q] = W96 ? wp[3] : 0u; // inside the buffer: the fast path keeps 128 bits from the window's dword
                sh[q] = (uint32_t)bit & 31u;
            }
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const uint64_t win = ((uint64_t)funnel_shr(w2[q], w1[q], sh[q]) << 32) | funnel_shr(w1[q], w0[q], sh[q]);
                int32_t out[PER];
                window_outputs(win, W96 ? funnel_shr(w3[q], w2[q], sh[q]) : 0u, out);
                emit(r, k0 + q * 256, out);
            }
        } else {
            // row ends, short rows, the end of the buffer: the same window from checked loads,
            // with the elements outside the row cleared
#pragma unroll 1
            for (int q = 0; q < U; ++q) {
                const int64_t k = k0 + q * 256;
                if (k >= row_out_dwords) break;
                const int64_t i0 = k * PER + p.shift_m - (TAPS - 1);
                const int64_t wbit = row_bit0 + i0 * c; // negative only before the first row: floor shift, bits 0..31
                const int64_t d = wbit >> 5;
                const uint32_t wsh = (uint32_t)wbit & 31u;
                const uint32_t v0 = load_dword_checked(p.x, d, p.total_dwords, p.total_bytes);
                const uint32_t v1 = load_dword_checked(p.x, d + 1, p.total_dwords, p.total_bytes);
                const uint32_t v2 = load_dword_checked(p.x, d + 2, p.total_dwords, p.total_bytes);
                uint64_t win = ((uint64_t)funnel_shr(v2, v1, wsh) << 32) | funnel_shr(v1, v0, wsh);
                uint32_t win_hi = W96 ? funnel_shr(load_dword_checked(p.x, d + 3, p.total_dwords, p.total_bytes), v2, wsh) : 0u;
                const int64_t lo = i0 < 0 ? -i0 : 0;
                int64_t hi = p.len - i0;
                if (hi > TAPS + PER - 1) hi = TAPS + PER - 1;
                if (hi <= lo) {
                    win = 0;
                    win_hi = 0;
                } else {
                    // lo < TAPS elements: lo_bits < 64; hi_bits up to 96 with four dwords
                    const uint32_t hi_bits = (uint32_t)hi * (uint32_t)c, lo_bits = (uint32_t)lo * (uint32_t)c;
                    const uint64_t m_hi = hi_bits >= 64 ? ~0ull : ((1ull << hi_bits) - 1ull);
                    win &= m_hi & ~((1ull << lo_bits) - 1ull);
                    if (hi_bits <= 64)
                        win_hi = 0;
                    else if (hi_bits < 96)
                        win_hi &= (1u << (hi_bits - 64)) - 1u;
                }
                int32_t out[PER];
                window_outputs(win, win_hi, out);
                emit(r, k, out);
            }
        }
    }
}

// Any taps / widths: one lane = one output dword, one checked load per element.
template <bool A_SIGNED>
__global__ __launch_bounds__(256) void k_conv1d_requant_unpacked_any(Conv1dArgs p)
{
    __shared__ int32_t s_g[64];
    if (threadIdx.x < p.taps)
        s_g[threadIdx.x] = p.w_signed ? (int32_t)(int8_t)p.g[threadIdx.x] : (int32_t)p.g[threadIdx.x];
    __syncthreads();
    const int per = 32 / p.rq_c_out;
    const int64_t row_out_dwords = (p.out_len + per - 1) / per;
    for (int64_t r = blockIdx.y; r < p.rows; r += gridDim.y) {
        const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
        if (k >= row_out_dwords) continue;
        const int64_t row_bit0 = r * p.row_stride_bits;
        uint32_t word = 0;
        for (int u = 0; u < per; ++u) {
            const int64_t o = k * per + u;
            if (o >= p.out_len) break;
            int32_t acc = 0;
            for (int kk = 0; kk < p.taps; ++kk) {
                const int64_t i = o + p.shift_m - kk;
                if (i < 0 || i >= p.len) continue;
                const int64_t eb = row_bit0 + i * p.c;
                const uint32_t w = load_dword_checked(p.x, eb >> 5, p.total_dwords, p.total_bytes);
                acc += field<A_SIGNED>(w, (uint32_t)(eb & 31), (uint32_t)p.b) * s_g[kk];
            }
            acc = acc < 0 ? 0 : acc;
            acc >>= p.rq_shift;
            acc = acc > p.rq_qmax ? p.rq_qmax : acc;
            word |= (uint32_t)acc << (u * p.rq_c_out);
        }
        p.rq_out[r * p.rq_row_dwords + k] = word;
    }
}

template <int N>
hipError_t launch_rq_n(const Conv1dArgs &a, bool a_signed, bool any_signed, dim3 g, hipStream_t stream)
{
    const bool multi = a.chunks > 1;
#define HIKONV_LAUNCH(AS, ANY, MU) hipLaunchKernelGGL((k_conv1d_requant<N, AS, ANY, MU>), g, dim3(256), 0, stream, a)
    if (a_signed) {
        if (multi) HIKONV_LAUNCH(true, true, true); else HIKONV_LAUNCH(true, true, false);
    } else if (any_signed) {
        if (multi) HIKONV_LAUNCH(false, true, true); else HIKONV_LAUNCH(false, true, false);
    } else {
        if (multi) HIKONV_LAUNCH(false, false, true); else HIKONV_LAUNCH(false, false, false);
    }
#undef HIKONV_LAUNCH
    return hipGetLastError();
}

template <int TAPS>
hipError_t launch_rq_unpacked_t(const Conv1dArgs &a, bool a_signed, dim3 g, hipStream_t stream)
{
#define HIKONV_LAUNCH(PER)                                                                                       \
    case PER:                                                                                                    \
        if (a_signed)                                                                                            \
            hipLaunchKernelGGL((k_conv1d_requant_unpacked<true, TAPS, PER>), g, dim3(256), 0, stream, a);        \
        else                                                                                                     \
            hipLaunchKernelGGL((k_conv1d_requant_unpacked<false, TAPS, PER>), g, dim3(256), 0, stream, a);       \
        break;
    // windows of 65..96 bits: 8-bit containers in and out, 6 or 7 taps
    if constexpr (TAPS >= 6) {
        if ((TAPS + 32 / a.rq_c_out - 1) * a.c > 64) {
            if (a.rq_c_out != 8 || (TAPS + 3) * a.c > 96) return hipErrorNotSupported;
            if (a_signed)
                hipLaunchKernelGGL((k_conv1d_requant_unpacked<true, TAPS, 4, true>), g, dim3(256), 0, stream, a);
            else
                hipLaunchKernelGGL((k_conv1d_requant_unpacked<false, TAPS, 4, true>), g, dim3(256), 0, stream, a);
            return hipGetLastError();
        }
    }
    switch (32 / a.rq_c_out) {
        HIKONV_LAUNCH(4) HIKONV_LAUNCH(8) HIKONV_LAUNCH(16) HIKONV_LAUNCH(32)
    default: return hipErrorNotSupported;
    }
#undef HIKONV_LAUNCH
    return hipGetLastError();
}

} // namespace

// outputs per wave run of the packed requantising kernel: whole output dwords that CH*63 blocks cover
bool conv1d_requant_streaming(int N, int c) { return N >= 1 && N <= 12 && N * c <= 32; }

int64_t conv1d_requant_run_outputs(int N, int c, int c_out)
{
    const int per = 32 / c_out;
    if (N < 1 || N > kAnyMaxN) return 0;
    if (!conv1d_requant_streaming(N, c)) return (int64_t)((kChunkBlocks * N - (N - 1)) / per) * per;
    int ch = 1;
    switch (N) {
#define HIKONV_CASE(n) case n: ch = rq_chunks(n); break;
        HIKONV_CASE(1) HIKONV_CASE(2) HIKONV_CASE(3) HIKONV_CASE(4) HIKONV_CASE(5) HIKONV_CASE(6)
        HIKONV_CASE(7) HIKONV_CASE(8) HIKONV_CASE(9) HIKONV_CASE(10) HIKONV_CASE(11) HIKONV_CASE(12)
#undef HIKONV_CASE
    default: return 0;
    }
    return (int64_t)((ch * kChunkBlocks * N - (N - 1)) / per) * per;
}

hipError_t launch_conv1d_requant(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream)
{
    if (a.N < 1 || a.N > kAnyMaxN || a.chunks < 1 || a.chunks > 8) return hipErrorNotSupported;
    if (a.rq_run_outputs <= 0 || a.rq_run_outputs != conv1d_requant_run_outputs(a.N, a.c, a.rq_c_out))
        return hipErrorNotSupported;
    const int64_t grid = ceil_div(a.tiles_per_row * a.rows, kWavesPerGroup);
    if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorNotSupported;
    dim3 g((unsigned)grid);
    if (!conv1d_requant_streaming(a.N, a.c)) {
        if (any_signed)
            hipLaunchKernelGGL(k_conv1d_requant_any<true>, g, dim3(256), 0, stream, a, (int)a_signed);
        else
            hipLaunchKernelGGL(k_conv1d_requant_any<false>, g, dim3(256), 0, stream, a, (int)a_signed);
        return hipGetLastError();
    }
    switch (a.N) {
#define HIKONV_CASE(n) case n: return launch_rq_n<n>(a, a_signed, any_signed, g, stream);
        HIKONV_CASE(1) HIKONV_CASE(2) HIKONV_CASE(3) HIKONV_CASE(4) HIKONV_CASE(5) HIKONV_CASE(6)
        HIKONV_CASE(7) HIKONV_CASE(8) HIKONV_CASE(9) HIKONV_CASE(10) HIKONV_CASE(11) HIKONV_CASE(12)
#undef HIKONV_CASE
    default: return hipErrorNotSupported;
    }
}

hipError_t launch_conv1d_requant_unpacked(const Conv1dArgs &a, bool a_signed, hipStream_t stream)
{
    const int per = 32 / a.rq_c_out;
    const bool windowed = a.taps <= 7 && ((a.taps + per - 1) * a.c <= 64 ||
                                          (a.taps >= 6 && a.rq_c_out == 8 && (a.taps + 3) * a.c <= 96)); // 96: four dwords
    const int64_t gx = ceil_div(ceil_div(a.out_len, per), windowed ? 256 * unpacked_unroll(per) : 256);
    if (gx <= 0 || gx > 0x7fffffffLL) return hipErrorNotSupported;
    dim3 g((unsigned)gx, (unsigned)(a.rows < 65535 ? a.rows : 65535));
    if (!windowed) {
        if (a_signed)
            hipLaunchKernelGGL(k_conv1d_requant_unpacked_any<true>, g, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL(k_conv1d_requant_unpacked_any<false>, g, dim3(256), 0, stream, a);
        return hipGetLastError();
    }
    switch (a.taps) {
#define HIKONV_CASE(t) case t: return launch_rq_unpacked_t<t>(a, a_signed, g, stream);
        HIKONV_CASE(1) HIKONV_CASE(2) HIKONV_CASE(3) HIKONV_CASE(4) HIKONV_CASE(5) HIKONV_CASE(6) HIKONV_CASE(7)
#undef HIKONV_CASE
    default: return hipErrorNotSupported;
    }
}

} // namespace hikonv

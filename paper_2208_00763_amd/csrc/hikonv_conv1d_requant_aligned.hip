// 1-D convolution with requantised bit-dense output, container-aligned slices.
//
// In a 1-D convolution every packed activation word meets one weight word only, so the cost
// of the packed path is the packing itself (Section "Single convolver architecture": features
// are packed at run time), not the multiplication.  This kernel uses the plan of Theorem 1
// with K = 1 that makes packing a mask: slices of S = 16 bits, N = 2 of them in a 32-bit
// word, and slice n of the word for residue rho holds the element rho + n*J of the window,
// J = 16 / c elements apart (c = container bits of the bit-dense input).  Then
//     A_tau = (window >> tau*c) & (value mask at bits 0 and 16)
// is the packed word of elements tau and tau + J, one shift and one AND, and
//     Y_rho = sum_k A_(rho + taps-1-k) * g[k]
// accumulates the taps in the packed domain (the accumulation of products before a split of
// the "DNN Convolution Extension", M = taps) and holds outputs rho and rho + J in its two
// slices.  The guard bits are what 16 bits leave above p + q: the launcher takes this path only
// when taps * max|a| * max|w| fits the slice (2^16 unsigned, 2^15 signed with the bias of
// Eq. output_split in bias form folded into the accumulator's start value).
// (One-bit unsigned values and taps, whose sums stay below 8, use slices of 4 bits, eight to a
// word, J = 4: see the kernel.)
// The slices are exactly the halves that the packed 16-bit instructions work on, so the
// next operator's ReLU, shift and clamp run on both outputs of a word at once, and because
// input and output containers have the same width the J words of a window, shifted by rho*c
// and ORed, are the output dword: no per-field extraction, no staging.
//
// One lane produces kUnroll consecutive output dwords from kUnroll + 2 consecutive dwords of
// the row (two loads, one 16-byte store), kSteps times, 256*kUnroll dwords apart, with the next
// step's loads in flight.
#include "hikonv_device.h"
#include "hikonv_launch.h"

namespace hikonv {
namespace {

typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
typedef int16_t i16x2 __attribute__((ext_vector_type(2)));
// rows start on dword boundaries only: vectors of dwords with dword alignment (global memory takes them)
typedef uint32_t u32x4_dw __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2_dw __attribute__((ext_vector_type(2), aligned(4)));

constexpr int kUnroll = 4;
constexpr int kSteps = 4;
static_assert(kUnroll == 4, "a lane stores its output dwords as one 16-byte vector");

__device__ __forceinline__ uint32_t checked_dword(const uint32_t *x, int64_t d, int64_t total_dwords, int64_t total_bytes)
{
    if (d < 0) return 0;
    if (d < total_dwords) return x[d];
    uint32_t v = 0;
    const uint8_t *xb = reinterpret_cast<const uint8_t *>(x);
    for (int t = 0; t < 4; ++t) {
        const int64_t byte = d * 4 + t;
        if (byte < total_bytes) v |= (uint32_t)xb[byte] << (8 * t);
    }
    return v;
}

// C = container bits (input and output), SW = slice bits (16, or 4 for one-bit values),
// TAPS taps, A_SIGNED / ANY_SIGNED as in the other kernels
template <int C, int SW, int TAPS, bool A_SIGNED, bool ANY_SIGNED>
__global__ __launch_bounds__(256) void k_conv1d_requant_aligned(Conv1dArgs p)
{
    constexpr int J = SW / C;          // residues = elements between neighbouring slices of a word
    constexpr int PER = 32 / C;        // outputs per dword = (32 / SW) * J
    constexpr int NA = J + TAPS - 1;   // packed words per window
    static_assert((PER + TAPS - 1) * C <= 64, "a window must fit 64 bits");
    static_assert(SW == 16 || (SW == 4 && C == 1 && !ANY_SIGNED && TAPS < 8), "nibble slices: one-bit unsigned values only");

    __shared__ int32_t s_g[8];
    if (threadIdx.x < TAPS)
        s_g[threadIdx.x] = p.w_signed ? (int32_t)(int8_t)p.g[threadIdx.x] : (int32_t)p.g[threadIdx.x];
    __syncthreads();
    int32_t gk[TAPS];
#pragma unroll
    for (int k = 0; k < TAPS; ++k) gk[k] = s_g[k];

    const int b = p.b;
    constexpr uint32_t kEverySlice = SW == 16 ? 0x00010001u : 0x11111111u; // bit 0 of every slice
    const uint32_t vmask = ((1u << b) - 1u) * kEverySlice;   // the value bits of every slice
    const int64_t total_bits = p.total_bytes * 8;
    const int64_t row_out_dwords = (p.out_len + PER - 1) / PER;
    // q = min(qmax, max(y, 0) >> shift) on 16-bit fields: a shift that empties the field gives 0
    const int field_bits = ANY_SIGNED ? 15 : 16;
    const uint32_t rsh = p.rq_shift < field_bits ? (uint32_t)p.rq_shift : 0u;
    const uint32_t qmax2 = (p.rq_shift < field_bits ? (uint32_t)p.rq_qmax : 0u) * 0x00010001u;
    uint32_t bias2 = ANY_SIGNED ? 0x80008000u : 0u;   // 2^15 in both slices
    uint64_t sign_flip = 0;                            // bit b-1 of every container of a window
    if (A_SIGNED) {
#pragma unroll
        for (int t = 0; t < 64 / C; ++t) sign_flip |= (uint64_t)(1u << (b - 1)) << (t * C);
        int32_t gsum = 0;
#pragma unroll
        for (int k = 0; k < TAPS; ++k) gsum += gk[k];
        bias2 -= (uint32_t)(gsum * (1 << (b - 1))) * 0x00010001u; // modular: the final sum is exact
    }

    // Nibble slices (one-bit unsigned values, at most 7 taps: a sum stays below 8): a one-bit tap
    // multiplies by AND with 0 or ~0; q = min(qmax, y >> shift) is 1 exactly where y >= 2^shift
    // (nowhere if qmax = 0 or 2^shift > 7): with bit 3 of every slice set, subtracting the threshold
    // leaves bit 3 set where the slice reaches it.
    uint32_t gm[TAPS];
#pragma unroll
    for (int k = 0; k < TAPS; ++k) gm[k] = 0u - (uint32_t)(gk[k] & 1);
    const uint32_t thr4 = (p.rq_qmax >= 1 && p.rq_shift < 3 ? (1u << p.rq_shift) : 8u) * 0x11111111u;

    // the output dword of a window (elements win[t] = x[i_first + t], zero outside the row)
    auto output_dword = [&](uint64_t win) -> uint32_t {
        // Signed activations: with the sign bit of every container flipped the value bits read as
        // f + 2^(b-1) >= 0, so every packed word is too large by 2^(b-1) in every slice and the sum
        // by 2^(b-1) * sum(g) in every slice: a constant of the kernel, taken off the start value.
        if (A_SIGNED) win ^= sign_flip;
        uint32_t a[NA];
#pragma unroll
        for (int t = 0; t < NA; ++t) a[t] = (uint32_t)(win >> (t * C)) & vmask;
        uint32_t word = 0;
#pragma unroll
        for (int rho = 0; rho < J; ++rho) {
            uint32_t q;
            if constexpr (SW == 4) {
                uint32_t y = 0;
#pragma unroll
                for (int k = 0; k < TAPS; ++k) y += a[rho + TAPS - 1 - k] & gm[k];
                q = (((y | 0x88888888u) - thr4) >> 3) & 0x11111111u;
            } else {
                uint32_t y = bias2;
#pragma unroll
                for (int k = 0; k < TAPS; ++k) {
                    if (ANY_SIGNED)
                        y = (uint32_t)(__mul24((int32_t)a[rho + TAPS - 1 - k], gk[k]) + (int32_t)y);
                    else
                        y = __umul24(a[rho + TAPS - 1 - k], (uint32_t)gk[k]) + y;
                    asm("" : "+v"(y)); // opaque: the products chain on the accumulator (one multiply-add each)
                }
                if (ANY_SIGNED) {
                    // biased fields -> two's complement halves, ReLU, shift, clamp
                    const i16x2 s = __builtin_bit_cast(i16x2, y ^ 0x80008000u);
                    const i16x2 zero = {0, 0};
                    const u16x2 r = __builtin_bit_cast(u16x2, __builtin_elementwise_max(s, zero));
                    const u16x2 shv = {(uint16_t)rsh, (uint16_t)rsh};
                    const u16x2 m = __builtin_elementwise_min(r >> shv, __builtin_bit_cast(u16x2, qmax2));
                    q = __builtin_bit_cast(uint32_t, m);
                } else {
                    const u16x2 r = __builtin_bit_cast(u16x2, y);
                    const u16x2 shv = {(uint16_t)rsh, (uint16_t)rsh};
                    const u16x2 m = __builtin_elementwise_min(r >> shv, __builtin_bit_cast(u16x2, qmax2));
                    q = __builtin_bit_cast(uint32_t, m);
                }
            }
            word |= q << (rho * C);
        }
        return word;
    };
    // Positions inside a row fit 32 bits (the launcher checks len * C < 2^31); only the row's
    // base is a 64-bit quantity, and it is uniform.
    const int out_len = (int)p.out_len, len = (int)p.len;
    const int out_dwords = (int)row_out_dwords;
    const int lead = p.shift_m - (TAPS - 1); // first element of the window of dword k: k*PER + lead

    // A lane's loads for one step: kUnroll + 2 dwords hold the windows of its kUnroll
    // consecutive output dwords (consecutive windows are 32 bits apart); ok = all of them lie
    // inside the row and the buffer, so the step takes the two-load path
    struct Fetch {
        u32x4_dw lo;
        u32x2_dw hi;
        uint32_t sh;
        bool ok;
    };
    for (int64_t r = blockIdx.y; r < p.rows; r += gridDim.y) {
        const int64_t row_bit0 = r * p.row_stride_bits;
        const uint32_t *row_dwords = p.x + (row_bit0 >> 5);     // the dword that holds the row's first bit
        const uint32_t row_sh = (uint32_t)row_bit0 & 31u;       // and that bit's position in it
        uint32_t *row_out = p.rq_out + r * p.rq_row_dwords;
        // last bit offset (from row_dwords) at which the kUnroll + 2 dwords of a step still lie in the buffer
        int64_t room = total_bits - (row_bit0 - row_sh) - 32 * (kUnroll + 2);
        const int bit_limit = room < 0 ? -1 : (room > 0x7fffffff ? 0x7fffffff : (int)room);
        auto store = [&](int k, uint32_t word) {
            const int valid = out_len - k * PER; // values past the row's end are not output
            if (valid < PER) word &= (1u << (uint32_t)(valid * C)) - 1u;
            row_out[k] = word;
        };
        auto fetch = [&](int k0) {
            Fetch f;
            const int i_first = k0 * PER + lead;
            const int bit = (int)row_sh + i_first * C; // offset from row_dwords (meaningful when i_first >= 0)
            f.ok = k0 + kUnroll <= out_dwords && i_first >= 0 && i_first + kUnroll * PER + TAPS - 1 <= len && bit <= bit_limit;
            f.sh = (uint32_t)bit & 31u;
            f.lo = u32x4_dw{0, 0, 0, 0};
            f.hi = u32x2_dw{0, 0};
            if (f.ok) {
                const uint32_t *wp = row_dwords + (bit >> 5);
                f.lo = *reinterpret_cast<const u32x4_dw *>(wp);
                f.hi = *reinterpret_cast<const u32x2_dw *>(wp + 4);
            }
            return f;
        };
        auto process = [&](int k0, const Fetch &f) {
            if (k0 >= out_dwords) return;
            if (f.ok) {
                const uint32_t w[kUnroll + 2] = {f.lo.x, f.lo.y, f.lo.z, f.lo.w, f.hi.x, f.hi.y};
                uint32_t out[kUnroll];
#pragma unroll
                for (int q = 0; q < kUnroll; ++q) {
                    const uint64_t win =
                        ((uint64_t)funnel_shr(w[q + 2], w[q + 1], f.sh) << 32) | funnel_shr(w[q + 1], w[q], f.sh);
                    out[q] = output_dword(win);
                }
                if (k0 + kUnroll < out_dwords || out_len % PER == 0) { // no partial dword among these
                    const u32x4_dw v = {out[0], out[1], out[2], out[3]};
                    *reinterpret_cast<u32x4_dw *>(row_out + k0) = v;
                } else {
#pragma unroll
                    for (int q = 0; q < kUnroll; ++q) store(k0 + q, out[q]);
                }
                return;
            }
            // row ends, short rows, the end of the buffer: one window at a time from checked
            // loads, with the elements outside the row cleared (zero extension of Eq. pad_f0)
#pragma unroll 1
            for (int q = 0; q < kUnroll; ++q) {
                const int k = k0 + q;
                if (k >= out_dwords) break;
                const int i0 = k * PER + lead;
                const int64_t wbit = row_bit0 + (int64_t)i0 * C; // negative only before the first row: floor shift, bits 0..31
                const int64_t d = wbit >> 5;
                const uint32_t wsh = (uint32_t)wbit & 31u;
                const uint32_t w0 = checked_dword(p.x, d, p.total_dwords, p.total_bytes);
                const uint32_t w1 = checked_dword(p.x, d + 1, p.total_dwords, p.total_bytes);
                const uint32_t w2 = checked_dword(p.x, d + 2, p.total_dwords, p.total_bytes);
                uint64_t win = ((uint64_t)funnel_shr(w2, w1, wsh) << 32) | funnel_shr(w1, w0, wsh);
                const int lo = i0 < 0 ? -i0 : 0;
                int hi = len - i0;
                if (hi > PER + TAPS - 1) hi = PER + TAPS - 1;
                if (hi <= lo) {
                    win = 0;
                } else {
                    const uint32_t hi_bits = (uint32_t)hi * C, lo_bits = (uint32_t)lo * C; // lo_bits < hi_bits <= 64
                    const uint64_t m_hi = hi_bits >= 64 ? ~0ull : ((1ull << hi_bits) - 1ull);
                    win &= m_hi & ~((1ull << lo_bits) - 1ull);
                }
                store(k, output_dword(win));
            }
        };
        // kSteps steps of 256 lanes x kUnroll dwords per workgroup; the loads of a step are in
        // flight during the arithmetic of the step before (the launcher keeps the grid within 2^31 dwords)
        const int k_first = (int)((blockIdx.x * (unsigned)(kSteps * 256) + threadIdx.x) * (unsigned)kUnroll);
        Fetch cur = fetch(k_first);
#pragma unroll
        for (int it = 0; it < kSteps; ++it) {
            const int k0 = k_first + it * 256 * kUnroll;
            Fetch nxt = cur;
            if (it + 1 < kSteps) nxt = fetch(k0 + 256 * kUnroll);
            process(k0, cur);
            cur = nxt;
        }
    }
}

template <int C, int TAPS>
hipError_t launch_aligned_ct(const Conv1dArgs &a, bool a_signed, bool any_signed, int bits_w, dim3 g, hipStream_t stream)
{
    if constexpr ((32 / C + TAPS - 1) * C <= 64) {
        if (a_signed)
            hipLaunchKernelGGL((k_conv1d_requant_aligned<C, 16, TAPS, true, true>), g, dim3(256), 0, stream, a);
        else if (any_signed)
            hipLaunchKernelGGL((k_conv1d_requant_aligned<C, 16, TAPS, false, true>), g, dim3(256), 0, stream, a);
        else if (conv1d_requant_aligned_slice(a, any_signed, bits_w) == 4)
            // one-bit unsigned values and taps: sums of at most 7 fit nibble slices, eight outputs per word
            hipLaunchKernelGGL((k_conv1d_requant_aligned<1, 4, TAPS, false, false>), g, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((k_conv1d_requant_aligned<C, 16, TAPS, false, false>), g, dim3(256), 0, stream, a);
        return hipGetLastError();
    } else {
        return hipErrorNotSupported;
    }
}

template <int C>
hipError_t launch_aligned_c(const Conv1dArgs &a, bool a_signed, bool any_signed, int bits_w, dim3 g, hipStream_t stream)
{
    switch (a.taps) {
#define HIKONV_CASE(t) case t: return launch_aligned_ct<C, t>(a, a_signed, any_signed, bits_w, g, stream);
        HIKONV_CASE(1) HIKONV_CASE(2) HIKONV_CASE(3) HIKONV_CASE(4) HIKONV_CASE(5) HIKONV_CASE(6) HIKONV_CASE(7)
#undef HIKONV_CASE
    default: return hipErrorNotSupported;
    }
}

} // namespace

// Same containers in and out, a window of one output dword within 64 bits, and every sum of
// taps products within a 16-bit slice (bits_w: weight value bits).
bool conv1d_requant_aligned_applicable(const Conv1dArgs &a, bool a_signed, int bits_w)
{
    if (a.c != a.rq_c_out || (a.c != 1 && a.c != 2 && a.c != 4 && a.c != 8)) return false;
    if (a.taps < 1 || a.taps > 7 || (32 / a.c + a.taps - 1) * a.c > 64) return false;
    if (a.b < 1 || a.b > a.c || bits_w < 1 || bits_w > 8) return false;
    if ((a.len + (1 << 18)) * a.c >= (1LL << 31)) return false; // positions inside a row (and a grid's overhang) are 32-bit in the kernel
    const bool w_signed = a.w_signed != 0;
    // signed products go through the 24-bit multiplier: a packed word (two values 16 bits apart) must fit 24 bits signed
    if ((a_signed || w_signed) && a.b > 7) return false;
    const int64_t max_a = a_signed ? (1LL << (a.b - 1)) : (1LL << a.b) - 1;
    const int64_t max_w = w_signed ? (1LL << (bits_w - 1)) : (1LL << bits_w) - 1;
    const int64_t bound = (int64_t)a.taps * max_a * max_w; // |sum| <= bound
    return (a_signed || w_signed) ? bound < (1LL << 15) : bound < (1LL << 16);
}

int conv1d_requant_aligned_slice(const Conv1dArgs &a, bool any_signed, int bits_w)
{
    return !any_signed && a.c == 1 && a.b == 1 && bits_w == 1 ? 4 : 16;
}

hipError_t launch_conv1d_requant_aligned(const Conv1dArgs &a, bool a_signed, bool any_signed, int bits_w, hipStream_t stream)
{
    const int per = 32 / a.c;
    const int64_t gx = ceil_div(ceil_div(a.out_len, per), 256 * kUnroll * kSteps);
    if (gx <= 0 || gx > 0x7fffffffLL) return hipErrorNotSupported;
    dim3 g((unsigned)gx, (unsigned)(a.rows < 65535 ? a.rows : 65535));
    switch (a.c) {
    case 1: return launch_aligned_c<1>(a, a_signed, any_signed, bits_w, g, stream);
    case 2: return launch_aligned_c<2>(a, a_signed, any_signed, bits_w, g, stream);
    case 4: return launch_aligned_c<4>(a, a_signed, any_signed, bits_w, g, stream);
    case 8: return launch_aligned_c<8>(a, a_signed, any_signed, bits_w, g, stream);
    default: return hipErrorNotSupported;
    }
}

} // namespace hikonv

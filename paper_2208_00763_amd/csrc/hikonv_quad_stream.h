// Shared skeleton of the two streaming 1-D kernels with int32 outputs (the packed
// quad-per-lane kernel and the one-product-per-multiply baseline): rows, aligned output quads,
// window loads, stores and row ends are the same code, so that the two kernels differ only in
// the arithmetic that turns a window of T elements into four outputs.
//
// A lane owns kStreamQuads aligned quads of outputs per row (kStreamThreads quads apart).  The
// window of a quad, its T consecutive elements starting at output index + lead_in, is read
// straight from global memory as three (WIDE: four) dwords and funnel-shifted to bit 0; the
// quad leaves as one int32x4 store with the streaming hint, and the quads of a wave cover
// whole 128-byte lines of y.  Everything that depends only on the row (the range of quads whose
// window lies inside the row and the buffer, bit and byte offsets) is worked out once per row
// with scalar arithmetic; a quad then costs two compares, four integer instructions for its
// addresses and one select.  Quads at a row's ends assemble the same window from checked
// element loads (zero outside the row, Eq. pad_f0).
#ifndef HIKONV_QUAD_STREAM_H
#define HIKONV_QUAD_STREAM_H

#include "hikonv_device.h"
#include "hikonv_launch.h"

namespace hikonv {

constexpr int kStreamThreads = 256;
constexpr int kStreamQuads = 4;

__device__ __forceinline__ uint32_t stream_dword_checked(const uint32_t *x, int64_t d, int64_t total_dwords,
                                                         int64_t total_bytes)
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

// floor(a / 4) and ceil(a / 4) for any sign
__device__ __forceinline__ int floor_quarter(int a) { return a >> 2; }
__device__ __forceinline__ int ceil_quarter(int a) { return (a + 3) >> 2; }

// the launcher's conditions for this skeleton: positions inside a row and byte offsets inside
// the input buffer fit 32 bits, the buffer holds at least four dwords, containers are 1, 2, 4 or 8 bits
inline bool quad_stream_applicable(const Conv1dArgs &a, int window_elems)
{
    if (window_elems * a.c > 96) return false;
    if (a.total_bytes < 16 || a.total_bytes >= (1LL << 32) - 64) return false;
    if (a.out_len >= (1LL << 28)) return false;                  // 16-byte quad offsets inside a row of y fit 32 bits
    return (a.len + (1 << 18)) * a.c < (1LL << 31);
}

inline dim3 quad_stream_grid(const Conv1dArgs &a)
{
    const int64_t nquads = (a.out_len + 6) / 4;
    const int64_t gx = ceil_div(nquads + 7, (int64_t)kStreamThreads * kStreamQuads); // lanes are shifted by up to 7 quads
    return dim3((unsigned)gx, (unsigned)(a.rows < 65535 ? a.rows : 65535));
}

// compute(win, win_hi, out): the T elements of the window sit at bits t*c of win_hi:win
template <int T, bool WIDE, typename F>
__device__ __forceinline__ void for_each_output_quad(const Conv1dArgs &p, int lead_in, F &&compute)
{
    const int out_len = (int)p.out_len, len = (int)p.len;
    const int nquads = (out_len + 3 + 3) / 4;
    const int c = WIDE ? 8 : p.c;
    const int lc = WIDE ? 3 : (p.c == 1 ? 0 : p.c == 2 ? 1 : p.c == 4 ? 2 : 3); // log2 of the container width
    const int64_t total_bits = p.total_bytes * 8;
    const char *xbytes = reinterpret_cast<const char *>(p.x);
    typedef uint32_t u32x3_dw __attribute__((ext_vector_type(3), aligned(4)));
    typedef uint32_t u32x4_dw __attribute__((ext_vector_type(4), aligned(4)));
    typedef int32_t v4i __attribute__((ext_vector_type(4)));

    for (int64_t r = blockIdx.y; r < p.rows; r += gridDim.y) {
        // ---- per row, wave-uniform ----
        const int a_off = (int)((r * p.out_len) & 3);
        // the quads of a wave start on a 128-byte line of y: the row's quad 0 sits `lead` quads
        // into its line, so the lanes are shifted back by that much
        const int lead = (int)(((p.y_phase + r * p.out_len - a_off) >> 2) & 7);
        const int64_t row_bit0 = r * p.row_stride_bits;
        const int row_sh = (int)(row_bit0 & 31);                    // bit of the row's first element in its dword
        const uint32_t row_byte = (uint32_t)((row_bit0 >> 5) << 2); // byte offset of that dword in the buffer
        const int64_t room = total_bits - (row_bit0 - row_sh) - (WIDE ? 160 : 128);
        const int bit_limit = room < 0 ? -1 : (room > 0x7fffffff ? 0x7fffffff : (int)room);
        // quad q: first output o0 = 4q - a_off, first element i0 = o0 + lead_in, window at bit
        // row_sh + i0*c of the row's first dword.  It is interior (window inside the row and the
        // buffer, all four outputs exist) for q_lo <= q <= q_hi:
        const int k_in = lead_in - a_off;                           // i0 = 4q + k_in
        int q_lo = ceil_quarter(-k_in);
        if (q_lo < ceil_quarter(a_off)) q_lo = ceil_quarter(a_off);
        if (q_lo < 0) q_lo = 0;
        int q_hi = nquads - 1;
        if (q_hi > floor_quarter(len - T - k_in)) q_hi = floor_quarter(len - T - k_in);
        if (q_hi > floor_quarter(out_len - 4 + a_off)) q_hi = floor_quarter(out_len - 4 + a_off);
        if (bit_limit < row_sh) {
            q_hi = q_lo - 1;
        } else {
            const int i_max = (bit_limit - row_sh) >> lc;           // largest i0 whose loads stay inside the buffer
            if (q_hi > floor_quarter(i_max - k_in)) q_hi = floor_quarter(i_max - k_in);
        }
        const uint32_t q_span = q_hi >= q_lo ? (uint32_t)(q_hi - q_lo) : 0u;
        const bool none = q_hi < q_lo;
        const int kb = row_sh + k_in * c;                           // window bit = (q << (2 + lc)) + kb
        int32_t *yrow = p.y + r * p.out_len;
        char *ybytes = reinterpret_cast<char *>(yrow) - 4 * a_off;  // quad q is stored at ybytes + 16 q

        // ---- per quad ----
        const int q_first = (int)(blockIdx.x * (unsigned)(kStreamQuads * kStreamThreads) + threadIdx.x) - lead;
        bool interior[kStreamQuads];
        uint32_t w0[kStreamQuads], w1[kStreamQuads], w2[kStreamQuads], w3[kStreamQuads], shv[kStreamQuads];
        bool any_edge = false;
        // all window loads of a lane's quads are issued before the first is used; they are
        // unconditional (a quad that is not interior reads the buffer's first dwords and ignores them)
#pragma unroll
        for (int s = 0; s < kStreamQuads; ++s) {
            const int q = q_first + s * kStreamThreads;
            interior[s] = !none && (uint32_t)(q - q_lo) <= q_span;
            any_edge |= !interior[s] && (uint32_t)q < (uint32_t)nquads;
            const int bit = (int)((uint32_t)q << (2 + lc)) + kb;
            shv[s] = (uint32_t)bit & 31u;
            const uint32_t off = interior[s] ? row_byte + (((uint32_t)bit >> 5) << 2) : 0u;
            if (WIDE) {
                const u32x4_dw v = *reinterpret_cast<const u32x4_dw *>(xbytes + off);
                w0[s] = v.x, w1[s] = v.y, w2[s] = v.z, w3[s] = v.w;
            } else {
                const u32x3_dw v = *reinterpret_cast<const u32x3_dw *>(xbytes + off);
                w0[s] = v.x, w1[s] = v.y, w2[s] = v.z, w3[s] = 0u;
            }
        }
#pragma unroll
        for (int s = 0; s < kStreamQuads; ++s) {
            if (!interior[s]) continue;
            int32_t out[4] = {0, 0, 0, 0};
            const uint32_t sh = shv[s];
            const uint64_t win = ((uint64_t)funnel_shr(w2[s], w1[s], sh) << 32) | funnel_shr(w1[s], w0[s], sh);
            compute(win, WIDE ? funnel_shr(w3[s], w2[s], sh) : 0u, out);
            const v4i v4 = {out[0], out[1], out[2], out[3]};
            const uint32_t yoff = (uint32_t)(q_first + s * kStreamThreads) << 4; // interior: q >= 0, and 16 q < 2^32 (launcher)
            __builtin_nontemporal_store(v4, reinterpret_cast<v4i *>(ybytes + yoff));
        }
        // quads at the row's ends (and where a load would leave the buffer): the same window from
        // checked loads, element by element, zero outside the row; the same arithmetic
        if (__builtin_amdgcn_ballot_w64(any_edge) != 0) {
#pragma unroll 1
            for (int s = 0; s < kStreamQuads; ++s) {
                const int q = q_first + s * kStreamThreads;
                const bool inside = !none && (uint32_t)(q - q_lo) <= q_span;
                if (inside || (uint32_t)q >= (uint32_t)nquads) continue;
                const int o0 = 4 * q - a_off;
                const int i0 = o0 + lead_in;
                uint64_t win = 0;
                uint32_t win_hi = 0;
                for (int t = 0; t < T; ++t) {
                    const int i = i0 + t;
                    if (i < 0 || i >= len) continue;
                    const int64_t eb = row_bit0 + (int64_t)i * c;
                    const uint32_t w = stream_dword_checked(p.x, eb >> 5, p.total_dwords, p.total_bytes);
                    const uint64_t v = (w >> (uint32_t)(eb & 31)) & ((1u << c) - 1u);
                    if (t * c < 64)
                        win |= v << (t * c);
                    else
                        win_hi |= (uint32_t)v << (t * c - 64);
                }
                int32_t out[4] = {0, 0, 0, 0};
                compute(win, win_hi, out);
                for (int u = 0; u < 4; ++u)
                    if (o0 + u >= 0 && o0 + u < out_len) yrow[o0 + u] = out[u];
            }
        }
    }
}

} // namespace hikonv
#endif

// Shared skeleton of the two streaming 1-D kernels with int32 outputs (the packed window
// kernel and the one-product-per-multiply baseline): rows, aligned output groups, window
// loads, stores and row ends are the same code, so that the two kernels differ only in the
// arithmetic that turns a window of T elements into G outputs.
//
// A workgroup makes one pass over one row and ends; walking several rows per workgroup with
// the next row's loads requested ahead was measured slower (0.207 against 0.183 ms over the
// 1-4 bit cases at four rows per workgroup), as were four groups of eight per lane.
//
// A lane owns aligned groups of G outputs (G = 8 where the window of taps + 7 containers fits
// 64 bits, i.e. containers of 1, 2 or 4 bits; else aligned quads, G = 4): 16 outputs per row
// pass, its groups kStreamThreads groups apart.  The window of a group, its T = taps + G - 1
// consecutive elements starting at output index + lead_in, is read straight from global memory
// as three (WIDE: four) dwords and funnel-shifted to bit 0; the group leaves as int32x4 stores
// and the groups of a wave cover whole 128-byte lines of y.  Eight outputs per window halve
// the index arithmetic per output and let neighbouring outputs share the window's elements
// (the packed kernel packs (taps + 7)/8 elements per output instead of (taps + 3)/4).  Everything that depends only on the row (the range of quads whose
// window lies inside the row and the buffer, bit and byte offsets) is worked out once per row
// with scalar arithmetic; a group then costs two compares, four integer instructions for its
// addresses and one select.  Groups at a row's ends assemble the same window from checked
// element loads (zero outside the row, Eq. pad_f0).
#ifndef HIKONV_QUAD_STREAM_H
#define HIKONV_QUAD_STREAM_H

#include "hikonv_device.h"
#include "hikonv_launch.h"

namespace hikonv {

constexpr int kStreamThreads = 256;
// outputs per window: 8 where taps + 7 containers fit 64 bits (containers of 1, 2 or 4 bits), else 4
inline int stream_group(int container_bits) { return container_bits <= 4 ? 8 : 4; }
// groups a lane makes per row pass: 16 outputs either way (measured: four groups of 8 are slower than two)
constexpr int stream_steps(int group) { return 16 / group; }

// the launcher's conditions for this skeleton: positions inside a row and byte offsets inside
// the input buffer fit 32 bits, the buffer holds at least four dwords, containers are 1, 2, 4 or 8 bits
inline bool quad_stream_applicable(const Conv1dArgs &a, int window_elems)
{
    if (window_elems * a.c > 96) return false;
    if (a.total_bytes < 16 || a.total_bytes >= (1LL << 32) - 64) return false;
    if (a.out_len >= (1LL << 28)) return false;                  // 16-byte quad offsets inside a row of y fit 32 bits
    return (a.len + (1 << 18)) * a.c < (1LL << 31);
}

inline dim3 quad_stream_grid(const Conv1dArgs &a, int group = 4)
{
    const int64_t ngroups = (a.out_len + 2 * (group - 1)) / group;
    const int steps = stream_steps(group);
    // lanes are shifted back by up to a 128-byte line of groups
    const int64_t gx = ceil_div(ngroups + 32 / group - 1, (int64_t)kStreamThreads * steps);
    return dim3((unsigned)gx, (unsigned)(a.rows < 65535 ? a.rows : 65535));
}

// compute(win, win_hi, out): the T = taps + G - 1 elements of the window sit at bits t*c of
// win_hi:win; out receives the group's G outputs.  G = 4: one streaming int32x4 store per group.
// G = 8 (windows within 64 bits): two int32x4 stores per group.
typedef int32_t stream_v4i __attribute__((ext_vector_type(4)));
// LDS the skeleton needs per workgroup, in 16-byte units (the caller declares it once per kernel,
// so that a kernel which instantiates the skeleton several times holds one copy)
constexpr int stream_turn_quads(int group) { return group == 8 ? kStreamThreads * 2 : 1; }

template <int G, int T, bool WIDE, int C, typename F>
__device__ __forceinline__ void for_each_output_group(const Conv1dArgs &p, int lead_in, stream_v4i *s_turn, F &&compute)
{
    static_assert(G == 4 || G == 8, "groups of 4 or 8 outputs");
    static_assert(G == 4 || !WIDE, "a window wider than 64 bits feeds a quad only");
    static_assert(C == 1 || C == 2 || C == 4 || C == 8, "container width");
    static_assert(!WIDE || C == 8, "a window wider than 64 bits has 8-bit containers");
    constexpr int LG = G == 4 ? 2 : 3;
    constexpr int STEPS = stream_steps(G);
    constexpr int LINE = 32 / G;                                    // groups per 128-byte line of y
    const int out_len = (int)p.out_len, len = (int)p.len;
    const int ngroups = (out_len + 2 * (G - 1)) / G;
    constexpr int c = C;                                            // the container width (p.c, chosen by the caller)
    constexpr int lc = C == 1 ? 0 : C == 2 ? 1 : C == 4 ? 2 : 3;    // its log2
    const int64_t total_bits = p.total_bytes * 8;
    const char *xbytes = reinterpret_cast<const char *>(p.x);
    typedef uint32_t u32x3_dw __attribute__((ext_vector_type(3), aligned(4)));
    typedef uint32_t u32x4_dw __attribute__((ext_vector_type(4), aligned(4)));
    typedef stream_v4i v4i;                                         // s_turn, G = 8: 2 KB per wave, see the stores below
    auto floor_g = [](int a) { return a >> LG; };                   // floor(a / G) and ceil(a / G) for any sign
    auto ceil_g = [](int a) { return (a + G - 1) >> LG; };

    for (int64_t r = blockIdx.y; r < p.rows; r += gridDim.y) {
        // ---- per row, wave-uniform ----
        // groups are aligned in memory (y_dev itself is 16-byte aligned): the row's first group
        // starts a_off outputs before the row
        const int a_off = (int)((p.y_phase + r * p.out_len) & (G - 1));
        // the groups of a wave start on a 128-byte line of y: the row's group 0 sits `lead` groups
        // into its line, so the lanes are shifted back by that much
        const int lead = (int)(((p.y_phase + r * p.out_len - a_off) >> LG) & (LINE - 1));
        const int64_t row_bit0 = r * p.row_stride_bits;
        const int row_sh = (int)(row_bit0 & 31);                    // bit of the row's first element in its dword
        const uint32_t row_byte = (uint32_t)((row_bit0 >> 5) << 2); // byte offset of that dword in the buffer
        const int64_t room = total_bits - (row_bit0 - row_sh) - (WIDE ? 160 : 128);
        const int bit_limit = room < 0 ? -1 : (room > 0x7fffffff ? 0x7fffffff : (int)room);
        // group q: first output o0 = G q - a_off, first element i0 = o0 + lead_in, window at bit
        // row_sh + i0*c of the row's first dword.  It is interior (window inside the row and the
        // buffer, all G outputs exist) for q_lo <= q <= q_hi:
        const int k_in = lead_in - a_off;                           // i0 = G q + k_in
        int q_lo = ceil_g(-k_in);
        if (q_lo < ceil_g(a_off)) q_lo = ceil_g(a_off);
        if (q_lo < 0) q_lo = 0;
        int q_hi = ngroups - 1;
        if (q_hi > floor_g(len - T - k_in)) q_hi = floor_g(len - T - k_in);
        if (q_hi > floor_g(out_len - G + a_off)) q_hi = floor_g(out_len - G + a_off);
        if (bit_limit < row_sh) {
            q_hi = q_lo - 1;
        } else {
            const int i_max = (bit_limit - row_sh) >> lc;           // largest i0 whose loads stay inside the buffer
            if (q_hi > floor_g(i_max - k_in)) q_hi = floor_g(i_max - k_in);
        }
        const uint32_t q_span = q_hi >= q_lo ? (uint32_t)(q_hi - q_lo) : 0u;
        const bool none = q_hi < q_lo;
        const int kb = row_sh + k_in * c;                           // window bit = (q << (LG + lc)) + kb
        int32_t *yrow = p.y + r * p.out_len;
        char *ybytes = reinterpret_cast<char *>(yrow) - 4 * a_off;  // group q is stored at ybytes + 4 G q

        // ---- per group ----
        const int q_first = (int)(blockIdx.x * (unsigned)(STEPS * kStreamThreads) + threadIdx.x) - lead;
        auto group_of = [&](int st) { return q_first + st * kStreamThreads; };
        bool interior[STEPS];
        uint32_t w0[STEPS], w1[STEPS], w2[STEPS], w3[STEPS], shv[STEPS];
        bool any_edge = false;
        // all window loads of a lane's groups are issued before the first is used; they are
        // unconditional (a group that is not interior reads the buffer's first dwords and ignores them)
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const int q = group_of(s);
            interior[s] = !none && (uint32_t)(q - q_lo) <= q_span;
            any_edge |= !interior[s] && (uint32_t)q < (uint32_t)ngroups;
            const int bit = (int)((uint32_t)q << (LG + lc)) + kb;
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
        // The workgroup's waves meet here, with their loads in flight, and so reach their stores
        // together: the 16 KB of y that a workgroup owns are then written within a short time.  Without
        // the barrier the headline case takes 0.181 instead of 0.174 ms and the 4-bit signed 7-tap
        // case 0.183 instead of 0.176; a barrier ahead of the stores instead measures the same.
        __syncthreads();
        // the loaded dwords are named here, after the last load has been issued and ahead of every
        // branch: the compiler otherwise moves a load into the branch that uses it, where its
        // round trip is waited for alone
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            asm volatile("" : "+v"(w0[s]), "+v"(w1[s]), "+v"(w2[s]));
            if (WIDE) asm volatile("" : "+v"(w3[s]));
        }
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            // every lane runs the arithmetic (a group that is not interior works on the dwords it
            // loaded from the buffer's start and stores nothing): no preset of the outputs and no
            // change of the execution mask around the arithmetic
            int32_t out[G];
            {
                const uint32_t sh = shv[s];
                const uint64_t win = ((uint64_t)funnel_shr(w2[s], w1[s], sh) << 32) | funnel_shr(w1[s], w0[s], sh);
                compute(win, WIDE ? funnel_shr(w3[s], w2[s], sh) : 0u, out);
            }
            // interior: q >= 0, and 4 G q < 2^32 (launcher)
            const uint32_t yoff = (uint32_t)group_of(s) << (LG + 2);
            if (G == 4) {
                if (!interior[s]) continue;
                const v4i v4 = {out[0], out[1], out[2], out[3]};
                __builtin_nontemporal_store(v4, reinterpret_cast<v4i *>(ybytes + yoff));
            } else {
                // A lane's eight outputs are 32 contiguous bytes, but a store instruction moves 16
                // per lane, and the memory pipeline wants the 64 pieces of one instruction side by
                // side.  So the wave's 2 KB pass through its own LDS region: lane l writes quads 2l
                // and 2l+1, reads quads l and 64+l, and each of the two stores covers 1 KB of y.
                // (A wave's LDS instructions execute in order; nothing else touches the region.)
                const v4i lo = {out[0], out[1], out[2], out[3]}, hi = {out[G - 4], out[G - 3], out[G - 2], out[G - 1]};
                if (__builtin_amdgcn_ballot_w64(interior[s]) == ~0ull) { // wave-uniform
                    v4i *mine = s_turn + (threadIdx.x & ~63) * 2;
                    const int lane = threadIdx.x & 63;
                    __builtin_amdgcn_wave_barrier();
                    mine[2 * lane] = lo;
                    mine[2 * lane + 1] = hi;
                    __builtin_amdgcn_wave_barrier();
                    const v4i t0 = mine[lane], t1 = mine[64 + lane];
                    __builtin_amdgcn_wave_barrier();
                    char *wave_y = ybytes + (yoff - 32u * (uint32_t)lane); // lane 0's group
                    __builtin_nontemporal_store(t0, reinterpret_cast<v4i *>(wave_y + 16 * lane));
                    __builtin_nontemporal_store(t1, reinterpret_cast<v4i *>(wave_y + 1024 + 16 * lane));
                } else if (interior[s]) {
                    *reinterpret_cast<v4i *>(ybytes + yoff) = lo;
                    *reinterpret_cast<v4i *>(ybytes + yoff + 16) = hi;
                }
            }
        }
        // groups at the row's ends (and where a load would leave the buffer): the same window from
        // one byte load per element (a container never straddles a byte; an element of the row is
        // inside the buffer), zero outside the row; the same arithmetic; checked element stores.
        // The loads of a window are unconditional (clamped) and independent, so they overlap.
        if (__builtin_amdgcn_ballot_w64(any_edge) != 0) {
            const uint8_t *xb = reinterpret_cast<const uint8_t *>(p.x);
#pragma unroll 1
            for (int s = 0; s < STEPS; ++s) {
                const int q = group_of(s);
                const bool inside = !none && (uint32_t)(q - q_lo) <= q_span;
                const bool edge = !inside && (uint32_t)q < (uint32_t)ngroups;
                if (__builtin_amdgcn_ballot_w64(edge) == 0) continue;   // wave-uniform
                const int o0 = G * q - a_off;
                const int i0 = o0 + lead_in;
                uint32_t e[T];
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    const int i = i0 + t;
                    const bool ok = edge && (uint32_t)i < (uint32_t)len;
                    // bits from the row's first dword fit 32 bits, byte offsets in the buffer too (launcher)
                    const uint32_t rel = (uint32_t)row_sh + (uint32_t)i * (uint32_t)c;
                    const uint32_t v = xb[ok ? row_byte + (rel >> 3) : 0u];
                    e[t] = ok ? (v >> (rel & 7u)) & ((1u << c) - 1u) : 0u;
                }
                uint64_t win = 0;
                uint32_t win_hi = 0;
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    if (t * c < 64)
                        win |= (uint64_t)e[t] << (t * c);
                    else
                        win_hi |= e[t] << (t * c - 64);
                }
                int32_t out[G];
                compute(win, win_hi, out);
                if (edge) {
#pragma unroll
                    for (int u = 0; u < G; ++u)
                        if (o0 + u >= 0 && o0 + u < out_len) yrow[o0 + u] = out[u];
                }
            }
        }
    }
}

} // namespace hikonv
#endif

// Packed DNN-layer kernels (Theorem 3 of the paper): the layer is a sum over input channels
// and kernel rows of 1-D row convolutions, each computed block-wise by packed multiplies;
// block products with the same (co, h, x) are accumulated in the packed domain over M
// (ci, kh) pairs before one split (Section "DNN Convolution Extension").
//
// Mapping: one lane owns one packed block x of one output row (n, ho) and CO_T output
// channels.  Activation words A[chunk][n][ci/4][row][x][ci%4] come pre-packed from k_pack_act
// (one 16-byte load brings the words of four terms); weight words B[co][term] are wave
// uniform: k_conv2d_pipe stages the channel tile's words in LDS once per workgroup and reads
// them back as broadcast 128-bit reads, k_conv2d_packed fetches them with scalar loads.  The
// multiply-accumulate is
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
// are walked in small groups through a table of activation offsets, the loads of the next
// group are issued before the multiplies of the current one, and the term range of a row
// group can be divided among the 2 or 4 waves of a workgroup (partial int32 sums are
// reduced through LDS), which supplies enough waves for layers with few output rows.
// {-1,+1} layers are ordinary signed layers here: their values (0 in the zero padding)
// travel as signed slices.
#ifndef HIKONV_CONV2D_KERNEL_H
#define HIKONV_CONV2D_KERNEL_H

#include "hikonv_device.h"
#include "hikonv_launch.h"

namespace hikonv {

// A[chunk][n][c/4][dp][hp][xi][c%4] = sum_j f[(xi-1)N + j - chunk*K] 2^(S j), f = row hp-pad of depth
// slice dp-pad_d of the image (zero outside it; Eq. I_PRIME / Eq. pad_f0).  Word xi = 0 of
// every row is zero.  A 2-D layer has one depth slice (Dp = 1).  The words of four channels sit side
// by side in a 16-byte cell, so that a lane fetches the words of four terms with one load.
// Ordinary layers: the packed channel c is the source channel and f[i] is its value i; the
// leading horizontal padding is not materialised, it only shifts the index at which an
// output is read (Eq. off).
// Polyphase layers (column stride s packed as s phases): packed channel c = (source channel
// c / s, phase c % s) and f[i] = padded source row at s*i + phase, i.e. source value
// s*i + phase - pad, so that a stride-s row convolution becomes the sum over the phases of
// stride-1 row convolutions with the phase kernels.
// One packed word: chunk ch, image n_img, packed channel c_packed, source depth d and row h
// (both inside the image), word xi > 0.  FMT: the source format (HIKONV_FMT_INT8,
// HIKONV_FMT_BITDENSE or kPackFromAcc), fixed at compile time in the kernels below.
// NV: the plan's N when it is known at compile time (the loops unroll and the loads of a word
// are issued together), 0 = read it from the arguments.
template <int FMT, int NV>
__device__ __forceinline__ uint32_t pack_act_word(const PackActArgs &p, int ch, int64_t n_img, int c_packed, int d, int h,
                                                  int xi)
{
    uint32_t a = 0;
    const int pN = NV ? NV : p.N;
    const int e0 = (xi - 1) * pN - ch * p.Kp;
    if (FMT == kPackFromAcc) {
        // fused epilogue of the producing layer (ReLU, shift, clamp, optional 2x2 max-pool); 2-D, one phase
        const int32_t *src = p.acc + (n_img * p.C + c_packed) * p.acc_H * p.acc_W;
#pragma unroll
        for (int j = 0; j < pN; ++j) {
            const int i = e0 + j;
            if (i < 0 || i >= p.W) continue;
            int32_t v;
            if (p.pool) {
                const int32_t *s0 = src + (int64_t)(2 * h) * p.acc_W + 2 * i;
                v = max(max(s0[0], s0[1]), max(s0[p.acc_W], s0[p.acc_W + 1]));
            } else {
                v = src[(int64_t)h * p.acc_W + i];
            }
            v = min(max(v, 0) >> p.shift, p.qmax);
            a += (uint32_t)v << (p.S * j);
        }
        return a;
    }
    const int csrc = c_packed / p.phases, phase = c_packed - csrc * p.phases;
    const uint8_t *rowp =
        static_cast<const uint8_t *>(p.x) + (((n_img * p.Csrc + csrc) * p.D + d) * p.H + h) * p.row_bytes;
    if (FMT == HIKONV_FMT_BITDENSE && NV > 0 && p.phases == 1 && NV * p.c <= 32) {
        // The word's N containers are consecutive bits of the row: one 32-bit window cut out of
        // two dwords that are loaded unconditionally (a load inside a branch is waited for
        // alone).  Dword indices are clamped into the row (bit-dense rows are whole dwords); a
        // clamped dword only supplies containers of elements outside the row, which are skipped.
        const int lo = e0 < 0 ? -e0 : 0;                     // elements lo .. hi-1 of the word exist
        const int hi = p.W - e0 < NV ? p.W - e0 : NV;
        const int bit0 = e0 * p.c;                           // may be negative: floor division below
        const int last = (int)(p.row_bytes >> 2) - 1;
        const int dw = bit0 >> 5;
        const int d0 = dw < 0 ? 0 : (dw > last ? last : dw), d1 = dw + 1 < 0 ? 0 : (dw + 1 > last ? last : dw + 1);
        const uint32_t *rw = reinterpret_cast<const uint32_t *>(rowp);
        const uint32_t raw = funnel_shr(rw[d1], rw[d0], (uint32_t)bit0 & 31u);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            int32_t v;
            if (p.bipolar)
                v = ((raw >> (j * p.c)) & 1u) ? 1 : -1;
            else
                v = p.a_signed ? __builtin_amdgcn_sbfe((int)raw, j * p.c, p.b) : (int)__builtin_amdgcn_ubfe(raw, j * p.c, p.b);
            if (j >= lo && j < hi) a += (uint32_t)v << (p.S * j);
        }
        return a;
    }
#pragma unroll
    for (int j = 0; j < pN; ++j) {
        const int i = e0 + j; // element of the packed row
        if (i < 0 || i >= p.W) continue;
        const int is = i * p.phases + phase - p.pad_w_mat; // source value
        if (is < 0 || is >= p.Wsrc) continue;
        int32_t v;
        if (FMT == HIKONV_FMT_INT8) {
            const uint8_t byte = rowp[is];
            if (p.bipolar)
                v = (int8_t)byte > 0 ? 1 : -1;
            else
                v = p.a_signed ? __builtin_amdgcn_sbfe((int)byte, 0, p.b) : (int)__builtin_amdgcn_ubfe(byte, 0, p.b);
        } else {
            const int bit = is * p.c;
            const uint32_t w = reinterpret_cast<const uint32_t *>(rowp)[bit >> 5];
            if (p.bipolar)
                v = ((w >> (bit & 31)) & 1u) ? 1 : -1;
            else
                v = p.a_signed ? __builtin_amdgcn_sbfe((int)w, bit & 31, p.b) : (int)__builtin_amdgcn_ubfe(w, bit & 31, p.b);
        }
        a += (uint32_t)v << (p.S * j);
    }
    return a;
}

// the table of activation offsets of the term groups (entry gi, zero beyond the groups):
// gi = ((cq*Kd + kd)*Kh + kh)*chunks + chunk  ->  byte offset 16*(chunk*chunk_stride + ((cq*Dp + kd)*Hp + kh)*Xs)
__device__ __forceinline__ void write_offset_entry(const PackActArgs &p, int gi)
{
    int32_t off = 0;
    if (gi < p.groups) {
        const int ch = gi % p.chunks, kh = (gi / p.chunks) % p.Kh, kd = (gi / (p.chunks * p.Kh)) % p.Kd;
        const int cq = gi / (p.chunks * p.Kh * p.Kd);
        off = (int32_t)(uint32_t)(16 * (ch * p.chunk_stride + (((int64_t)cq * p.Dp + kd) * p.Hp + kh) * p.Xs)); // < 2^32
    }
    p.toff[gi] = off;
}

template <bool WIDE>
struct acc_type {
    typedef uint64_t type;
};
template <>
struct acc_type<false> {
    typedef uint32_t type;
};

// Workgroup -> (row-group block bx, channel tile by).  Workgroups are handed to the eight
// XCDs of the chip in turn (workgroup i runs on XCD i mod 8) and every XCD has its own L2, so
// the tiles are numbered such that one XCD gets a contiguous range of them, channel tile
// fastest: the workgroups that read the same activation rows run on the same XCD, close in
// time, and an XCD's L2 sees only its share of the activations.  Returns false for the
// workgroups that pad the grid to a multiple of 8.
__device__ __forceinline__ bool tile_of_workgroup(const Conv2dArgs &p, int *bx, int *by)
{
    // every quantity here is below 2^31 (the launcher checks the grid), so the divisions are 32-bit
    uint32_t v = blockIdx.x;
    if (p.per_xcd) v = (blockIdx.x & 7u) * (uint32_t)p.per_xcd + (blockIdx.x >> 3);
    if (v >= (uint32_t)p.tiles_x * (uint32_t)p.tiles_y) return false;
    // channel tile fastest: neighbours in time share the activation rows
    const uint32_t x = v / (uint32_t)p.tiles_y;
    const uint32_t y = v - x * (uint32_t)p.tiles_y;
    // the divisions run on the vector ALU; the results are workgroup uniform and are used as scalars
    *bx = __builtin_amdgcn_readfirstlane((int)x);
    *by = __builtin_amdgcn_readfirstlane((int)y);
    return true;
}

// lane -> (output row, packed word index xi); block x = xi - 1
struct LaneMap {
    int n, ho, xi;   // image, output row inside the image (depth slice * Ho2d + row), packed word index
    int64_t in_row;  // packed input row that kernel row 0 of this output row reads
    bool active, halo;
};

__device__ __forceinline__ LaneMap map_lane(const Conv2dArgs &p, int64_t row_group_in, int lane)
{
    // row groups and rows are below 2^31 (the launcher checks both): 32-bit divisions
    const uint32_t row_group = (uint32_t)row_group_in;
    LaneMap m;
    uint32_t row;
    if (p.segs == 0) { // several whole rows per wave
        const int rw = (int)((uint32_t)lane / (uint32_t)p.Xs);
        m.xi = lane - rw * p.Xs;
        row = row_group * (uint32_t)p.rows_per_wave + (uint32_t)rw;
        m.active = rw < p.rows_per_wave && row < (uint32_t)p.wave_rows;
        m.halo = m.xi == 0;
    } else { // one 63-block segment of a long row per wave
        row = row_group / (uint32_t)p.segs;
        const int seg = (int)(row_group - row * (uint32_t)p.segs);
        m.xi = seg * 63 + lane;
        m.active = row < (uint32_t)p.wave_rows && m.xi < p.Xs;
        m.halo = lane == 0;
    }
    if (!m.active) {
        row = 0;
        m.xi = 0;
    }
    m.n = (int)(row / (uint32_t)p.Ho);
    m.ho = (int)(row - (uint32_t)m.n * (uint32_t)p.Ho);
    // first packed input row of this output row: image, output depth, output row inside the depth slice
    const int d = (int)((uint32_t)m.ho / (uint32_t)p.Ho2d);
    m.in_row = (int64_t)m.n * p.img_rows + (int64_t)d * p.d_rows + (int64_t)(m.ho - d * p.Ho2d) * p.stride;
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
            acc_t comb = acc[c];
            if (SN < (WIDE ? 64u : 32u)) { // wave-uniform; one-tap kernels that fill the word have no high part
                if (WIDE) {
                    const uint64_t a64 = (uint64_t)acc[c];
                    comb = (acc_t)(a64 + lane_shr1(ANY_SIGNED ? (uint64_t)((int64_t)a64 >> SN) : a64 >> SN));
                } else {
                    const uint32_t a32 = (uint32_t)acc[c];
                    comb = (acc_t)(a32 + lane_shr1(ANY_SIGNED ? (uint32_t)((int32_t)a32 >> SN) : a32 >> SN));
                }
            }
#pragma unroll
            for (int j = 0; j < N; ++j) out[c][j] += (int32_t)((uint32_t)(comb >> (S * j)) & fmask);
            acc[c] = bias;
        }
    }
};

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

// Output stores of a wave: raw buffer stores whose per-lane byte offset is either the
// output's offset inside the wave's window of y or, for a lane or field that has no output
// there (halo block, column outside the row, column dropped by the stride), an offset beyond
// the buffer's size -- the hardware drops out-of-range buffer stores.  The offsets are
// computed once per wave and serve every channel: the window of channel c starts c channel
// planes further on.  The N own fields of a lane are consecutive output columns (unit
// column stride), so a lane that stores all fields of a group of up to four does it with one
// 8/12/16-byte store (dword aligned: global memory takes that); lanes at the ends of a row,
// the high fields and strided layers use one store per field.  The window starts at the
// output row of the wave's first lane; the launcher sets fast_store only when every lane's
// offset from there is below 2^31 bytes.
constexpr uint32_t kNoStore = 0x80000000u; // = size given to the buffer: never in range
typedef int32_t i32x2 __attribute__((ext_vector_type(2)));
typedef int32_t i32x3 __attribute__((ext_vector_type(3)));

template <int N, int HI>
struct OutputStores {
    static constexpr int NF = N + HI;
    static constexpr int NV = (N + 3) / 4; // groups of up to four own fields
    uint32_t vgroup[NV]; // offset of the group's first field where the lane stores the whole group, else kNoStore
    uint32_t vone[NF];   // offset of field j where the lane stores it by itself, else kNoStore
    bool singles;        // the lane has such a field
    uint64_t base;       // wave-uniform: address of (first lane's image, channel co0, first lane's row)
    int64_t chan_bytes;  // wave-uniform: bytes between channel planes

    // n, ho, x: the lane's image, output row and block; flag[j]: the lane writes field j at
    // all; fields are consecutive stride-1 columns starting at x*N - off
    __device__ __forceinline__ void init(const Conv2dArgs &p, int n, int ho, int x, int co0, const bool (&flag)[NF])
    {
        const int n0 = __builtin_amdgcn_readfirstlane(n), ho0 = __builtin_amdgcn_readfirstlane(ho);
        chan_bytes = (int64_t)p.Ho * p.Wo * 4;
        base = reinterpret_cast<uint64_t>(p.y) + (uint64_t)((((int64_t)n0 * p.Co + co0) * p.Ho + ho0) * p.Wo * 4);
        // rows between the lane's output row and the window's first row (lanes are in row order)
        const uint32_t drow = (uint32_t)(n - n0) * (uint32_t)p.Co * (uint32_t)p.Ho + (uint32_t)(ho - ho0); // wraps only on lanes that store nothing
        const uint32_t row_byte = drow * (uint32_t)p.Wo * 4u;
        bool ok[NF];
        uint32_t off[NF];
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            const int w1 = x * p.N + j - p.off; // stride-1 output column
            ok[j] = flag[j] && w1 >= 0 && w1 < p.Wo1;
            uint32_t wo = (uint32_t)w1;
            if (p.stride_w != 1) { // wave-uniform
                wo = (uint32_t)w1 / (uint32_t)p.stride_w;
                ok[j] = ok[j] && wo * (uint32_t)p.stride_w == (uint32_t)w1;
            }
            off[j] = row_byte + wo * 4u;
        }
        singles = false;
#pragma unroll
        for (int g = 0; g < NV; ++g) {
            bool whole = p.stride_w == 1;
#pragma unroll
            for (int j = 4 * g; j < 4 * g + 4 && j < N; ++j) whole = whole && ok[j];
            vgroup[g] = whole ? off[4 * g] : kNoStore;
#pragma unroll
            for (int j = 4 * g; j < 4 * g + 4 && j < N; ++j) {
                const bool one = ok[j] && !whole;
                vone[j] = one ? off[j] : kNoStore;
                singles = singles || one;
            }
        }
#pragma unroll
        for (int j = N; j < NF; ++j) {
            vone[j] = ok[j] ? off[j] : kNoStore;
            singles = singles || ok[j];
        }
    }

    __device__ __forceinline__ i32x4 channel(int c) const
    {
        const uint64_t b = base + (uint64_t)(c * chan_bytes);
        i32x4 r;
        r.x = __builtin_amdgcn_readfirstlane((int32_t)(uint32_t)b);
        r.y = __builtin_amdgcn_readfirstlane((int32_t)(uint32_t)((b >> 32) & 0xffffu));
        r.z = (int32_t)kNoStore; // size in bytes (no stride): every real offset is below it
        r.w = 0x00020000;        // raw 32-bit data
        return r;
    }

    // the NF values of channel c (tile-relative) of this lane
    __device__ __forceinline__ void store_channel(int c, const int32_t (&v)[NF]) const
    {
        const i32x4 window = channel(c);
#pragma unroll
        for (int g = 0; g < NV; ++g) {
            constexpr int kFull = 4;
            const int width = N - 4 * g < kFull ? N - 4 * g : kFull; // compile-time after unrolling
            if (width == 4) {
                const i32x4 d = {v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};
                asm volatile("buffer_store_dwordx4 %0, %1, %2, 0 offen" : : "v"(d), "v"(vgroup[g]), "s"(window) : "memory");
            } else if (width == 3) {
                const i32x3 d = {v[4 * g], v[4 * g + 1], v[4 * g + 2]};
                asm volatile("buffer_store_dwordx3 %0, %1, %2, 0 offen" : : "v"(d), "v"(vgroup[g]), "s"(window) : "memory");
            } else if (width == 2) {
                const i32x2 d = {v[4 * g], v[4 * g + 1]};
                asm volatile("buffer_store_dwordx2 %0, %1, %2, 0 offen" : : "v"(d), "v"(vgroup[g]), "s"(window) : "memory");
            } else {
                asm volatile("buffer_store_dword %0, %1, %2, 0 offen" : : "v"(v[4 * g]), "v"(vgroup[g]), "s"(window) : "memory");
            }
        }
        if (singles) { // few lanes: ends of rows, high fields; all lanes of a strided layer
#pragma unroll
            for (int j = 0; j < NF; ++j)
                asm volatile("buffer_store_dword %0, %1, %2, 0 offen" : : "v"(v[j]), "v"(vone[j]), "s"(window) : "memory");
        }
    }
};

// Stores channels c_begin .. c_end-1 of the tile (out - unbias).  Every lane of the wave calls it.
template <int N, int CO_T>
__device__ __forceinline__ void store_outputs(const Conv2dArgs &p, const LaneMap &m, int co0, const int32_t (&out)[CO_T][N],
                                              int32_t unbias, int c_begin, int c_end)
{
    if (p.fast_store) { // wave-uniform
        bool flag[N];
#pragma unroll
        for (int j = 0; j < N; ++j) flag[j] = m.active && !m.halo;
        OutputStores<N, 0> os;
        os.init(p, m.n, m.ho, m.xi - 1, co0, flag);
#pragma unroll
        for (int c = 0; c < CO_T; ++c) {
            if (c < c_begin || c >= c_end || co0 + c >= p.Co) continue; // wave-uniform
            int32_t v[N];
#pragma unroll
            for (int j = 0; j < N; ++j) v[j] = out[c][j] - unbias;
            os.store_channel(c, v);
        }
        return;
    }
    // windows of 2^31 bytes or more: plain stores with 64-bit addresses
    if (!m.active || m.halo) return;
    const int x = m.xi - 1;
#pragma unroll
    for (int c = 0; c < CO_T; ++c) {
        if (c < c_begin || c >= c_end || co0 + c >= p.Co) continue;
        int32_t *yrow = p.y + (((int64_t)m.n * p.Co + co0 + c) * p.Ho + m.ho) * p.Wo;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const int w1 = x * N + j - p.off; // stride-1 output column
            if (w1 >= 0 && w1 < p.Wo1 && (p.stride_w == 1 || w1 % p.stride_w == 0)) {
                const int wo = p.stride_w == 1 ? w1 : w1 / p.stride_w;
                yrow[wo] = out[c][j] - unbias;
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
    int bx, by;
    if (!tile_of_workgroup(p, &bx, &by)) return; // workgroup-uniform, no barrier in this kernel
    const int64_t wave = (int64_t)bx * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const LaneMap m = map_lane(p, wave, lane);
    const int co0 = by * CO_T;
    const char *a_base = reinterpret_cast<const char *>(apk) + (m.in_row * p.Xs + m.xi) * 16; // this lane's 16-byte cells
    const uint32_t *w_ptr = wp + ((int64_t)(p.cog0 + co0 / 8) * p.terms_pad) * 8 + (co0 & 7);

    SplitState<N, CO_T, ANY_SIGNED, WIDE> st;
    st.init(p.S);
    int since = 0, nsplit = 0;
    // term groups in the order of the offset table: channel quad, kernel row (depth x height), chunk;
    // one 16-byte load brings the activation words of the group's four channels
    for (int gi = 0; gi < p.terms / 4; ++gi) {
        const uint4 q = *reinterpret_cast<const uint4 *>(a_base + (uint32_t)p.toff[gi]);
        const uint32_t a4[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int c = 0; c < CO_T; ++c) st.mad(c, a4[u], w_ptr[c]);
            w_ptr += 8;
            if (++since == p.split_terms_any) {
                asm volatile("" ::: "memory"); // keep the split out of the multiply block (no speculation)
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
    store_outputs<N, CO_T>(p, m, co0, st.out, ANY_SIGNED ? nsplit * (1 << (p.S - 1)) : 0, 0, CO_T);
}


constexpr int kTermTile = 1536; // terms whose weights are staged in LDS at a time (54 KB + offsets at most)

template <int N, int CO_T, bool ANY_SIGNED, bool WIDE>
__global__ __launch_bounds__(256) void k_conv2d_pipe(Conv2dArgs p)
{
    constexpr int U = kTermGroup;
    static_assert(U == 4, "a term group is the four channels of a quad");
    constexpr int CE = CO_T;
    // LDS: weight words of the current term tile [tile][CO_T], the activation offsets of its
    // term groups [tile / U + 1]; reused at the end for the slice reduction
    extern __shared__ __attribute__((aligned(16))) uint32_t s_mem[];

    const uint32_t *__restrict__ apk = p.apk;
    const uint32_t *__restrict__ wp = p.wp;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ks = wave % p.ksplit;                  // which slice of every term tile
    int bx, by;
    if (!tile_of_workgroup(p, &bx, &by)) return; // workgroup-uniform, before any barrier
    const int64_t row_group = (int64_t)bx * (4 / p.ksplit) + wave / p.ksplit;
    const LaneMap m = map_lane(p, row_group, lane);
    const int co0 = by * CO_T;
    // byte offset of this lane's 16-byte cell inside a term group's activation row (< 2^32, host check)
    const uint32_t lane_byte = (uint32_t)((m.in_row * p.Xs + m.xi) * 16);
    const uint32_t *w_tile = wp + ((int64_t)(p.cog0 + co0 / 8) * p.terms_pad) * 8 + (co0 & 7);

    const int tile_cap = p.terms_pad < kTermTile ? p.terms_pad : kTermTile;
    uint32_t *s_w = s_mem;                                   // [tile_cap][CO_T]
    int32_t *s_off = reinterpret_cast<int32_t *>(s_w + tile_cap * CO_T); // [tile_cap / U + 1], one per term group

    SplitState<N, CE, ANY_SIGNED, WIDE> st;
    st.init(p.S);
    int since = 0, nsplit = 0;

    for (int tile0 = 0; tile0 < p.terms_pad; tile0 += tile_cap) {
        const int tile_n = p.terms_pad - tile0 < tile_cap ? p.terms_pad - tile0 : tile_cap; // multiple of U
        if (tile0 > 0) __syncthreads();
        // stage the tile: weight words (8 per term are contiguous in memory and zero beyond the
        // real terms) and the activation offsets of the terms, with 128-bit copies issued in
        // batches so that a thread waits for memory once per batch
        if (CO_T == 8) {
            const int total = tile_n * 2; // uint4 units
            const uint4 *src = reinterpret_cast<const uint4 *>(w_tile + (int64_t)tile0 * 8);
            uint4 *dst = reinterpret_cast<uint4 *>(s_w);
            for (int i = tid; i < total; i += 1024) {
                const int i1 = i + 256, i2 = i + 512, i3 = i + 768;
                const uint4 v0 = src[i];
                const uint4 v1 = src[i1 < total ? i1 : i];
                const uint4 v2 = src[i2 < total ? i2 : i];
                const uint4 v3 = src[i3 < total ? i3 : i];
                dst[i] = v0;
                if (i1 < total) dst[i1] = v1;
                if (i2 < total) dst[i2] = v2;
                if (i3 < total) dst[i3] = v3;
            }
        } else {
            const int total = tile_n * CO_T;
            for (int i = tid; i < total; i += 256) {
                const int t = i / CO_T, c = i - t * CO_T;
                s_w[i] = w_tile[(int64_t)(tile0 + t) * 8 + c];
            }
        }
        for (int t = tid; t < tile_n / U + 1; t += 256) s_off[t] = p.toff[tile0 / U + t];
        __syncthreads();

        // this wave's slice of the tile, in groups of U terms, four register buffers for the
        // activation words: the next groups' loads are in flight during the multiplies
        const int slice = ((tile_n / U + p.ksplit - 1) / p.ksplit) * U;
        const int t_begin = ks * slice;
        int t_end = t_begin + slice;
        if (t_end > tile_n) t_end = tile_n;
        if (t_begin >= t_end) continue; // wave-uniform; barriers are outside this part

        uint32_t a0[U], a1[U], a2[U], a3[U];
        auto request = [&](uint32_t (&a)[U], int t) {
            // the words of the group's four channels sit side by side: one 16-byte load
            // (uniform base + 32-bit lane offset: one VALU add)
            const uint4 q = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(apk) +
                                                             (uint32_t)(lane_byte + (uint32_t)s_off[t / U]));
            a[0] = q.x;
            a[1] = q.y;
            a[2] = q.z;
            a[3] = q.w;
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
#pragma unroll
                for (int c = 0; c < CE; ++c) st.mad(c, a[u], w[c]);
            }
            since += U;
            if (since >= p.split_terms) { // split_terms is a multiple of U
                asm volatile("" ::: "memory"); // keep the split out of the multiply block (no speculation)
                st.split();
                since = 0;
                ++nsplit;
            }
        };

        // three groups in flight while one is multiplied: on small layers the loop is a chain
        // of memory round trips, and this makes it a quarter as long
        const int t_last = t_end - U;
        auto clamp = [&](int t) { return t < t_end ? t : t_last; }; // past the end: re-read the last group
        request(a0, t_begin);
        request(a1, clamp(t_begin + U));
        request(a2, clamp(t_begin + 2 * U));
        for (int t = t_begin; t < t_end; t += 4 * U) {
            request(a3, clamp(t + 3 * U));
            multiply(a0, t);
            if (t + U >= t_end) break;
            request(a0, clamp(t + 4 * U));
            multiply(a1, t + U);
            if (t + 2 * U >= t_end) break;
            request(a1, clamp(t + 5 * U));
            multiply(a2, t + 2 * U);
            if (t + 3 * U >= t_end) break;
            request(a2, clamp(t + 6 * U));
            multiply(a3, t + 3 * U);
        }
    }
    if (since) {
        st.split();
        ++nsplit;
    }
    const int32_t unbias = ANY_SIGNED ? nsplit * (1 << (p.S - 1)) : 0;

    // Epilogue.  With ksplit > 1 the slices' partial sums meet in LDS and every wave of the
    // row group finishes an equal share of the channels (sum, {-1,+1} correction, store).
    int c_begin = 0, c_end = CO_T;
    if (p.ksplit > 1) {
        int32_t *s_red = reinterpret_cast<int32_t *>(s_mem); // [4 waves][CE*N][64]
        __syncthreads();                                      // the weight tile is no longer read
        int32_t *dst = s_red + (wave * CE * N) * 64 + lane;
#pragma unroll
        for (int c = 0; c < CE; ++c)
#pragma unroll
            for (int j = 0; j < N; ++j) dst[(c * N + j) * 64] = st.out[c][j] - unbias;
        __syncthreads();
        c_begin = ks * CO_T / p.ksplit;
        c_end = (ks + 1) * CO_T / p.ksplit;
        const int w0 = wave - ks; // first wave of this row group
#pragma unroll
        for (int c = 0; c < CE; ++c) {
            if (!(c >= c_begin && c < c_end)) continue;
#pragma unroll
            for (int j = 0; j < N; ++j) {
                int32_t v = 0;
                for (int k2 = 0; k2 < p.ksplit; ++k2) v += s_red[((w0 + k2) * CE * N + c * N + j) * 64 + lane];
                st.out[c][j] = v + unbias; // store_outputs subtracts it again
            }
        }
    }
    store_outputs<N, CO_T>(p, m, co0, st.out, unbias, c_begin, c_end);
}

// dynamic LDS bytes of k_conv2d_pipe
inline size_t conv2d_pipe_lds(const Conv2dArgs &a, int co_tile, int n)
{
    const int ce = co_tile;
    const size_t tile_cap = a.terms_pad < kTermTile ? a.terms_pad : kTermTile;
    const size_t stage = (tile_cap * co_tile + tile_cap / kTermGroup + 4) * 4;
    const size_t reduce = a.ksplit > 1 ? (size_t)4 * ce * n * 64 * 4 : 0;
    return stage > reduce ? stage : reduce;
}

template <int N, bool ANY_SIGNED, bool WIDE>
inline void launch_conv2d_n(const Conv2dArgs &a, int co_tile, dim3 g, hipStream_t stream)
{
    if (a.pipelined) {
        const size_t lds = conv2d_pipe_lds(a, co_tile, N);
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
    default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

hipError_t launch_conv2d_wide(const Conv2dArgs &a, bool any_signed, int co_tile, dim3 g, hipStream_t stream);
hipError_t launch_conv2d_narrow(const Conv2dArgs &a, bool any_signed, int co_tile, dim3 g, hipStream_t stream);

} // namespace hikonv
#endif

// Packed DNN-layer kernel with the weight words in scalar registers (Theorem 3 of the paper;
// products accumulated in the packed domain before a split, Section "DNN Convolution
// Extension").
//
// One lane owns one packed block x of one output row and eight output channels.  The B
// words of a term (ci, kh, chunk) are the same for every lane of a wave, so they are read
// with scalar loads (32 bytes per term) and a packed multiply-accumulate is one
// v_mad_u64_u32 / v_mad_i64_i32 with an SGPR operand; the A words of four terms (the channels of
// a quad) are one 16-byte load per lane from the packed activation rows.  No LDS traffic in
// the term loop.
//
// Software pipeline over groups of U terms:
//   scalar loads of B for group g+1 and of the activation offset for group g+4,
//   one 16-byte buffer load of A (the four channels of a quad) for group g+3 (they return in order, so three groups can be in flight;
//   the address is resource + lane offset + a scalar term offset: no address arithmetic),
//   multiply-accumulates of group g.
// Scalar loads return out of order, so the only safe wait is "all of them"; it sits at the
// top of a stage, before the next scalar loads are issued, and therefore never waits for
// loads younger than one stage.
//
// Split (Eq. output_split in bias form): the accumulated word holds N + HI segments
// (HI = taps per B word - 1).  Every segment but the top one starts from a bias of 2^(S-1)
// when data are signed, so each is read as a non-negative field; the top segment is read
// with a plain (arithmetic) shift and may be narrower than S bits.  All N + HI fields go to
// int32 registers of the lane; the overlap-add of Theorem 2 (segments N.. of block x-1 land
// on segments 0.. of block x) happens once, in int32, after the last split, through a DPP
// move from the previous lane.  A segment therefore collects at most M*min(K,N) products,
// as in the paper's guard-bit rule for this case.
//
// Lane mapping: rows of at most 64 blocks: several whole rows per wave, lanes only for the
// blocks that hold input values; the last block of a row stores its high segments itself.
// Longer rows: segments of 63 blocks whose lane 0 recomputes the preceding block.
//
// The term range of a row group can be divided over the 2 or 4 waves of the workgroup;
// partial int32 sums meet in LDS (two passes over half of the channels each, to keep the
// buffer small) and every wave finishes an equal share of the channels.
#ifndef HIKONV_CONV2D_SREG_H
#define HIKONV_CONV2D_SREG_H

#include "hikonv_conv2d_kernel.h"

namespace hikonv {

struct LaneMapS {
    int n, ho, xi; // image, output row inside the image (depth slice * Ho2d + row), packed word index
    int64_t in_row; // packed input row that kernel row 0 of this output row reads
    bool active;   // lane stands for a block of an existing output row
    bool recv;     // the previous lane holds the preceding block of the same row
    bool store;    // lane writes its own N outputs
    bool store_hi; // lane also writes its high segments (no lane owns the following block)
};

__device__ __forceinline__ LaneMapS map_lane_sreg(const Conv2dArgs &p, int64_t row_group_in, int lane)
{
    // row groups and rows are below 2^31 (the launcher checks both): 32-bit divisions
    const uint32_t row_group = (uint32_t)row_group_in;
    LaneMapS m;
    uint32_t row;
    if (p.segs == 0) {
        const int rw = (int)((uint32_t)lane / (uint32_t)p.Lr);
        const int l = lane - rw * p.Lr;
        m.xi = l + 1;
        row = row_group * (uint32_t)p.rows_per_wave + (uint32_t)rw;
        m.active = rw < p.rows_per_wave && row < (uint32_t)p.wave_rows;
        m.recv = l != 0;
        m.store = m.active;
        m.store_hi = m.active && l == p.Lr - 1;
    } else {
        row = row_group / (uint32_t)p.segs;
        const int seg = (int)(row_group - row * (uint32_t)p.segs);
        m.xi = seg * 63 + lane;
        m.active = row < (uint32_t)p.wave_rows && m.xi < p.Xs;
        m.recv = lane != 0;
        m.store = m.active && lane != 0;
        m.store_hi = false;
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

// Overlap-add with the previous lane's high segments, bounds and stride handling, store of
// one output channel.  v: N own fields then HI high fields.
template <int N, int HI>
__device__ __forceinline__ void finish_channel(const Conv2dArgs &p, const LaneMapS &m, int co, const int32_t (&v)[N + HI])
{
    int32_t o[N];
#pragma unroll
    for (int j = 0; j < N; ++j) o[j] = v[j];
#pragma unroll
    for (int j = 0; j < HI; ++j) {
        const int32_t r = (int32_t)lane_shr1((uint32_t)v[N + j]); // every lane takes part in the move
        if (j < N) o[j] += m.recv ? r : 0;
    }
    if (co >= p.Co) return;
    int32_t *yrow = p.y + (((int64_t)m.n * p.Co + co) * p.Ho + m.ho) * p.Wo;
    const int x = m.xi - 1;
#pragma unroll
    for (int j = 0; j < N + HI; ++j) {
        const bool own = j < N;
        if (!(own ? m.store : m.store_hi)) continue;
        const int w1 = x * N + j - p.off; // stride-1 output column
        if (w1 >= 0 && w1 < p.Wo1 && (p.stride_w == 1 || w1 % p.stride_w == 0)) {
            const int wo = p.stride_w == 1 ? w1 : w1 / p.stride_w;
            yrow[wo] = own ? o[j] : v[j];
        }
    }
}

// The same through precomputed buffer-store offsets (see OutputStores): no branch, no
// address arithmetic per channel.  c = channel inside the tile.
template <int N, int HI>
__device__ __forceinline__ void finish_channel_fast(const OutputStores<N, HI> &os, bool recv, int c,
                                                    const int32_t (&v)[N + HI])
{
    int32_t o[N + HI];
#pragma unroll
    for (int j = 0; j < N + HI; ++j) o[j] = v[j];
#pragma unroll
    for (int j = 0; j < HI; ++j) {
        const int32_t r = (int32_t)lane_shr1((uint32_t)v[N + j]); // every lane takes part in the move
        if (j < N) o[j] += recv ? r : 0;
    }
    os.store_channel(c, o);
}

typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Scalar loads and the packed multiply-accumulate are written as instructions: the B words
// must stay in SGPRs, the four products of a group must chain on the accumulator (no
// re-association into a separate sum), and the wait for the scalar loads must sit where the
// pipeline wants it.  Every value loaded by sload_* is undefined until the next
// wait_scalar_loads that names it; it is not read, copied or carried over a loop edge before.
template <int BYTE_OFFSET>
__device__ __forceinline__ void sload_x8(u32x8 &dst, const void *uniform_ptr)
{
    asm volatile("s_load_dwordx8 %0, %1, %2" : "=&s"(dst) : "s"(uniform_ptr), "n"(BYTE_OFFSET));
}
template <int BYTE_OFFSET>
__device__ __forceinline__ void sload_x1(int32_t &dst, const void *uniform_ptr)
{
    asm volatile("s_load_dword %0, %1, %2" : "=&s"(dst) : "s"(uniform_ptr), "n"(BYTE_OFFSET));
}
template <int BYTE_OFFSET>
__device__ __forceinline__ void sload_x4(i32x4 &dst, const void *uniform_ptr)
{
    asm volatile("s_load_dwordx4 %0, %1, %2" : "=&s"(dst) : "s"(uniform_ptr), "n"(BYTE_OFFSET));
}
__device__ __forceinline__ void wait_scalar_loads(u32x8 (&b)[4], i32x4 &o4)
{
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(b[0]), "+s"(b[1]), "+s"(b[2]), "+s"(b[3]), "+s"(o4));
}
__device__ __forceinline__ void wait_scalar_loads(u32x8 (&b)[4], int32_t &o)
{
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(b[0]), "+s"(b[1]), "+s"(b[2]), "+s"(b[3]), "+s"(o));
}

// Keeps the multiply-accumulates of a stage behind the loads issued at its top: the (empty)
// statement is ordered after those loads and the first accumulator passes through it.
__device__ __forceinline__ void pin_before_multiply(uint64_t &acc0) { asm volatile("" : "+v"(acc0)); }

// acc += a * b with b in a scalar register: v_mad_u64_u32 / v_mad_i64_i32 (Theorem 1's
// multiply fused with the accumulation of products before a split)
template <bool SIGNED>
__device__ __forceinline__ void mad_sreg(uint64_t &acc, uint32_t a, uint32_t b_uniform)
{
    acc = mad_wide<SIGNED>(a, b_uniform, acc);
    asm("" : "+v"(acc)); // opaque: the products of a group chain on the accumulator, no separate sum
}

// 2^(S-1) in every segment but the top one
template <int NF>
__device__ __forceinline__ uint64_t field_bias(int S)
{
    uint64_t bias = 0;
#pragma unroll
    for (int j = 0; j < NF - 1; ++j) bias += (uint64_t)1 << (S * j + S - 1);
    return bias;
}

template <int N, int HI, bool ANY_SIGNED>
__global__ __launch_bounds__(256) void k_conv2d_sreg(Conv2dArgs p)
{
    constexpr int U = kTermGroup;
    constexpr int CO_T = 8;
    constexpr int CE = CO_T;
    constexpr int NF = N + HI;
    static_assert(U == 4, "a term group is the four channels of a quad");
    extern __shared__ __attribute__((aligned(16))) int32_t s_red[]; // [4 waves][4*NF][64]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ks = wave % p.ksplit; // which slice of the term range
    int bx, by;
    if (!tile_of_workgroup(p, &bx, &by)) return; // workgroup-uniform, before any barrier
    const int64_t row_group = (int64_t)bx * (4 / p.ksplit) + wave / p.ksplit;
    LaneMapS m = map_lane_sreg(p, row_group, lane);
    // the lane's flags travel through the term loop as bits of one vector register, not as lane masks in
    // scalar registers (which the loop needs for the weight words)
    uint32_t lane_flags = (m.recv ? 1u : 0u) | (m.store ? 2u : 0u) | (m.store_hi ? 4u : 0u);
    asm volatile("" : "+v"(lane_flags));
    const int co0 = by * CO_T;
    // byte offset of this lane's 16-byte cell inside a group's activation row (< 2^32, host check)
    const uint32_t lane_byte = (uint32_t)((m.in_row * p.Xs + m.xi) * 16);
    // weight rows of this channel tile: 32 bytes per term
    const char *wrow = reinterpret_cast<const char *>(p.wp) + (int64_t)(p.cog0 + by) * p.terms_pad * 32;
    const char *trow = reinterpret_cast<const char *>(p.toff); // 4 bytes per term group

    const int S = p.S;
    const uint64_t bias = ANY_SIGNED ? field_bias<NF>(S) : 0;
    uint64_t acc[CE];
    int32_t out[CE][NF];
#pragma unroll
    for (int c = 0; c < CE; ++c) {
        acc[c] = bias;
#pragma unroll
        for (int j = 0; j < NF; ++j) out[c][j] = 0;
    }
    int since = 0, nsplit = 0;

    auto split = [&]() {
        // shift amounts and masks are recomputed here from an opaque copy of S so that they do
        // not occupy scalar registers across the term loop
        int Sl = S;
        asm volatile("" : "+s"(Sl));
        const uint32_t fm = (1u << Sl) - 1u;
#pragma unroll
        for (int c = 0; c < CE; ++c) {
            const uint64_t a = acc[c];
#pragma unroll
            for (int j = 0; j < NF - 1; ++j) out[c][j] += (int32_t)((uint32_t)(a >> (Sl * j)) & fm);
            out[c][NF - 1] += ANY_SIGNED ? (int32_t)((int64_t)a >> (Sl * (NF - 1))) : (int32_t)(uint32_t)(a >> (Sl * (NF - 1)));
            acc[c] = ANY_SIGNED ? field_bias<NF>(Sl) : 0;
        }
        since = 0;
        ++nsplit;
    };

    // this wave's slice of the term groups
    const int groups = p.terms_pad / U;
    const int per = (groups + p.ksplit - 1) / p.ksplit;
    const int g_begin = ks * per;
    int g_end = g_begin + per;
    if (g_end > groups) g_end = groups;

    if (g_begin < g_end) { // wave-uniform; barriers are outside this part
        // Two pointers walk the weight rows (128 bytes per group) and the offset table (4 bytes
        // per group); the groups of a stage are reached through immediate offsets, so a pair of
        // stages costs two scalar pointer updates.  The loads run up to two groups past the
        // wave's range: the weight buffer and the offset table are padded for that.
        u32x8 b0[U], b1[U];
        int32_t o; // byte offset of the next group's activation cells; refilled right after the load that reads it
        u32x4 a0, a1, a2, a3; // activation words of four groups in flight (one channel quad each)
        // Buffer loads: address = packed activations + lane offset (VGPR) + group offset (SGPR,
        // straight from the table), so the 16-byte load that brings the four words of a group
        // costs no VALU or SALU instruction.  They are written as instructions because three
        // groups stay in flight across loop iterations and the wait for the oldest one is a
        // count of younger loads (buffer loads return in order): a value loaded here is
        // undefined until a wait_a that names it, and every buffer stays named until the drain
        // after the loop.
        i32x4 arsrc; // buffer resource: base, no stride, size in bytes, raw 32-bit data
        {
            const uint64_t base = reinterpret_cast<uint64_t>(p.apk);
            arsrc.x = (int32_t)(uint32_t)base;
            arsrc.y = (int32_t)(uint32_t)((base >> 32) & 0xffffu);
            arsrc.z = (int32_t)p.apk_bytes;
            arsrc.w = 0x00020000;
        }
        auto load_a = [&](u32x4 &a, const int32_t &o) {
            asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "=v"(a) : "v"(lane_byte), "s"(arsrc), "s"(o));
        };
        // the group loaded three stages ago has arrived once at most 3 younger loads are pending
        auto wait_a = [&](u32x4 &a) { asm volatile("s_waitcnt vmcnt(3)" : "+v"(a)); };
        auto multiply = [&](const u32x4 &a4, const u32x8 (&b)[U]) {
            const uint32_t a[U] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
            for (int u = 0; u < U; ++u) {
                mad_sreg<ANY_SIGNED>(acc[0], a[u], b[u].s0);
                mad_sreg<ANY_SIGNED>(acc[1], a[u], b[u].s1);
                mad_sreg<ANY_SIGNED>(acc[2], a[u], b[u].s2);
                mad_sreg<ANY_SIGNED>(acc[3], a[u], b[u].s3);
                mad_sreg<ANY_SIGNED>(acc[4], a[u], b[u].s4);
                mad_sreg<ANY_SIGNED>(acc[5], a[u], b[u].s5);
                mad_sreg<ANY_SIGNED>(acc[6], a[u], b[u].s6);
                mad_sreg<ANY_SIGNED>(acc[7], a[u], b[u].s7);
            }
            since += U;
            if (since >= p.split_terms) split(); // split_terms is a multiple of U
        };

        const char *bp = wrow + (int64_t)g_begin * (U * 32); // weights of the group the next stage multiplies
        const char *tp = trow + (int64_t)g_begin * 4;        // its activation offset
        // prologue: B of the first group and the offsets of the first four with one wait, then A of
        // the first three (the table is padded past the wave's range, like the weights)
        i32x4 o4;
        sload_x8<0>(b0[0], bp);
        sload_x8<32>(b0[1], bp);
        sload_x8<64>(b0[2], bp);
        sload_x8<96>(b0[3], bp);
        sload_x4<0>(o4, tp);
        wait_scalar_loads(b0, o4);
        load_a(a0, o4.x);
        load_a(a1, o4.y);
        load_a(a2, o4.z);
        o = o4.w;
        int left = g_end - g_begin; // groups still to multiply
        // One stage, k-th of four, for group g+k: B of g+k+1, A of g+k+3 (o holds its offsets),
        // offsets of g+k+4, then the multiply-accumulates of g+k.
#define HIKONV_SREG_STAGE(k, a_cur, a_new, b_cur, b_new)          \
        sload_x8<(k + 1) * 128 + 0>(b_new[0], bp);                 \
        sload_x8<(k + 1) * 128 + 32>(b_new[1], bp);                \
        sload_x8<(k + 1) * 128 + 64>(b_new[2], bp);                \
        sload_x8<(k + 1) * 128 + 96>(b_new[3], bp);                \
        load_a(a_new, o);                                          \
        sload_x1<(k + 4) * 4>(o, tp);                              \
        wait_a(a_cur);                                             \
        pin_before_multiply(acc[0]);                               \
        multiply(a_cur, b_cur);                                    \
        wait_scalar_loads(b_new, o);                               \
        if (--left == 0) break;
        while (true) {
            HIKONV_SREG_STAGE(0, a0, a3, b0, b1)
            HIKONV_SREG_STAGE(1, a1, a0, b1, b0)
            HIKONV_SREG_STAGE(2, a2, a1, b0, b1)
            HIKONV_SREG_STAGE(3, a3, a2, b1, b0)
            bp += 4 * U * 32;
            tp += 4 * 4;
        }
#undef HIKONV_SREG_STAGE
        // nothing may reuse the buffers' registers while loads into them are in flight
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3));
    }
    if (since) split();

    // remove the biases: every split added 2^(S-1) to each segment but the top one
    if (ANY_SIGNED) {
        const int32_t unbias = nsplit * (1 << (S - 1));
#pragma unroll
        for (int c = 0; c < CE; ++c)
#pragma unroll
            for (int j = 0; j < NF - 1; ++j) out[c][j] -= unbias;
    }

    m.recv = (lane_flags & 1u) != 0;
    m.store = (lane_flags & 2u) != 0;
    m.store_hi = (lane_flags & 4u) != 0;
    OutputStores<N, HI> os;
    if (p.fast_store) { // wave-uniform
        bool flag[NF];
#pragma unroll
        for (int j = 0; j < NF; ++j) flag[j] = j < N ? m.store : m.store_hi;
        // the offsets are wanted here, not in registers across the term loop
        int n_l = m.n, ho_l = m.ho, xi_l = m.xi;
        asm volatile("" : "+v"(n_l), "+v"(ho_l), "+v"(xi_l));
        os.init(p, n_l, ho_l, xi_l - 1, co0, flag);
    }
    auto finish = [&](int c, const int32_t (&v)[NF]) {
        if (co0 + c >= p.Co) return; // wave-uniform
        if (p.fast_store)
            finish_channel_fast<N, HI>(os, m.recv, c, v);
        else
            finish_channel<N, HI>(p, m, co0 + c, v);
    };

    if (p.ksplit == 1) {
#pragma unroll
        for (int c = 0; c < CO_T; ++c) finish(c, out[c]);
        return;
    }

    // ksplit > 1: two passes through LDS, pass 0 = channels 0..3, pass 1 = channels 4..7.
    // Slot s of a pass holds one channel: [wave][s*NF + j][lane].
    constexpr int SLOTS = 4;
    const int w0 = wave - ks; // first wave of this row group
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if (pass) __syncthreads(); // pass 0 has been read
        int32_t *dst = s_red + (wave * SLOTS * NF) * 64 + lane;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int j = 0; j < NF; ++j) dst[(s * NF + j) * 64] = out[pass * 4 + s][j];
        __syncthreads();
        for (int s = ks; s < 4; s += p.ksplit) { // wave-uniform trip count
            int32_t v[NF];
#pragma unroll
            for (int j = 0; j < NF; ++j) v[j] = 0;
#pragma unroll 1
            for (int k2 = 0; k2 < p.ksplit; ++k2) { // one slice's fields at a time: few registers
                const int32_t *src = s_red + ((w0 + k2) * SLOTS * NF + s * NF) * 64 + lane;
#pragma unroll
                for (int j = 0; j < NF; ++j) v[j] += src[j * 64];
            }
            finish(pass * 4 + s, v);
        }
    }
}

inline size_t conv2d_sreg_lds(const Conv2dArgs &a, int n, int hi)
{
    return a.ksplit > 1 ? (size_t)4 * 4 * (n + hi) * 64 * 4 : 0;
}

template <int N, bool ANY_SIGNED>
inline void launch_conv2d_sreg_n(const Conv2dArgs &a, int hi, dim3 g, hipStream_t stream)
{
    const size_t lds = conv2d_sreg_lds(a, N, hi);
    switch (hi) {
    case 0: hipLaunchKernelGGL((k_conv2d_sreg<N, 0, ANY_SIGNED>), g, dim3(256), lds, stream, a); break;
    case 1:
        if constexpr (N >= 1) hipLaunchKernelGGL((k_conv2d_sreg<N, 1, ANY_SIGNED>), g, dim3(256), lds, stream, a);
        break;
    case 2:
        if constexpr (N >= 2) hipLaunchKernelGGL((k_conv2d_sreg<N, 2, ANY_SIGNED>), g, dim3(256), lds, stream, a);
        break;
    default: break;
    }
}

template <bool ANY_SIGNED>
inline hipError_t launch_conv2d_sreg_sw(const Conv2dArgs &a, int hi, dim3 g, hipStream_t stream)
{
    switch (a.N) {
    case 1: launch_conv2d_sreg_n<1, ANY_SIGNED>(a, hi, g, stream); break;
    case 2: launch_conv2d_sreg_n<2, ANY_SIGNED>(a, hi, g, stream); break;
    case 3: launch_conv2d_sreg_n<3, ANY_SIGNED>(a, hi, g, stream); break;
    case 4: launch_conv2d_sreg_n<4, ANY_SIGNED>(a, hi, g, stream); break;
    case 5: launch_conv2d_sreg_n<5, ANY_SIGNED>(a, hi, g, stream); break;
    case 6: launch_conv2d_sreg_n<6, ANY_SIGNED>(a, hi, g, stream); break;
    case 7: launch_conv2d_sreg_n<7, ANY_SIGNED>(a, hi, g, stream); break;
    case 8: launch_conv2d_sreg_n<8, ANY_SIGNED>(a, hi, g, stream); break;
    default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

hipError_t launch_conv2d_sreg_unsigned(const Conv2dArgs &a, int hi, dim3 g, hipStream_t stream);
hipError_t launch_conv2d_sreg_signed(const Conv2dArgs &a, int hi, dim3 g, hipStream_t stream);

} // namespace hikonv
#endif

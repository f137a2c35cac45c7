// Kernels around the packed DNN-layer path: runtime packing of activation rows into A
// words, offline packing of weights into B words, and the unpacked
// one-product-per-multiply baseline.
#include <cstdlib>
#include <type_traits>
#include "hikonv_conv2d_kernel.h"
#include "hikonv_conv2d_sreg.h"

namespace hikonv {
namespace {

// One thread per word.  Grid: x over the 4*Xs words of a packed row (four channels of a quad
// side by side), y = padded row hp (groups of rows_per_block rows when a row is shorter than a block), z = ((chunk*Nimg + n)*Cq + quad)*Dp + dp, so a thread finds
// its coordinates without dividing; block (0,0,0) also writes the offset table.
template <int FMT, int NV>
__global__ __launch_bounds__(256) void k_pack_act_rows(PackActArgs p)
{
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
        for (int gi = threadIdx.x; gi < p.toff_entries; gi += 256) write_offset_entry(p, gi);
    // short rows: a block takes rows_per_block of them (one 32-bit division per thread)
    int t = blockIdx.x * 256 + threadIdx.x, r = 0;
    if (p.rows_per_block > 1) {
        r = (int)((uint32_t)threadIdx.x / (uint32_t)(p.Xs * 4));
        t = threadIdx.x - r * p.Xs * 4;
        if (r >= p.rows_per_block) return;
    }
    if (t >= p.Xs * 4) return;
    const int u = t & 3, xi = t >> 2;
    const int hp = blockIdx.y * p.rows_per_block + r;
    if (hp >= p.Hp) return;
    // workgroup-uniform coordinates
    uint32_t z = blockIdx.z;
    uint32_t q = z / (uint32_t)p.Dp;
    const int dp = (int)(z - q * (uint32_t)p.Dp);
    z = q;
    q = z / (uint32_t)p.Cq;
    const int cq = (int)(z - q * (uint32_t)p.Cq);
    z = q;
    const int ch = (int)(z / (uint32_t)p.Nimg);
    const int n_img = (int)(z - (uint32_t)ch * (uint32_t)p.Nimg);
    const int c_packed = cq * 4 + u;
    const int h = hp - p.pad, d = dp - p.pad_d;
    uint32_t a = 0;
    if (c_packed < p.C && xi > 0 && h >= 0 && h < p.H && d >= 0 && d < p.D)
        a = pack_act_word<FMT, NV>(p, ch, n_img, c_packed, d, h, xi);
    p.apk[(((int64_t)blockIdx.z * p.Hp + hp) * p.Xs + xi) * 4 + u] = a;
}

// The same with a 1-D grid (any size): a thread decodes its word index.
__global__ __launch_bounds__(256) void k_pack_act(PackActArgs p)
{
    const int64_t total = (int64_t)p.chunks * p.Nimg * p.Cq * p.Dp * p.Hp * p.Xs * 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx < p.toff_entries) write_offset_entry(p, (int)idx);
    if (idx >= total) return;
    const int u = (int)(idx & 3); // channel inside the quad
    // fewer than 2^30 words in all (checked by the caller): 32-bit divisions
    uint32_t t = (uint32_t)(idx >> 2);
    uint32_t q = t / (uint32_t)p.Xs;
    const int xi = (int)(t - q * (uint32_t)p.Xs);
    t = q;
    q = t / (uint32_t)p.Hp;
    const int hp = (int)(t - q * (uint32_t)p.Hp);
    t = q;
    q = t / (uint32_t)p.Dp;
    const int dp = (int)(t - q * (uint32_t)p.Dp);
    t = q;
    const uint32_t ncq_all = (uint32_t)p.Nimg * (uint32_t)p.Cq;
    const int ch = (int)(t / ncq_all);
    const uint32_t ncq = t - (uint32_t)ch * ncq_all;
    const int n_img = (int)(ncq / (uint32_t)p.Cq);
    const int c_packed = (int)(ncq - (uint32_t)n_img * (uint32_t)p.Cq) * 4 + u;
    const int h = hp - p.pad, d = dp - p.pad_d;
    uint32_t a = 0;
    if (c_packed < p.C && xi > 0 && h >= 0 && h < p.H && d >= 0 && d < p.D) {
        if (p.x_format == kPackFromAcc)
            a = pack_act_word<kPackFromAcc, 0>(p, ch, n_img, c_packed, d, h, xi);
        else if (p.x_format == HIKONV_FMT_INT8)
            a = pack_act_word<HIKONV_FMT_INT8, 0>(p, ch, n_img, c_packed, d, h, xi);
        else
            a = pack_act_word<HIKONV_FMT_BITDENSE, 0>(p, ch, n_img, c_packed, d, h, xi);
    }
    p.apk[idx] = a;
}

// B[group][term][8], term = ((c/4*Kh + kh)*chunks + chunk)*4 + c%4 (Kh counts depth x height kernel rows),
// word = sum_k g[chunk*K + k] 2^(S k) with g = the reversed kernel row (Eq. I_PRIME) of the
// packed channel c: the source row W[co][c][kh][Kw-1:0], or, for a polyphase layer, the
// reversed phase kernel g_phase[j] = W[co][c / s][kh][j*s + phase] (zero beyond the row).
__global__ __launch_bounds__(256) void k_pack_weights(PackWArgs p)
{
    const int terms = p.terms_pad;
    const int64_t total = (int64_t)p.n_cog * p.terms_pad * 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int c8 = (int)(idx & 7);
    const int term = (int)((idx >> 3) % p.terms_pad);
    const int cog = (int)((idx >> 3) / p.terms_pad);
    if (term >= terms) { // padding of the pipeline group: contributes nothing
        p.wp[idx] = 0;
        return;
    }
    // term = (((quad*Kh + kh)*chunks + chunk)*4 + channel of the quad)
    const int gi = term >> 2;
    const int ch = gi % p.chunks;
    const int kh = (gi / p.chunks) % p.Kh;
    const int c = (gi / (p.chunks * p.Kh)) * 4 + (term & 3);
    if (c >= p.C) { // channels that only fill the last quad
        p.wp[idx] = 0;
        return;
    }
    const int csrc = c / p.phases, phase = c - csrc * p.phases;
    const int co = cog * 8 + c8;
    uint32_t bw = 0;
    for (int k = 0; k < p.Kp; ++k) {
        const int j = ch * p.Kp + k; // tap of the reversed row
        if (j >= p.Kw) break;
        int32_t v = 0;
        const int ksrc = (p.Kw - 1 - j) * p.phases + phase; // source tap
        if (co < p.Co && ksrc < p.Kwsrc) {
            const uint8_t byte = p.w[(((int64_t)co * p.Csrc + csrc) * p.Kh + kh) * p.Kwsrc + ksrc];
            if (p.bipolar)
                v = (int8_t)byte > 0 ? 1 : -1;
            else
                v = p.w_signed ? (int32_t)(int8_t)byte : (int32_t)byte;
        }
        bw += (uint32_t)v << (p.S * k);
    }
    p.wp[idx] = bw;
}

// Baseline: direct layer, one v_mad_i32_i24 per low-bit product.  One lane owns one output
// pixel and 8 output channels; the weights of 16 input channels are staged in LDS as int32.
constexpr int kCiTile = 16;
constexpr int kMaxTaps2d = 49;

template <bool A_SIGNED>
__global__ __launch_bounds__(256) void k_conv2d_unpacked(Conv2dDirectArgs p)
{
    __shared__ __attribute__((aligned(16))) int32_t s_w[kCiTile * kMaxTaps2d * 8];
    const int64_t pix = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t npix = (int64_t)p.Nimg * p.Ho * p.Wo;
    const bool active = pix < npix;
    const int64_t pc = active ? pix : 0;
    const int wo = (int)(pc % p.Wo), ho = (int)((pc / p.Wo) % p.Ho), n = (int)(pc / ((int64_t)p.Wo * p.Ho));
    const int co0 = blockIdx.y * 8;
    const int taps = p.Kh * p.Kw;
    int32_t acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int ci0 = 0; ci0 < p.C; ci0 += kCiTile) {
        const int nci = p.C - ci0 < kCiTile ? p.C - ci0 : kCiTile;
        __syncthreads();
        for (int i = threadIdx.x; i < nci * taps * 8; i += 256) {
            const int c8 = i & 7, t = (i >> 3) % taps, ci = (i >> 3) / taps;
            int32_t v = 0;
            if (co0 + c8 < p.Co) {
                const uint8_t byte = p.w[((int64_t)(co0 + c8) * p.C + ci0 + ci) * taps + t];
                v = p.w_signed ? (int32_t)(int8_t)byte : (int32_t)byte;
            }
            s_w[i] = v;
        }
        __syncthreads();
        for (int ci = 0; ci < nci; ++ci) {
            const uint8_t *xc = p.x + ((int64_t)n * p.C + ci0 + ci) * p.H * p.W;
            for (int kh = 0; kh < p.Kh; ++kh) {
                const int ih = ho * p.stride + kh - p.pad;
                for (int kw = 0; kw < p.Kw; ++kw) {
                    const int iw = wo * p.stride + kw - p.pad;
                    int32_t v = 0;
                    if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W) {
                        const uint8_t byte = xc[(int64_t)ih * p.W + iw];
                        v = A_SIGNED ? (int32_t)(int8_t)byte : (int32_t)byte;
                    }
                    const int4 *wv = reinterpret_cast<const int4 *>(&s_w[(ci * taps + kh * p.Kw + kw) * 8]);
                    const int4 w0 = wv[0], w1 = wv[1];
                    acc[0] = __mul24(v, w0.x) + acc[0];
                    acc[1] = __mul24(v, w0.y) + acc[1];
                    acc[2] = __mul24(v, w0.z) + acc[2];
                    acc[3] = __mul24(v, w0.w) + acc[3];
                    acc[4] = __mul24(v, w1.x) + acc[4];
                    acc[5] = __mul24(v, w1.y) + acc[5];
                    acc[6] = __mul24(v, w1.z) + acc[6];
                    acc[7] = __mul24(v, w1.w) + acc[7];
                }
            }
        }
    }
    if (!active) return;
#pragma unroll
    for (int c = 0; c < 8; ++c)
        if (co0 + c < p.Co) p.y[(((int64_t)n * p.Co + co0 + c) * p.Ho + ho) * p.Wo + wo] = acc[c];
}

// Tuned form of the baseline for 3x3 kernels: the same work decomposition as the packed
// kernel (one lane = one output pixel x 8 channels, weights of the channel tile staged in
// LDS, the input-channel range divided among the waves of a workgroup when the layer is
// small, next channel's activations loaded while the current one is multiplied), still one
// v_mad_i32_i24 per low-bit product.
constexpr int kCiStage = 64; // input channels whose weights are staged at a time (18 KB)

template <bool A_SIGNED>
__global__ __launch_bounds__(256) void k_conv2d_unpacked_3x3(Conv2dDirectArgs p, int ksplit)
{
    __shared__ __attribute__((aligned(16))) int32_t s_w[kCiStage * 9 * 8];
    __shared__ int32_t s_red[3 * 8 * 64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ks = wave % ksplit;
    const int64_t group = (int64_t)blockIdx.x * (4 / ksplit) + wave / ksplit;
    const int64_t npix = (int64_t)p.Nimg * p.Ho * p.Wo;
    const int64_t pix = group * 64 + lane;
    const bool active = pix < npix;
    const int64_t pc = active ? pix : 0;
    const int wo = (int)(pc % p.Wo), ho = (int)((pc / p.Wo) % p.Ho), n = (int)(pc / ((int64_t)p.Wo * p.Ho));
    const int co0 = blockIdx.y * 8;
    // the nine tap offsets of this pixel (clamped inside the image) and their validity
    int off[9];
    bool ok[9];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const int ih = ho * p.stride + kh - p.pad, iw = wo * p.stride + kw - p.pad;
            const bool v = ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
            ok[kh * 3 + kw] = v;
            off[kh * 3 + kw] = v ? ih * p.W + iw : 0;
        }
    const uint8_t *xn = p.x + (int64_t)n * p.C * p.H * p.W;
    const int64_t plane = (int64_t)p.H * p.W;
    int32_t acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};

    auto fetch = [&](int32_t (&v)[9], int ci) {
        const uint8_t *xc = xn + ci * plane;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const uint8_t byte = xc[off[t]];
            const int32_t val = A_SIGNED ? (int32_t)(int8_t)byte : (int32_t)byte;
            v[t] = ok[t] ? val : 0;
        }
    };
    auto multiply = [&](const int32_t (&v)[9], int cl) {
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int4 *wv = reinterpret_cast<const int4 *>(&s_w[(cl * 9 + t) * 8]);
            const int4 w0 = wv[0], w1 = wv[1];
            acc[0] = __mul24(v[t], w0.x) + acc[0];
            acc[1] = __mul24(v[t], w0.y) + acc[1];
            acc[2] = __mul24(v[t], w0.z) + acc[2];
            acc[3] = __mul24(v[t], w0.w) + acc[3];
            acc[4] = __mul24(v[t], w1.x) + acc[4];
            acc[5] = __mul24(v[t], w1.y) + acc[5];
            acc[6] = __mul24(v[t], w1.z) + acc[6];
            acc[7] = __mul24(v[t], w1.w) + acc[7];
        }
    };

    for (int ci0 = 0; ci0 < p.C; ci0 += kCiStage) {
        const int nci = p.C - ci0 < kCiStage ? p.C - ci0 : kCiStage;
        if (ci0 > 0) __syncthreads();
        for (int i = tid; i < nci * 72; i += 256) {
            const int c8 = i & 7, t = (i >> 3) % 9, ci = (i >> 3) / 9;
            int32_t v = 0;
            if (co0 + c8 < p.Co) {
                const uint8_t byte = p.w[((int64_t)(co0 + c8) * p.C + ci0 + ci) * 9 + t];
                v = p.w_signed ? (int32_t)(int8_t)byte : (int32_t)byte;
            }
            s_w[i] = v;
        }
        __syncthreads();
        // this wave's share of the staged channels
        const int per = (nci + ksplit - 1) / ksplit;
        const int c_begin = ks * per;
        int c_end = c_begin + per;
        if (c_end > nci) c_end = nci;
        if (c_begin >= c_end) continue;
        int32_t va[9], vb[9];
        fetch(va, ci0 + c_begin);
        for (int cl = c_begin; cl < c_end; cl += 2) {
            fetch(vb, ci0 + (cl + 1 < c_end ? cl + 1 : cl));
            multiply(va, cl);
            if (cl + 1 >= c_end) break;
            fetch(va, ci0 + (cl + 2 < c_end ? cl + 2 : cl + 1));
            multiply(vb, cl + 1);
        }
    }
    if (ksplit > 1) {
        __syncthreads();
        if (ks > 0) {
            int32_t *dst = s_red + ((wave - wave / ksplit - 1) * 8) * 64 + lane;
#pragma unroll
            for (int c = 0; c < 8; ++c) dst[c * 64] = acc[c];
        }
        __syncthreads();
        if (ks > 0) return;
        for (int k2 = 1; k2 < ksplit; ++k2) {
            const int w2 = wave + k2;
            const int32_t *src = s_red + ((w2 - w2 / ksplit - 1) * 8) * 64 + lane;
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] += src[c * 64];
        }
    }
    if (!active) return;
#pragma unroll
    for (int c = 0; c < 8; ++c)
        if (co0 + c < p.Co) p.y[(((int64_t)n * p.Co + co0 + c) * p.Ho + ho) * p.Wo + wo] = acc[c];
}

inline hipError_t grid_1d(int64_t total, dim3 *g)
{
    const int64_t blocks = ceil_div(total, 256);
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorNotSupported;
    *g = dim3((unsigned)blocks);
    return hipSuccess;
}

} // namespace

hipError_t launch_pack_act(const PackActArgs &a, hipStream_t stream)
{
    const int64_t planes = (int64_t)a.chunks * a.Nimg * a.Cq * a.Dp;
    if (planes <= 65535 && a.Hp <= 65535) { // the grid's y and z hold the rows and the planes
        PackActArgs b = a;
        b.rows_per_block = a.Xs * 4 >= 256 ? 1 : 256 / (a.Xs * 4);
        dim3 g((unsigned)ceil_div((int64_t)a.Xs * 4, 256), (unsigned)ceil_div(a.Hp, b.rows_per_block), (unsigned)planes);
#define HIKONV_PACK(NV)                                                                              \
    case NV:                                                                                         \
        if (a.x_format == kPackFromAcc)                                                              \
            hipLaunchKernelGGL((k_pack_act_rows<kPackFromAcc, NV>), g, dim3(256), 0, stream, b);          \
        else if (a.x_format == HIKONV_FMT_INT8)                                                      \
            hipLaunchKernelGGL((k_pack_act_rows<HIKONV_FMT_INT8, NV>), g, dim3(256), 0, stream, b);       \
        else                                                                                         \
            hipLaunchKernelGGL((k_pack_act_rows<HIKONV_FMT_BITDENSE, NV>), g, dim3(256), 0, stream, b);   \
        break;
        switch (a.N <= 8 ? a.N : 0) {
            HIKONV_PACK(1) HIKONV_PACK(2) HIKONV_PACK(3) HIKONV_PACK(4) HIKONV_PACK(5) HIKONV_PACK(6) HIKONV_PACK(7)
            HIKONV_PACK(8)
        default:
            HIKONV_PACK(0)
        }
#undef HIKONV_PACK
        return hipGetLastError();
    }
    dim3 g;
    int64_t threads = (int64_t)a.chunks * a.Nimg * a.Cq * a.Dp * a.Hp * a.Xs * 4;
    if (threads < a.toff_entries) threads = a.toff_entries;
    hipError_t e = grid_1d(threads, &g);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_pack_act, g, dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_pack_weights(const PackWArgs &a, hipStream_t stream)
{
    dim3 g;
    hipError_t e = grid_1d((int64_t)a.n_cog * a.terms_pad * 8, &g);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_pack_weights, g, dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_conv2d_packed(const Conv2dArgs &a_in, bool wide, bool any_signed, int co_tile, hipStream_t stream)
{
    Conv2dArgs a = a_in;
    int64_t row_groups;
    if (a.segs == 0)
        row_groups = ceil_div(a.wave_rows, a.rows_per_wave);
    else
        row_groups = a.wave_rows * a.segs;
    const int64_t gx = ceil_div(row_groups, a.pipelined ? 4 / a.ksplit : 4);
    const int64_t gy = ceil_div(a.Co, co_tile);
    if (gx <= 0 || gy <= 0 || gx * gy > 0x3fffffffLL) return hipErrorNotSupported;
    // the kernels index rows and row groups with 32-bit arithmetic (row group * rows per wave + 63 < 2^31)
    if (a.wave_rows >= 0x3fffffffLL || row_groups >= 0x3fffffffLL) return hipErrorNotSupported;
    // 1-D grid, tiles dealt to the XCDs in contiguous ranges
    a.tiles_x = (int)gx;
    a.tiles_y = (int)gy;
    a.per_xcd = gx * gy >= 64 ? (int)ceil_div(gx * gy, 8) : 0;
    dim3 g((unsigned)(a.per_xcd ? (int64_t)a.per_xcd * 8 : gx * gy));
    // Stores through 32-bit buffer offsets from the output row of a wave's first lane: the
    // lanes of a wave share one row (long rows) or cover rows_per_wave consecutive rows, which
    // may run into the following images.  Larger windows, or the caller's HIKONV_F_STORES64,
    // take the stores with 64-bit addresses.
    {
        int64_t window_rows = 1;
        if (a.segs == 0) {
            const int64_t more_images = (a.rows_per_wave - 1 + a.Ho - 1) / a.Ho;
            window_rows = more_images * a.Co * a.Ho + a.rows_per_wave + 1;
        }
        a.fast_store = window_rows * a.Wo * 4 < 0x7fffffffLL && !a.stores64 ? 1 : 0;
    }
    if (a.sreg) {
        if (!wide || co_tile != 8) return hipErrorNotSupported;
        const int hi = a.Kp - 1;
        return any_signed ? launch_conv2d_sreg_signed(a, hi, g, stream) : launch_conv2d_sreg_unsigned(a, hi, g, stream);
    }
    return wide ? launch_conv2d_wide(a, any_signed, co_tile, g, stream)
                : launch_conv2d_narrow(a, any_signed, co_tile, g, stream);
}

hipError_t launch_conv2d_unpacked(const Conv2dDirectArgs &a, hipStream_t stream)
{
    if (a.Kh * a.Kw > kMaxTaps2d) return hipErrorNotSupported;
    const int64_t gy = ceil_div(a.Co, 8);
    if (gy <= 0 || gy > 65535) return hipErrorNotSupported;
    if (a.Kh == 3 && a.Kw == 3) {
        const int64_t groups = ceil_div((int64_t)a.Nimg * a.Ho * a.Wo, 64);
        const int ksplit = groups * gy < 2048 && a.C >= 16 ? 4 : (groups * gy < 4096 && a.C >= 8 ? 2 : 1);
        const int64_t gx3 = ceil_div(groups, 4 / ksplit);
        if (gx3 <= 0 || gx3 > 0x7fffffffLL) return hipErrorNotSupported;
        dim3 g3((unsigned)gx3, (unsigned)gy);
        if (a.a_signed)
            hipLaunchKernelGGL((k_conv2d_unpacked_3x3<true>), g3, dim3(256), 0, stream, a, ksplit);
        else
            hipLaunchKernelGGL((k_conv2d_unpacked_3x3<false>), g3, dim3(256), 0, stream, a, ksplit);
        return hipGetLastError();
    }
    const int64_t gx = ceil_div((int64_t)a.Nimg * a.Ho * a.Wo, 256);
    if (gx <= 0 || gx > 0x7fffffffLL) return hipErrorNotSupported;
    dim3 g((unsigned)gx, (unsigned)gy);
    if (a.a_signed)
        hipLaunchKernelGGL((k_conv2d_unpacked<true>), g, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((k_conv2d_unpacked<false>), g, dim3(256), 0, stream, a);
    return hipGetLastError();
}

} // namespace hikonv

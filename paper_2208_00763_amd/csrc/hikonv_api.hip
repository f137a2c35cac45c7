// extern "C" entry points of libhikonv.so: argument checks, workspace layout, launches.
// No entry point allocates device memory or synchronises.
#include <atomic>
#include <cstdlib>

#include "../../include/hikonv_bench.h"
#include "hikonv_launch.h"

using namespace hikonv;

namespace {

thread_local int g_last_hip_error = 0;

inline int hip_result(hipError_t e)
{
    if (e == hipSuccess) return HIKONV_OK;
    g_last_hip_error = (int)e;
    // the launchers of this library answer hipErrorNotSupported when no kernel covers a request;
    // everything else comes from the HIP runtime
    return e == hipErrorNotSupported ? HIKONV_EUNSUPPORTED : HIKONV_EHIP;
}

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

inline int64_t max_abs(int bits, int is_signed) { return is_signed ? (1LL << (bits - 1)) : (1LL << bits) - 1; }

// fills Conv1dArgs from the public arguments; returns HIKONV_OK, or 1 if there is nothing to do
int conv1d_common(int bits_a, int a_signed, int w_signed, const void *x_dev, int x_format, int64_t rows,
                  int64_t len, const void *g_dev, int taps, int out_mode, int32_t *y_dev, Conv1dArgs *a)
{
    if (bits_a < 1 || bits_a > 8 || rows < 0 || len < 0 || taps < 1 || taps > 64) return HIKONV_EINVAL;
    if (x_format != HIKONV_FMT_INT8 && x_format != HIKONV_FMT_BITDENSE) return HIKONV_EINVAL;
    if (out_mode != HIKONV_OUT_FULL && out_mode != HIKONV_OUT_VALID) return HIKONV_EINVAL;
    const int64_t out_len = out_mode == HIKONV_OUT_FULL ? len + taps - 1 : len - taps + 1;
    if (rows == 0 || len == 0 || out_len <= 0) return 1;
    if (!x_dev || !g_dev || !y_dev) return HIKONV_EINVAL;
    if (!aligned(x_dev, 4) || !aligned(y_dev, 16)) return HIKONV_EINVAL;
    if (rows > (1LL << 31) || len > (1LL << 40)) return HIKONV_EINVAL;
    a->x = static_cast<const uint32_t *>(x_dev);
    a->c = x_format == HIKONV_FMT_INT8 ? 8 : container_bits(bits_a);
    a->b = bits_a;
    const int64_t row_bytes = x_format == HIKONV_FMT_INT8 ? len : hikonv_bitdense_row_bytes(len, bits_a);
    a->row_stride_bits = row_bytes * 8;
    a->total_bytes = rows * row_bytes;
    a->total_dwords = a->total_bytes / 4;
    a->rows = rows;
    a->len = len;
    a->g = static_cast<const uint8_t *>(g_dev);
    a->taps = taps;
    a->w_signed = w_signed;
    a->shift_m = out_mode == HIKONV_OUT_VALID ? taps - 1 : 0;
    a->out_len = out_len;
    a->y = y_dev;
    (void)a_signed;
    return HIKONV_OK;
}

// Geometry of a layer call.  "Packed" quantities describe the rows the kernels see: a
// polyphase layer packs the column phases of each source channel as separate channels and
// materialises the horizontal padding; a 3-D layer adds a padded depth axis and counts the
// kernel's depth x height rows as the rows of a packed channel.
struct Conv2dGeom {
    int phases;          // column phases packed separately (= stride) or 1
    int Ce, We, Kwe;     // packed channels, values per packed row, taps per packed kernel row
    int Cq;              // channel quads: the packed channels are stored four to a 16-byte cell (zero beyond Ce)
    int padwe;           // horizontal padding that only shifts the read index (0 when materialised)
    int stride_w;        // column decimation on store (1 when the phases are packed separately)
    int pad_d, Dp, Do;   // depth padding, padded depth, output depth (0, 1, 1 for a 2-D layer)
    int Khe;             // kernel rows per packed channel (Kd*Kh)
    int Ho, Wo, Wo1, X, Xs, Hp, terms, terms_pad, n_cog;
    size_t apk_bytes, toff_bytes, wp_bytes;
};

// taps a plan must cover for a kernel row of Kw taps at column stride `stride`, polyphase form
inline int polyphase_taps(int Kw, int stride) { return (Kw + stride - 1) / stride; }

int conv_geom(const hikonv_plan_t *plan, int N, int C, int D, int H, int W, int Co, int Kd, int Kh, int Kw, int stride,
              int pad, int is3d, Conv2dGeom *g)
{
    if (!plan) return HIKONV_EINVAL;
    if (N < 1 || C < 1 || D < 1 || H < 1 || W < 1 || Co < 1 || Kd < 1 || Kh < 1 || Kw < 1 || stride < 1 || pad < 0)
        return HIKONV_EINVAL;
    if (plan->mode != HIKONV_MODE_DNN || plan->M < 1) return HIKONV_EINVAL;
    const bool polyphase = stride > 1 && plan->taps != Kw && plan->taps == polyphase_taps(Kw, stride);
    if (!polyphase && plan->taps != Kw) return HIKONV_EINVAL;
    g->phases = polyphase ? stride : 1;
    g->Kwe = polyphase ? polyphase_taps(Kw, stride) : Kw;
    if (plan->N < 1 || plan->K < 1 || plan->S < 1 || plan->chunks != (g->Kwe + plan->K - 1) / plan->K) return HIKONV_EINVAL;
    const bool wide = plan->L_A == 32 && plan->L_B == 32 && (plan->L_acc == 64 || plan->L_acc == 0);
    const bool narrow = plan->L_A == 24 && plan->L_B == 24 && plan->L_acc == 32;
    if (!wide && !narrow) return HIKONV_EUNSUPPORTED;
    if (plan->N > HIKONV_LAYER_MAX_N || plan->stride_elems > 1 || plan->chunks > 8 || Kd > 64 || Kh > 64 || Kw > 64) return HIKONV_EUNSUPPORTED;
    if (!polyphase && pad > Kw - 1) return HIKONV_EUNSUPPORTED; // the leading padding must fit inside the kernel width
    if (H + 2 * pad < Kh || W + 2 * pad < Kw || (is3d && D + 2 * pad < Kd)) return HIKONV_EINVAL;
    if (!is3d && (D != 1 || Kd != 1)) return HIKONV_EINVAL;
    if (hikonv_plan_check(plan) != HIKONV_OK) return HIKONV_EOVERFLOW;
    const int64_t worst = (int64_t)C * Kd * Kh * Kw * (plan->bipolar ? 1 : max_abs(plan->bits_a, plan->a_signed) *
                                                                                max_abs(plan->bits_w, plan->w_signed));
    if (worst >= (1LL << 31)) return HIKONV_EOVERFLOW;
    g->pad_d = is3d ? pad : 0;
    g->Dp = D + 2 * g->pad_d;
    g->Do = is3d ? (D + 2 * pad - Kd) / stride + 1 : 1;
    g->Khe = Kd * Kh;
    g->Ho = (H + 2 * pad - Kh) / stride + 1;
    g->Wo = (W + 2 * pad - Kw) / stride + 1;
    if (polyphase) {
        // output w reads the padded source row at s*w + k = s*(w + j) + phase: phase rows of
        // Wo + Kwe - 1 values, convolved at stride 1 with the phase kernels, no padding left
        g->Ce = C * stride;
        g->We = g->Wo + g->Kwe - 1;
        g->padwe = 0;
        g->stride_w = 1;
        g->Wo1 = g->Wo;
    } else {
        g->Ce = C;
        g->We = W;
        g->padwe = pad;
        g->stride_w = stride;
        g->Wo1 = W + 2 * pad - Kw + 1;
    }
    g->X = (g->We + g->padwe + plan->N - 1) / plan->N;
    g->Xs = g->X + 1;
    g->Hp = H + 2 * pad;
    g->Cq = (g->Ce + 3) / 4;
    if ((int64_t)g->Cq * 4 * g->Khe * plan->chunks >= (1 << 24)) return HIKONV_EUNSUPPORTED;
    g->terms = g->Cq * 4 * g->Khe * plan->chunks; // four channels of a quad per (kernel row, chunk): a multiple of the term group
    g->terms_pad = g->terms;
    g->n_cog = (Co + 7) / 8;
    if ((int64_t)plan->chunks * N * g->Cq * 4 * g->Dp * g->Hp * g->Xs >= (1LL << 30)) return HIKONV_EUNSUPPORTED;
    if ((int64_t)N * g->Do * g->Ho >= (1LL << 31) || (int64_t)g->Do * g->Ho >= (1LL << 30)) return HIKONV_EUNSUPPORTED;
    g->apk_bytes = round256((size_t)plan->chunks * N * g->Cq * g->Dp * g->Hp * g->Xs * 16);
    g->wp_bytes = round256((size_t)g->n_cog * g->terms_pad * 8 * 4 + kTermGroup * 32); // one group of slack: read ahead, never used
    g->toff_bytes = round256((size_t)(g->terms / kTermGroup + 8) * 4); // one offset per term group, zeros beyond
    return HIKONV_OK;
}

int conv2d_geom(const hikonv_plan_t *plan, int N, int C, int H, int W, int Co, int Kh, int Kw, int stride, int pad,
                Conv2dGeom *g)
{
    return conv_geom(plan, N, C, 1, H, W, Co, 1, Kh, Kw, stride, pad, 0, g);
}

// C, Kw: the source tensor's channels and kernel width; Khe = Kd*Kh kernel rows per channel
int pack_weights_impl(const hikonv_plan_t *plan, const Conv2dGeom &g, const void *w_dev, int Co, int C, int Kh,
                      int Kw, void *packed_dev, hipStream_t stream)
{
    PackWArgs a;
    a.w = static_cast<const uint8_t *>(w_dev);
    a.Co = Co;
    a.C = g.Ce;
    a.Csrc = C;
    a.phases = g.phases;
    a.Kh = g.Khe;
    a.Kw = g.Kwe;
    a.Kwsrc = Kw;
    (void)Kh;
    a.w_signed = plan->w_signed;
    a.bipolar = plan->bipolar;
    a.Kp = plan->K;
    a.S = plan->S;
    a.chunks = plan->chunks;
    a.n_cog = g.n_cog;
    a.terms_pad = g.terms_pad;
    a.wp = static_cast<uint32_t *>(packed_dev);
    return hip_result(launch_pack_weights(a, stream));
}

// Geometry part of the activation-packing arguments (source fields are left to the caller).
PackActArgs pack_act_args(const hikonv_plan_t *plan, const Conv2dGeom &g, int N, int C, int D, int H, int W, int Kd,
                          int Kh, int pad, uint32_t *apk, int32_t *toff)
{
    PackActArgs pa = {};
    pa.b = plan->bits_a;
    pa.a_signed = plan->a_signed;
    pa.bipolar = plan->bipolar;
    pa.Nimg = N;
    pa.C = g.Ce;
    pa.Csrc = C;
    pa.phases = g.phases;
    pa.pad_w_mat = g.phases > 1 ? pad : 0;
    pa.D = D;
    pa.Dp = g.Dp;
    pa.pad_d = g.pad_d;
    pa.H = H;
    pa.W = g.We;
    pa.Wsrc = W;
    pa.pad = pad;
    pa.N = plan->N;
    pa.Kp = plan->K;
    pa.S = plan->S;
    pa.chunks = plan->chunks;
    pa.Hp = g.Hp;
    pa.Xs = g.Xs;
    pa.apk = apk;
    pa.toff = toff;
    pa.toff_entries = g.terms / kTermGroup + 8; // zero beyond the groups: the kernels read up to four groups ahead
    pa.groups = g.terms / kTermGroup;
    pa.Cq = g.Cq;
    pa.Kh = Kh;
    pa.Kd = Kd;
    pa.chunk_stride = (int64_t)N * g.Cq * g.Dp * g.Hp * g.Xs;
    return pa;
}

int layer_impl(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C, int D, int H, int W,
               const void *w_dev, int prepacked, int Co, int Kd, int Kh, int Kw, int stride, int pad, int is3d,
               void *workspace_dev, size_t workspace_bytes, int32_t *y_dev, void *stream_v)
{
    Conv2dGeom g;
    int rc = conv_geom(plan, N, C, D, H, W, Co, Kd, Kh, Kw, stride, pad, is3d, &g);
    if (rc != HIKONV_OK) return rc;
    if (!w_dev || !y_dev) return HIKONV_EINVAL;
    if (x_format != HIKONV_FMT_INT8 && x_format != HIKONV_FMT_BITDENSE && x_format != HIKONV_FMT_PACKED)
        return HIKONV_EINVAL;
    if (x_format != HIKONV_FMT_PACKED && (!x_dev || !aligned(x_dev, 4))) return HIKONV_EINVAL;
    if (!aligned(y_dev, 4) || !aligned(w_dev, prepacked ? 256 : 1)) return HIKONV_EINVAL;
    const size_t need = g.apk_bytes + g.toff_bytes + (prepacked ? 0 : g.wp_bytes);
    if (!workspace_dev || !aligned(workspace_dev, 256) || workspace_bytes < need) return HIKONV_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    uint8_t *ws = static_cast<uint8_t *>(workspace_dev);
    uint32_t *apk = reinterpret_cast<uint32_t *>(ws);
    int32_t *toff = reinterpret_cast<int32_t *>(ws + g.apk_bytes);
    const uint8_t *wpk = static_cast<const uint8_t *>(w_dev);
    if (!prepacked) {
        uint8_t *dst = ws + g.apk_bytes + g.toff_bytes;
        rc = pack_weights_impl(plan, g, w_dev, Co, C, Kh, Kw, dst, stream);
        if (rc != HIKONV_OK) return rc;
        wpk = dst;
    }

    if (x_format != HIKONV_FMT_PACKED) {
        PackActArgs pa = pack_act_args(plan, g, N, C, D, H, W, Kd, Kh, pad, apk, toff);
        pa.x = x_dev;
        pa.x_format = x_format;
        pa.c = x_format == HIKONV_FMT_INT8 ? 8 : container_bits(plan->bits_a);
        pa.row_bytes = x_format == HIKONV_FMT_INT8 ? W : hikonv_bitdense_row_bytes(W, plan->bits_a);
        rc = hip_result(launch_pack_act(pa, stream));
        if (rc != HIKONV_OK) return rc;
    }

    Conv2dArgs ca;
    ca.apk = apk;
    ca.wp = reinterpret_cast<const uint32_t *>(wpk);
    ca.Nimg = N;
    ca.C = g.Ce;
    ca.Ho = g.Do * g.Ho;
    ca.Ho2d = g.Ho;
    ca.img_rows = (int64_t)g.Cq * g.Dp * g.Hp;
    ca.d_rows = (int64_t)stride * g.Hp;
    ca.stride_w = g.stride_w;
    ca.Wo1 = g.Wo1;
    ca.Kh = Kh;
    ca.stride = stride;
    ca.off = g.Kwe - 1 - g.padwe;
    ca.Hp = g.Hp;
    ca.Xs = g.Xs;
    ca.X = g.X;
    ca.N = plan->N;
    ca.S = plan->S;
    ca.chunks = plan->chunks;
    ca.M = plan->M;
    ca.terms = g.terms;
    ca.terms_pad = g.terms_pad;
    ca.chunk_stride = (int64_t)N * g.Cq * g.Dp * g.Hp * g.Xs;
    if (g.Xs <= 64) {
        ca.rows_per_wave = 64 / g.Xs;
        ca.segs = 0;
    } else {
        ca.rows_per_wave = 1;
        ca.segs = (g.X + 62) / 63;
    }
    ca.wave_rows = (int64_t)N * g.Do * g.Ho;
    ca.Wo = g.Wo;
    const bool wide = plan->L_A == 32;
    const bool any_signed = plan->bipolar || plan->a_signed || plan->w_signed; // {-1,+1}: signed slices
    // the pipelined kernels split after a whole number of term groups
    // A term adds at most K products to a segment, and the terms between two splits may be any
    // mix of chunks: M*taps/K terms keep a segment within the M*taps products the plan allows.
    const int split_terms_any = (int)((int64_t)plan->M * g.Kwe / plan->K);
    const int split_terms = split_terms_any / kTermGroup * kTermGroup;
    ca.pipelined = split_terms >= kTermGroup ? 1 : 0;
    ca.split_terms = split_terms;
    ca.split_terms_any = split_terms_any > 0 ? split_terms_any : 1;
    // Kernel choice.  With the weights in scalar registers the term loop has no LDS traffic
    // and rows need no lane for their zero word; it needs enough (row group, channel tile)
    // pairs to fill the chip and is slower on small layers.
    // plan->kernel: HIKONV_KERNEL_LDS = LDS-staged kernels only, HIKONV_KERNEL_SREG =
    // scalar-register kernel wherever the plan allows it, HIKONV_KERNEL_AUTO = by layer size.
    const int forced_kernel = plan->kernel;
    if (forced_kernel > HIKONV_KERNEL_SREG) return HIKONV_EINVAL;
    ca.sreg = 0;
    if (forced_kernel != 1 && Co >= 8 &&
        conv2d_sreg_applicable(plan->N, plan->K, split_terms, wide)) {
        const int real = (g.We + (plan->chunks - 1) * plan->K + plan->N - 1) / plan->N;
        const int lanes = ca.segs ? 64 : (real < g.X ? real : g.X);
        const int64_t groups_s = ca.segs ? ca.wave_rows * ca.segs : ceil_div(ca.wave_rows, 64 / lanes);
        // measured: from about 768 (row group, channel tile) pairs on it wins (the LDS-staged
        // kernel is bound by its broadcast reads of B and its split needs a lane exchange); on
        // smaller layers, with few waves per SIMD to cover the scalar-load latency, it is slower
        const int64_t pairs = groups_s * ((Co + 7) / 8);
        const bool pick = pairs >= 768;
        ca.sreg = forced_kernel == 2 || pick ? 1 : 0;
    }
    ca.Lr = g.X;
    if (ca.sreg && ca.segs == 0) {
        // lanes only for the blocks that hold input values in some chunk
        const int real = (g.We + (plan->chunks - 1) * plan->K + plan->N - 1) / plan->N;
        ca.Lr = real < g.X ? real : g.X;
        ca.rows_per_wave = 64 / ca.Lr;
    }
    const int64_t row_groups = ca.segs ? ca.wave_rows * ca.segs : ceil_div(ca.wave_rows, ca.rows_per_wave);

    // enough waves to cover the load latency: divide the term range over 2 or 4 waves of a
    // workgroup when the layer has few (row group, channel tile) pairs
    auto choose_split = [&](int64_t base_waves, Conv2dArgs *args) {
        int ks = 1;
        if (args->pipelined) {
            if (base_waves < 2048 && g.terms_pad >= 64)
                ks = 4;
            else if (base_waves < 4096 && g.terms_pad >= 32)
                ks = 2;
        }
        args->ksplit = ks;
    };

    ca.toff = toff;
    ca.apk_bytes = (uint32_t)((size_t)plan->chunks * N * g.Cq * g.Dp * g.Hp * g.Xs * 16);
    ca.Kp = plan->K;
    ca.Co = Co;
    ca.cog0 = 0;
    ca.y = y_dev;
    ca.stores64 = (plan->flags & HIKONV_F_STORES64) ? 1 : 0;
    // Eight output channels per wave reuse every activation word eight times; layers with few
    // (row group, channel tile) pairs run faster with two channels per wave and four times the waves.
    int co_tile = Co >= 8 ? 8 : 2;
    if (!ca.sreg && ca.pipelined && row_groups * ((Co + 7) / 8) < 768) co_tile = 2;
    choose_split(row_groups * ((Co + co_tile - 1) / co_tile), &ca);
    rc = hip_result(launch_conv2d_packed(ca, wide, any_signed, co_tile, stream));
    if (rc != HIKONV_OK) return rc;

    return rc;
}

} // namespace

extern "C" int hikonv_last_hip_error(void) { return g_last_hip_error; }

extern "C" int hikonv_compact(const void *x_dev, int64_t rows, int64_t len, int bits, int bipolar, void *out_dev,
                              void *stream)
{
    if (container_bits(bits) == 0 || rows < 0 || len < 0 || (bipolar && bits != 1)) return HIKONV_EINVAL;
    if (rows == 0 || len == 0) return HIKONV_OK;
    if (!x_dev || !out_dev || !aligned(out_dev, 4)) return HIKONV_EINVAL;
    const int64_t row_dwords = hikonv_bitdense_row_bytes(len, bits) / 4;
    return hip_result(launch_compact(static_cast<const uint8_t *>(x_dev), rows, len, bits, bipolar,
                                     static_cast<uint32_t *>(out_dev), row_dwords, static_cast<hipStream_t>(stream)));
}

extern "C" int hikonv_check_range(const void *x_dev, int64_t count, int bits, int is_signed, int bipolar,
                                  uint32_t *violations_dev, void *stream)
{
    if (container_bits(bits) == 0 || count < 0 || (bipolar && bits != 1)) return HIKONV_EINVAL;
    if (count == 0) return HIKONV_OK;
    if (!x_dev || !violations_dev || !aligned(violations_dev, 4)) return HIKONV_EINVAL;
    const bool sgn = is_signed || bipolar;
    const int lo = sgn ? -(1 << (bits - 1)) : 0;
    const int hi = sgn ? (1 << (bits - 1)) - 1 : (1 << bits) - 1;
    return hip_result(launch_check_range(static_cast<const uint8_t *>(x_dev), count, lo, hi, sgn, bipolar != 0,
                                         violations_dev, static_cast<hipStream_t>(stream)));
}

extern "C" int hikonv_conv1d(const hikonv_plan_t *plan, const void *x_dev, int x_format, int64_t rows, int64_t len,
                             const void *g_dev, int taps, int out_mode, int32_t *y_dev, void *stream)
{
    if (!plan) return HIKONV_EINVAL;
    if (plan->mode != HIKONV_MODE_CONV1D || plan->taps != taps) return HIKONV_EINVAL;
    if (plan->bipolar) return HIKONV_EUNSUPPORTED;
    if (plan->stride_elems > 1) return HIKONV_EUNSUPPORTED; // container-aligned slices: requantised outputs only
    if (plan->L_A != 32 || plan->L_B != 32 || (plan->L_acc != 64 && plan->L_acc != 0)) return HIKONV_EUNSUPPORTED;
    if (plan->N < 1 || plan->N > 32 || plan->K < 1 || plan->S < 1 || plan->chunks < 1 || plan->chunks > 8)
        return HIKONV_EUNSUPPORTED;
    if (plan->chunks != (taps + plan->K - 1) / plan->K) return HIKONV_EINVAL;
    if (hikonv_plan_check(plan) != HIKONV_OK) return HIKONV_EOVERFLOW;
    Conv1dArgs a = {};
    int rc = conv1d_common(plan->bits_a, plan->a_signed, plan->w_signed, x_dev, x_format, rows, len, g_dev, taps,
                           out_mode, y_dev, &a);
    if (rc != HIKONV_OK) return rc == 1 ? HIKONV_OK : rc;
    a.N = plan->N;
    a.Kp = plan->K;
    a.S = plan->S;
    a.chunks = plan->chunks;
    const int64_t m_end = out_mode == HIKONV_OUT_VALID ? len : len + taps - 1;
    a.n_blocks = ceil_div(m_end, a.N);
    const bool any_signed = plan->a_signed || plan->w_signed;
    if (plan->kernel != HIKONV_KERNEL_AUTO && plan->kernel != HIKONV_KERNEL_LANES && plan->kernel != HIKONV_KERNEL_WINDOW)
        return HIKONV_EINVAL;
    // Kernel form: a lane per aligned group of 8 or 4 outputs where the plan allows it (its stores follow
    // the order of y across the whole workgroup, which the memory system takes faster than
    // per-wave runs); else a lane per block with the high parts exchanged between lanes.
    if (plan->kernel != HIKONV_KERNEL_LANES && conv1d_window_applicable(a)) {
        a.y_phase = (int)((reinterpret_cast<uintptr_t>(y_dev) >> 2) & 31);
        return hip_result(launch_conv1d_window(a, plan->a_signed != 0, any_signed, static_cast<hipStream_t>(stream)));
    }
    if (plan->kernel == HIKONV_KERNEL_WINDOW) return HIKONV_EUNSUPPORTED;
    if (conv1d_fast_applicable(a)) {
        a.CH = 0;
        a.aligned_runs = 1;     // a wave's output interval ends on 128-byte lines of y
        a.align_outputs = 32;
        a.tiles_per_row = conv1d_fast_runs_per_row(a);
        if (a.aligned_runs) {
            a.run_outputs = conv1d_fast_run_outputs(a);
            a.y_phase = (int)((reinterpret_cast<uintptr_t>(y_dev) >> 2) & (a.align_outputs - 1));
            if (a.run_outputs >= a.align_outputs)
                a.tiles_per_row = ceil_div(a.out_len + a.align_outputs - 1, a.run_outputs);
            else
                a.aligned_runs = 0;
        }
        return hip_result(launch_conv1d_fast(a, plan->a_signed != 0, any_signed, static_cast<hipStream_t>(stream)));
    }
    a.CH = conv1d_tile_chunks(a.N, a.n_blocks);
    a.tiles_per_row = ceil_div(a.n_blocks, (int64_t)4 * a.CH * 63);
    return hip_result(launch_conv1d_packed(a, plan->a_signed != 0, any_signed, static_cast<hipStream_t>(stream)));
}

extern "C" int hikonv_conv1d_unpacked(int bits_a, int bits_w, int signedness, const void *x_dev, int x_format,
                                      int64_t rows, int64_t len, const void *g_dev, int taps, int out_mode,
                                      int32_t *y_dev, void *stream)
{
    if (bits_w < 1 || bits_w > 8 || signedness < 0 || signedness > 3) return HIKONV_EINVAL;
    Conv1dArgs a = {};
    int rc = conv1d_common(bits_a, signedness & HIKONV_A_SIGNED, (signedness & HIKONV_W_SIGNED) ? 1 : 0, x_dev,
                           x_format, rows, len, g_dev, taps, out_mode, y_dev, &a);
    if (rc != HIKONV_OK) return rc == 1 ? HIKONV_OK : rc;
    a.y_phase = (int)((reinterpret_cast<uintptr_t>(y_dev) >> 2) & 31);
    return hip_result(launch_conv1d_unpacked(a, (signedness & HIKONV_A_SIGNED) != 0, static_cast<hipStream_t>(stream)));
}

namespace {

// Output side of the requantising 1-D entry points.
int requant_common(int shift, int qmax, int out_bits, void *q_dev, Conv1dArgs *a)
{
    const int c_out = container_bits(out_bits);
    if (c_out == 0 || shift < 0 || shift > 31 || qmax < 0 || qmax > (1 << out_bits) - 1) return HIKONV_EINVAL;
    a->rq_out = static_cast<uint32_t *>(q_dev);
    a->rq_row_dwords = hikonv_bitdense_row_bytes(a->out_len, out_bits) / 4;
    a->rq_shift = shift;
    a->rq_qmax = qmax;
    a->rq_c_out = c_out;
    a->y = nullptr;
    return HIKONV_OK;
}

} // namespace

extern "C" int hikonv_conv1d_requant(const hikonv_plan_t *plan, const void *x_dev, int x_format, int64_t rows,
                                     int64_t len, const void *g_dev, int taps, int out_mode, int shift, int qmax,
                                     int out_bits, void *q_dev, void *stream)
{
    if (!plan) return HIKONV_EINVAL;
    if (plan->mode != HIKONV_MODE_CONV1D || plan->taps != taps) return HIKONV_EINVAL;
    if (plan->bipolar) return HIKONV_EUNSUPPORTED;
    if (plan->L_A != 32 || plan->L_B != 32 || (plan->L_acc != 64 && plan->L_acc != 0)) return HIKONV_EUNSUPPORTED;
    if (plan->N < 1 || plan->K < 1 || plan->S < 1 || plan->S > 31 || plan->chunks < 1) return HIKONV_EUNSUPPORTED;
    if (plan->chunks != (taps + plan->K - 1) / plan->K) return HIKONV_EINVAL;
    if (hikonv_plan_check(plan) != HIKONV_OK) return HIKONV_EOVERFLOW;
    Conv1dArgs a = {};
    int rc = conv1d_common(plan->bits_a, plan->a_signed, plan->w_signed, x_dev, x_format, rows, len, g_dev, taps,
                           out_mode, static_cast<int32_t *>(q_dev), &a);
    if (rc != HIKONV_OK) return rc == 1 ? HIKONV_OK : rc;
    rc = requant_common(shift, qmax, out_bits, q_dev, &a);
    if (rc != HIKONV_OK) return rc;
    const bool any_signed = plan->a_signed || plan->w_signed;
    // Container-aligned slices (K = 1, the elements of a word S/c apart: packing becomes a mask):
    // the planner returns them under the measured-cost objective; the kernel takes its slice
    // width from the operands exactly as the planner does, so the two must agree.
    if (plan->stride_elems > 1) {
        if (!conv1d_requant_aligned_applicable(a, plan->a_signed != 0, plan->bits_w)) return HIKONV_EINVAL;
        const int sw = conv1d_requant_aligned_slice(a, any_signed, plan->bits_w);
        if (plan->S != sw || plan->N != 32 / sw || plan->K != 1 || plan->stride_elems != sw / a.c) return HIKONV_EINVAL;
        return hip_result(launch_conv1d_requant_aligned(a, plan->a_signed != 0, any_signed, plan->bits_w,
                                                        static_cast<hipStream_t>(stream)));
    }
    // One value and one tap per multiply (Theorem 1 with N = K = 1): nothing is packed, and the
    // one-product-per-multiply kernel is that plan's kernel.  The measured-cost objective returns
    // it where no packed plan is cheaper (8-bit operands, for one).
    if (plan->N == 1 && plan->K == 1)
        return hip_result(launch_conv1d_requant_unpacked(a, plan->a_signed != 0, static_cast<hipStream_t>(stream)));
    a.N = plan->N;
    a.Kp = plan->K;
    a.S = plan->S;
    a.chunks = plan->chunks;
    if (a.N > 32 || a.chunks > 8) return HIKONV_EUNSUPPORTED;
    a.rq_run_outputs = conv1d_requant_run_outputs(a.N, a.c, a.rq_c_out);
    if (a.rq_run_outputs <= 0) return HIKONV_EUNSUPPORTED;
    a.tiles_per_row = ceil_div(a.out_len, a.rq_run_outputs);
    return hip_result(launch_conv1d_requant(a, plan->a_signed != 0, any_signed, static_cast<hipStream_t>(stream)));
}

extern "C" int hikonv_conv1d_requant_unpacked(int bits_a, int bits_w, int signedness, const void *x_dev, int x_format,
                                              int64_t rows, int64_t len, const void *g_dev, int taps, int out_mode,
                                              int shift, int qmax, int out_bits, void *q_dev, void *stream)
{
    if (bits_w < 1 || bits_w > 8 || signedness < 0 || signedness > 3) return HIKONV_EINVAL;
    Conv1dArgs a = {};
    int rc = conv1d_common(bits_a, signedness & HIKONV_A_SIGNED, (signedness & HIKONV_W_SIGNED) ? 1 : 0, x_dev,
                           x_format, rows, len, g_dev, taps, out_mode, static_cast<int32_t *>(q_dev), &a);
    if (rc != HIKONV_OK) return rc == 1 ? HIKONV_OK : rc;
    rc = requant_common(shift, qmax, out_bits, q_dev, &a);
    if (rc != HIKONV_OK) return rc;
    return hip_result(
        launch_conv1d_requant_unpacked(a, (signedness & HIKONV_A_SIGNED) != 0, static_cast<hipStream_t>(stream)));
}

namespace {

// weight-side geometry only (no activations): the fields pack_weights_impl reads
int weights_geom(const hikonv_plan_t *plan, int Co, int C, int Kd, int Kh, int Kw, int stride, Conv2dGeom *g)
{
    if (!plan || Co < 1 || C < 1 || Kd < 1 || Kh < 1 || Kw < 1 || stride < 1) return HIKONV_EINVAL;
    if (plan->mode != HIKONV_MODE_DNN || plan->K < 1 || plan->S < 1 || plan->chunks < 1) return HIKONV_EINVAL;
    const bool polyphase = stride > 1 && plan->taps != Kw && plan->taps == polyphase_taps(Kw, stride);
    if (!polyphase && plan->taps != Kw) return HIKONV_EINVAL;
    *g = Conv2dGeom{};
    g->phases = polyphase ? stride : 1;
    g->Kwe = polyphase ? polyphase_taps(Kw, stride) : Kw;
    if (plan->chunks != (g->Kwe + plan->K - 1) / plan->K) return HIKONV_EINVAL;
    g->Ce = C * g->phases;
    g->Cq = (g->Ce + 3) / 4;
    g->Khe = Kd * Kh;
    if ((int64_t)g->Cq * 4 * g->Khe * plan->chunks >= (1 << 24)) return HIKONV_EUNSUPPORTED;
    g->terms = g->Cq * 4 * g->Khe * plan->chunks;
    g->terms_pad = g->terms;
    g->n_cog = (Co + 7) / 8;
    g->wp_bytes = round256((size_t)g->n_cog * g->terms_pad * 8 * 4 + kTermGroup * 32); // one group of slack: read ahead, never used
    return HIKONV_OK;
}

} // namespace

extern "C" size_t hikonv_packed_weights_bytes_ex(const hikonv_plan_t *plan, int Co, int C, int Kd, int Kh, int Kw,
                                                 int stride)
{
    Conv2dGeom g;
    if (weights_geom(plan, Co, C, Kd, Kh, Kw, stride, &g) != HIKONV_OK) return 0;
    return g.wp_bytes;
}

extern "C" size_t hikonv_packed_weights_bytes(const hikonv_plan_t *plan, int Co, int C, int Kh, int Kw)
{
    return hikonv_packed_weights_bytes_ex(plan, Co, C, 1, Kh, Kw, 1);
}

extern "C" int hikonv_pack_weights_ex(const hikonv_plan_t *plan, const void *w_dev, int Co, int C, int Kd, int Kh,
                                      int Kw, int stride, void *packed_dev, void *stream)
{
    if (!w_dev || !packed_dev) return HIKONV_EINVAL;
    Conv2dGeom g;
    int rc = weights_geom(plan, Co, C, Kd, Kh, Kw, stride, &g);
    if (rc != HIKONV_OK) return rc;
    if (!aligned(packed_dev, 256)) return HIKONV_EINVAL;
    return pack_weights_impl(plan, g, w_dev, Co, C, Kh, Kw, packed_dev, static_cast<hipStream_t>(stream));
}

extern "C" int hikonv_pack_weights(const hikonv_plan_t *plan, const void *w_dev, int Co, int C, int Kh, int Kw,
                                   void *packed_dev, void *stream)
{
    return hikonv_pack_weights_ex(plan, w_dev, Co, C, 1, Kh, Kw, 1, packed_dev, stream);
}

extern "C" size_t hikonv_conv2d_workspace_bytes(const hikonv_plan_t *plan, int N, int C, int H, int W, int Co, int Kh,
                                                int Kw, int stride, int pad, int prepacked)
{
    Conv2dGeom g;
    if (conv2d_geom(plan, N, C, H, W, Co, Kh, Kw, stride, pad, &g) != HIKONV_OK) return 0;
    return g.apk_bytes + g.toff_bytes + (prepacked ? 0 : g.wp_bytes);
}

extern "C" int hikonv_conv2d(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C, int H, int W,
                             const void *w_dev, int Co, int Kh, int Kw, int stride, int pad, void *workspace_dev,
                             size_t workspace_bytes, int32_t *y_dev, void *stream)
{
    return layer_impl(plan, x_dev, x_format, N, C, 1, H, W, w_dev, 0, Co, 1, Kh, Kw, stride, pad, 0, workspace_dev,
                      workspace_bytes, y_dev, stream);
}

extern "C" int hikonv_conv2d_prepacked(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C,
                                       int H, int W, const void *w_packed_dev, int Co, int Kh, int Kw, int stride,
                                       int pad, void *workspace_dev, size_t workspace_bytes, int32_t *y_dev,
                                       void *stream)
{
    return layer_impl(plan, x_dev, x_format, N, C, 1, H, W, w_packed_dev, 1, Co, 1, Kh, Kw, stride, pad, 0,
                      workspace_dev, workspace_bytes, y_dev, stream);
}

// ---- layer call for callers that cannot allocate ------------------------------------
//
// The workspace of hikonv_conv2d (packed activation words, term-offset table, packed weight
// words) lives in a fixed array in device memory instead of a caller buffer.  Every GPU the
// library runs on holds its own copy of the array, at its own address, until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the device
// address is looked up once per device, with that device current, and only that address is
// ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[HIKONV_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices]; // device address of `scratch` on each device (nullptr: not looked up yet)

// device address of this device's copy of `scratch`; nullptr (and the HIP error recorded) on failure
void *scratch_of_current_device()
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        g_last_hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidDevice);
        return nullptr;
    }
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr) return ptr;
    // two threads may both get here: the lookup has no side effect and both read the same address
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
        g_last_hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidSymbol);
        return nullptr;
    }
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    return ptr;
}

} // namespace

extern "C" int hikonv_conv2d_noalloc(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C, int H,
                                     int W, const void *w_dev, int Co, int Kh, int Kw, int stride, int pad,
                                     int32_t *y_dev, void *stream)
{
    if (x_format == HIKONV_FMT_PACKED) return HIKONV_EINVAL; // nobody else can have filled the library's own array
    Conv2dGeom g;
    int rc = conv2d_geom(plan, N, C, H, W, Co, Kh, Kw, stride, pad, &g);
    if (rc != HIKONV_OK) return rc;
    if (g.apk_bytes + g.toff_bytes + g.wp_bytes > (size_t)HIKONV_NOALLOC_SCRATCH_BYTES) return HIKONV_ESCRATCH;
    void *ptr = scratch_of_current_device();
    if (!ptr) return HIKONV_EHIP;
    // Every word of the array that the layer kernels read is written by this call's own packing
    // kernels first (zero words, padding rows and the tail of the offset table included), so
    // nothing has to be cleared between calls; all of it is ordered on `stream`.
    return layer_impl(plan, x_dev, x_format, N, C, 1, H, W, w_dev, 0, Co, 1, Kh, Kw, stride, pad, 0, ptr,
                      (size_t)HIKONV_NOALLOC_SCRATCH_BYTES, y_dev, stream);
}

extern "C" size_t hikonv_conv3d_workspace_bytes(const hikonv_plan_t *plan, int N, int C, int D, int H, int W, int Co,
                                                int Kd, int Kh, int Kw, int stride, int pad, int prepacked)
{
    Conv2dGeom g;
    if (conv_geom(plan, N, C, D, H, W, Co, Kd, Kh, Kw, stride, pad, 1, &g) != HIKONV_OK) return 0;
    return g.apk_bytes + g.toff_bytes + (prepacked ? 0 : g.wp_bytes);
}

extern "C" int hikonv_conv3d(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C, int D, int H,
                             int W, const void *w_dev, int prepacked, int Co, int Kd, int Kh, int Kw, int stride,
                             int pad, void *workspace_dev, size_t workspace_bytes, int32_t *y_dev, void *stream)
{
    if (x_format == HIKONV_FMT_PACKED) return HIKONV_EINVAL;
    return layer_impl(plan, x_dev, x_format, N, C, D, H, W, w_dev, prepacked ? 1 : 0, Co, Kd, Kh, Kw, stride, pad, 1,
                      workspace_dev, workspace_bytes, y_dev, stream);
}

extern "C" int hikonv_conv2d_unpacked(int bits_a, int bits_w, int signedness, const void *x_dev, int N, int C, int H,
                                      int W, const void *w_dev, int Co, int Kh, int Kw, int stride, int pad,
                                      int32_t *y_dev, void *stream)
{
    if (bits_a < 1 || bits_a > 8 || bits_w < 1 || bits_w > 8 || signedness < 0 || signedness > 7) return HIKONV_EINVAL;
    if (N < 1 || C < 1 || H < 1 || W < 1 || Co < 1 || Kh < 1 || Kw < 1 || stride < 1 || pad < 0) return HIKONV_EINVAL;
    if (H + 2 * pad < Kh || W + 2 * pad < Kw || !x_dev || !w_dev || !y_dev) return HIKONV_EINVAL;
    Conv2dDirectArgs a;
    a.x = static_cast<const uint8_t *>(x_dev);
    a.w = static_cast<const uint8_t *>(w_dev);
    const bool bip = (signedness & HIKONV_BIPOLAR) != 0;
    a.a_signed = bip || (signedness & HIKONV_A_SIGNED);
    a.w_signed = bip || (signedness & HIKONV_W_SIGNED);
    a.Nimg = N;
    a.C = C;
    a.H = H;
    a.W = W;
    a.Co = Co;
    a.Kh = Kh;
    a.Kw = Kw;
    a.stride = stride;
    a.pad = pad;
    a.Ho = (H + 2 * pad - Kh) / stride + 1;
    a.Wo = (W + 2 * pad - Kw) / stride + 1;
    a.y = y_dev;
    return hip_result(launch_conv2d_unpacked(a, static_cast<hipStream_t>(stream)));
}

extern "C" int hikonv_epilogue(const int32_t *acc_dev, int N, int C, int H, int W, int shift, int qmax, int pool,
                               int out_bits, int out_format, void *out_dev, void *stream)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || shift < 0 || shift > 31 || container_bits(out_bits) == 0) return HIKONV_EINVAL;
    if (qmax < 0 || qmax > (1 << out_bits) - 1 || !acc_dev || !out_dev || !aligned(out_dev, 4)) return HIKONV_EINVAL;
    if (out_format != HIKONV_FMT_INT8 && out_format != HIKONV_FMT_BITDENSE) return HIKONV_EINVAL;
    EpilogueArgs a;
    a.acc = acc_dev;
    a.Nimg = N;
    a.C = C;
    a.H = H;
    a.W = W;
    a.shift = shift;
    a.qmax = qmax;
    a.pool = pool ? 1 : 0;
    a.Ho = pool ? H / 2 : H;
    a.Wo = pool ? W / 2 : W;
    if (a.Ho < 1 || a.Wo < 1) return HIKONV_EINVAL;
    a.out_format = out_format;
    a.c = out_format == HIKONV_FMT_BITDENSE ? container_bits(out_bits) : 8;
    a.out_row_bytes = out_format == HIKONV_FMT_BITDENSE ? hikonv_bitdense_row_bytes(a.Wo, out_bits) : a.Wo;
    a.out = static_cast<uint8_t *>(out_dev);
    return hip_result(launch_epilogue(a, static_cast<hipStream_t>(stream)));
}

extern "C" int hikonv_epilogue_pack(const int32_t *acc_dev, int N, int C, int H, int W, int shift, int qmax, int pool,
                                    const hikonv_plan_t *next_plan, int next_Co, int next_Kh, int next_Kw,
                                    int next_stride, int next_pad, void *next_workspace_dev,
                                    size_t next_workspace_bytes, void *stream)
{
    if (!next_plan || N < 1 || C < 1 || H < 1 || W < 1 || shift < 0 || shift > 31 || !acc_dev) return HIKONV_EINVAL;
    if (next_plan->bipolar || next_plan->a_signed) return HIKONV_EUNSUPPORTED; // the outputs are unsigned values
    if (qmax < 0 || qmax > (1 << next_plan->bits_a) - 1) return HIKONV_EINVAL;
    const int Hn = pool ? H / 2 : H, Wn = pool ? W / 2 : W;
    if (Hn < 1 || Wn < 1) return HIKONV_EINVAL;
    Conv2dGeom g;
    int rc = conv2d_geom(next_plan, N, C, Hn, Wn, next_Co, next_Kh, next_Kw, next_stride, next_pad, &g);
    if (rc != HIKONV_OK) return rc;
    if (g.phases != 1) return HIKONV_EUNSUPPORTED; // the fused packing writes one column phase
    if (!next_workspace_dev || !aligned(next_workspace_dev, 256) ||
        next_workspace_bytes < g.apk_bytes + g.toff_bytes)
        return HIKONV_EWORKSPACE;
    uint8_t *ws = static_cast<uint8_t *>(next_workspace_dev);
    PackActArgs pa = pack_act_args(next_plan, g, N, C, 1, Hn, Wn, 1, next_Kh, next_pad, reinterpret_cast<uint32_t *>(ws),
                                   reinterpret_cast<int32_t *>(ws + g.apk_bytes));
    pa.x_format = kPackFromAcc;
    pa.acc = acc_dev;
    pa.acc_H = H;
    pa.acc_W = W;
    pa.pool = pool ? 1 : 0;
    pa.shift = shift;
    pa.qmax = qmax;
    return hip_result(launch_pack_act(pa, static_cast<hipStream_t>(stream)));
}

extern "C" int hikonv_conv2d_fused(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C, int H,
                                   int W, const void *w_packed_dev, int Co, int Kh, int Kw, int pad,
                                   void *workspace_dev, size_t workspace_bytes, int32_t *y_dev, int shift, int qmax,
                                   int pool, const hikonv_plan_t *next_plan, int next_Co, int next_Kh, int next_Kw,
                                   int next_pad, void *next_workspace_dev, size_t next_workspace_bytes, void *stream_v)
{
    Conv2dGeom g;
    int rc = conv2d_geom(plan, N, C, H, W, Co, Kh, Kw, 1, pad, &g);
    if (rc != HIKONV_OK) return rc;
    if (!w_packed_dev || !aligned(w_packed_dev, 256) || (y_dev && !aligned(y_dev, 4))) return HIKONV_EINVAL;
    if (!next_plan && !y_dev) return HIKONV_EINVAL; // nothing would be produced
    if (x_format != HIKONV_FMT_INT8 && x_format != HIKONV_FMT_BITDENSE && x_format != HIKONV_FMT_PACKED)
        return HIKONV_EINVAL;
    if (x_format != HIKONV_FMT_PACKED && (!x_dev || !aligned(x_dev, 4))) return HIKONV_EINVAL;
    if (!(plan->L_A == 32 && plan->L_B == 32 && (plan->L_acc == 64 || plan->L_acc == 0)) || plan->N > 4)
        return HIKONV_EUNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);

    FusedLayerArgs f = {};
    f.pool = pool ? 1 : 0;
    f.n_tiles = (Co + 7) / 8;
    f.segs = g.Xs <= 64 ? 1 : (g.X + 62) / 63;
    // rows per wave: as many whole rows as fit 64 lanes, fewer while that leaves the chip with
    // under 128 workgroups; with pooling a workgroup holds an even number of rows
    f.rpw = f.segs > 1 ? 1 : 64 / g.Xs;
    if (f.rpw > g.Ho) f.rpw = g.Ho;
    f.wr = 1;
    const int rpw_min = f.pool ? 2 : 1;
    if (f.pool) {
        if (f.rpw >= 2)
            f.rpw &= ~1;
        else
            f.wr = 2;
    }
    while (f.rpw > rpw_min && (int64_t)N * ((g.Ho + f.rpw * f.wr - 1) / (f.rpw * f.wr)) * f.n_tiles < 128) f.rpw = f.rpw / 2 < rpw_min ? rpw_min : (f.pool ? (f.rpw / 2 + 1) & ~1 : f.rpw / 2);
    f.shift = shift;
    f.qmax = qmax;
    f.has_next = next_plan ? 1 : 0;
    if (f.wr * f.segs > 16) return HIKONV_EUNSUPPORTED; // a workgroup holds at most 16 waves
    // the term range of a (rows, segment) divided over as many waves as the workgroup still holds,
    // two term groups per wave at least
    f.ksplit = 1;
    while (f.ksplit < 8 && f.wr * f.segs * f.ksplit * 2 <= 16 && g.terms / 4 >= f.ksplit * 4) f.ksplit *= 2;
    if (next_plan) {
        if (shift < 0 || shift > 31) return HIKONV_EINVAL;
        if (next_plan->bipolar || next_plan->a_signed) return HIKONV_EUNSUPPORTED; // the outputs are unsigned values
        if (qmax < 0 || qmax > (1 << next_plan->bits_a) - 1) return HIKONV_EINVAL;
        const int Hn = pool ? g.Ho / 2 : g.Ho, Wn = pool ? g.Wo / 2 : g.Wo;
        if (Hn < 1 || Wn < 1) return HIKONV_EINVAL;
        Conv2dGeom gn;
        rc = conv2d_geom(next_plan, N, Co, Hn, Wn, next_Co, next_Kh, next_Kw, 1, next_pad, &gn);
        if (rc != HIKONV_OK) return rc;
        if (!next_workspace_dev || !aligned(next_workspace_dev, 256) || next_workspace_bytes < gn.apk_bytes + gn.toff_bytes)
            return HIKONV_EWORKSPACE;
        uint8_t *nws = static_cast<uint8_t *>(next_workspace_dev);
        f.nx = pack_act_args(next_plan, gn, N, Co, 1, Hn, Wn, 1, next_Kh, next_pad, reinterpret_cast<uint32_t *>(nws),
                             reinterpret_cast<int32_t *>(nws + gn.apk_bytes));
    }
    Conv2dArgs &ca = f.c;
    ca.wp = static_cast<const uint32_t *>(w_packed_dev);
    ca.Nimg = N;
    ca.C = g.Ce;
    ca.Ho = g.Ho;
    ca.Ho2d = g.Ho;
    ca.Wo = g.Wo;
    ca.Wo1 = g.Wo1;
    ca.img_rows = (int64_t)g.Cq * g.Hp;
    ca.stride = 1;
    ca.stride_w = 1;
    ca.off = g.Kwe - 1 - g.padwe;
    ca.Hp = g.Hp;
    ca.Xs = g.Xs;
    ca.X = g.X;
    ca.N = plan->N;
    ca.S = plan->S;
    ca.Kp = plan->K;
    ca.chunks = plan->chunks;
    ca.M = plan->M;
    ca.terms = g.terms;
    ca.terms_pad = g.terms_pad;
    const int split_any = (int)((int64_t)plan->M * g.Kwe / plan->K);
    ca.split_terms_any = split_any > 0 ? split_any : 1;
    f.split_terms = split_any / kTermGroup * kTermGroup;
    ca.Co = Co;
    ca.Kh = Kh;
    ca.chunk_stride = (int64_t)N * g.Cq * g.Dp * g.Hp * g.Xs;
    ca.y = y_dev;

    // Input not packed yet: the workgroups pack the rows they need into LDS themselves when
    // that fits (no packing kernel, no workspace); else a packing kernel fills the workspace first.
    if (x_format != HIKONV_FMT_PACKED) {
        f.in = pack_act_args(plan, g, N, C, 1, H, W, 1, Kh, pad, nullptr, nullptr);
        f.in.x = x_dev;
        f.in.x_format = x_format;
        f.in.c = x_format == HIKONV_FMT_INT8 ? 8 : container_bits(plan->bits_a);
        f.in.row_bytes = x_format == HIKONV_FMT_INT8 ? W : hikonv_bitdense_row_bytes(W, plan->bits_a);
        // in-kernel packing reads a word's N containers as one 32-bit window of a tensor that is a
        // whole number of dwords below 2^32 bytes, with bit offsets inside an image below 2^30
        const int64_t in_bytes = (int64_t)N * C * H * f.in.row_bytes;
        f.pack_input = plan->N * f.in.c <= 32 && (in_bytes & 3) == 0 && in_bytes < (1LL << 32) &&
                               (int64_t)H * f.in.row_bytes * 32 < (1LL << 30)
                           ? 1
                           : 0;
        if (f.pack_input && conv2d_fused_lds(f) > 64 * 1024) f.pack_input = 0;
        // Every channel tile of a row group packs the same rows again, so this pays only while a
        // workgroup's share is small (measured: a 3-channel 320-wide layer gains a kernel launch;
        // on the 64-channel 56x56 layer the one-kernel form takes 17 us against 10.4 us for the
        // packing kernel plus the layer kernel).  HIKONV_KERNEL_LDS in the plan asks for it anyway.
        const int64_t words = (int64_t)plan->chunks * g.Cq * (f.rpw * f.wr + Kh - 1) * g.Xs * 4;
        if (f.pack_input && words > 2048 && plan->kernel != HIKONV_KERNEL_LDS) f.pack_input = 0;
    }
    if (!f.pack_input) {
        if (!workspace_dev || !aligned(workspace_dev, 256) || workspace_bytes < g.apk_bytes + g.toff_bytes)
            return HIKONV_EWORKSPACE;
        uint8_t *ws = static_cast<uint8_t *>(workspace_dev);
        ca.apk = reinterpret_cast<uint32_t *>(ws);
        ca.toff = reinterpret_cast<int32_t *>(ws + g.apk_bytes);
        if (conv2d_fused_lds(f) > 64 * 1024) return HIKONV_EUNSUPPORTED; // the tile's B words and int32 sums live in LDS
        if (x_format != HIKONV_FMT_PACKED) {
            PackActArgs pa = f.in;
            pa.apk = const_cast<uint32_t *>(ca.apk);
            pa.toff = const_cast<int32_t *>(ca.toff);
            rc = hip_result(launch_pack_act(pa, stream));
            if (rc != HIKONV_OK) return rc;
        }
    }
    const bool any_signed = plan->bipolar || plan->a_signed || plan->w_signed;
    return hip_result(launch_conv2d_fused(f, any_signed, stream));
}

extern "C" int hikonv_ubench(int kind, int iters, int blocks, void *buf_dev, size_t bytes, void *stream)
{
    if (!buf_dev || iters < 0 || blocks < 1 || blocks > (1 << 20) || !aligned(buf_dev, 16)) return HIKONV_EINVAL;
    return hip_result(launch_ubench(kind, iters, blocks, buf_dev, bytes, static_cast<hipStream_t>(stream)));
}

extern "C" int hikonv_selftest_lane_shift(int32_t *out_dev, void *stream)
{
    if (!out_dev) return HIKONV_EINVAL;
    return hip_result(launch_selftest_lane_shift(out_dev, static_cast<hipStream_t>(stream)));
}

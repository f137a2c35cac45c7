// One kernel per layer of a chain (Section "Complete model evaluation": a layer is the
// convolution followed by activation and pooling): the packed layer convolution whose store
// stage applies the next operator's ReLU, requantisation and optional 2x2 max-pool and writes
// the result as the NEXT layer's packed activation words (Eq. inpack; features are packed at
// run time - here by the workgroup that produced them), so that neither the int32
// accumulators nor a separate packing pass touch HBM between two layers.
//
// A workgroup owns R consecutive output rows of one image (R = 2 with pooling, so that a
// pooled row is complete inside it) and a tile of eight output channels (two whole 4-channel
// cells of the next layer's layout).  Its waves divide (row, 63-block segment of a long row,
// slice of the term range) among themselves; a lane owns one packed block:
//   stage     the tile's B words go to LDS once per workgroup, the int32 tile [R][8][Wo] is cleared;
//   multiply  as in k_conv2d_pipe: one 16-byte load brings the A words of four terms (up to
//             eight such loads in flight), B words come as broadcast LDS reads, Acc += A * B
//             over M terms before a split (Theorem 3, "DNN Convolution Extension");
//   split     high part to the next lane (DPP), N fields per channel (Eq. output_split, bias form);
//   reduce    every wave adds its partial int32 sums into the LDS tile (the slices of the term
//             range meet there);
//   epilogue  every thread then works from the tile: the accumulators go to y if the caller
//             wants them, and the packed words of the next layer are built:
//             q = min(qmax, max(acc, 0) >> shift) of the (pooled) values, N' of them shifted
//             to their slices, stored in the next layer's cell layout; the workgroups at the
//             image's top and bottom also write the zero padding rows of their channels, the
//             first workgroup the next layer's term-offset table.
#include "hikonv_conv2d_kernel.h"

namespace hikonv {
namespace {

constexpr int kFusedBatch = 8; // activation cells (term groups) a lane requests before it multiplies

// GROUP_SPLITS: the plan allows at least four terms between splits, which then fall on the
// boundaries of term groups (f.split_terms, a multiple of 4); else a split may follow any term
template <int N, bool ANY_SIGNED, bool GROUP_SPLITS>
__global__ __launch_bounds__(1024) void k_conv2d_fused(FusedLayerArgs f)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t s_mem[];
    const Conv2dArgs &p = f.c;
    uint32_t *s_w = s_mem;                                                  // [terms_pad][8]
    int32_t *s_acc = reinterpret_cast<int32_t *>(s_mem + (size_t)p.terms_pad * 8); // [R][8][Wo]
    const uint32_t *__restrict__ apk = p.apk;
    const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // workgroup -> (image, row group, channel tile), tile fastest: neighbours share the activation rows
    const int groups_per_img = (p.Ho + f.R - 1) / f.R;
    uint32_t v = blockIdx.x;
    const int tile = (int)(v % (uint32_t)f.n_tiles);
    v /= (uint32_t)f.n_tiles;
    const int n = (int)(v / (uint32_t)groups_per_img);
    const int rg = (int)(v - (uint32_t)n * (uint32_t)groups_per_img);
    const int r0 = rg * f.R;
    const int co0 = tile * 8;
    // wave -> (slice of the term range, segment of the row, row of the group)
    const int ks = wave % f.ksplit;
    const int seg = (wave / f.ksplit) % f.segs;
    const int rl = wave / (f.ksplit * f.segs);
    const int ho = r0 + rl;
    const int xi_raw = (f.segs > 1 ? seg * 63 : 0) + lane;
    const bool active = ho < p.Ho && xi_raw < p.Xs;
    const bool halo = lane == 0; // the row's zero word, or the block before a segment (recomputed for its high part)
    const int xi = active ? xi_raw : 0;
    const int64_t in_row = (int64_t)n * p.img_rows + (int64_t)(active ? ho : 0) * p.stride;
    const char *a_base = reinterpret_cast<const char *>(apk) + (in_row * p.Xs + xi) * 16;

    // this wave's slice of the term groups; group gi = (channel quad * Kh + kernel row) * chunks + chunk
    // reads the 16-byte cells at a byte offset that is plain arithmetic here (2-D layer, no
    // table read: the table sits in memory that another kernel has just written)
    const int groups = p.terms / 4;
    const int per = (groups + f.ksplit - 1) / f.ksplit;
    const int g_begin = ks * per;
    const int g_end = g_begin + per < groups ? g_begin + per : groups;
    auto group_offset = [&](int gi) -> uint32_t {
        const uint32_t q = (uint32_t)gi / (uint32_t)p.chunks, ch = (uint32_t)gi - q * (uint32_t)p.chunks;
        const uint32_t cq = q / (uint32_t)p.Kh, kh = q - cq * (uint32_t)p.Kh;
        return 16u * (uint32_t)(ch * p.chunk_stride + ((int64_t)cq * p.Hp + kh) * p.Xs); // < 2^32 (host check)
    };
    auto request = [&](uint4 (&cell)[kFusedBatch], int g0) {
#pragma unroll
        for (int b = 0; b < kFusedBatch; ++b) {
            const int gi = g0 + b < g_end ? g0 + b : g_end - 1; // past the end: the last group again, not used
            cell[b] = *reinterpret_cast<const uint4 *>(a_base + group_offset(gi < 0 ? 0 : gi));
        }
    };
    // the first activation cells are requested before anything else: their round trip to
    // memory overlaps the staging below
    uint4 cell[kFusedBatch];
    request(cell, g_begin);

    // stage the tile's B words (eight per term, contiguous in memory) and clear the int32 tile
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(p.wp + ((int64_t)tile * p.terms_pad) * 8);
        uint4 *dst = reinterpret_cast<uint4 *>(s_w);
        for (int i = tid; i < p.terms_pad * 2; i += nthreads) dst[i] = src[i];
        const int tile_ints = f.R * 8 * p.Wo;
        for (int i = tid; i < tile_ints; i += nthreads) s_acc[i] = 0;
    }
    __syncthreads();

    SplitState<N, 8, ANY_SIGNED, true> st;
    st.init(p.S);
    int since = 0, nsplit = 0;
    for (int g0 = g_begin; g0 < g_end; g0 += kFusedBatch) {
        if (g0 > g_begin) request(cell, g0);
#pragma unroll
        for (int b = 0; b < kFusedBatch; ++b) {
            if (g0 + b >= g_end) break; // wave-uniform
            const uint32_t a4[4] = {cell[b].x, cell[b].y, cell[b].z, cell[b].w};
            // the B words of the group's four terms: eight 128-bit broadcast reads issued together
            uint4 wq[8];
#pragma unroll
            for (int h = 0; h < 8; ++h) wq[h] = *reinterpret_cast<const uint4 *>(&s_w[(g0 + b) * 32 + 4 * h]);
            if (GROUP_SPLITS) {
                // splits fall on group boundaries: the 32 multiply-accumulates of a group form one block
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t w[8] = {wq[2 * u].x, wq[2 * u].y, wq[2 * u].z, wq[2 * u].w,
                                           wq[2 * u + 1].x, wq[2 * u + 1].y, wq[2 * u + 1].z, wq[2 * u + 1].w};
#pragma unroll
                    for (int c = 0; c < 8; ++c) st.mad(c, a4[u], w[c]);
                }
                since += 4;
                if (since >= f.split_terms) {
                    asm volatile("" ::: "memory"); // keep the split out of the multiply block
                    st.split();
                    since = 0;
                    ++nsplit;
                }
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t w[8] = {wq[2 * u].x, wq[2 * u].y, wq[2 * u].z, wq[2 * u].w,
                                           wq[2 * u + 1].x, wq[2 * u + 1].y, wq[2 * u + 1].z, wq[2 * u + 1].w};
#pragma unroll
                    for (int c = 0; c < 8; ++c) st.mad(c, a4[u], w[c]);
                    if (++since == p.split_terms_any) {
                        asm volatile("" ::: "memory");
                        st.split();
                        since = 0;
                        ++nsplit;
                    }
                }
            }
        }
    }
    if (since) {
        st.split();
        ++nsplit;
    }
    const int32_t unbias = ANY_SIGNED ? nsplit * (1 << (p.S - 1)) : 0;

    // the lane's N columns of eight channels join the other slices' sums in the tile
    if (active && !halo && g_begin < g_end) {
        const int x = xi - 1;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            int32_t *trow = s_acc + (rl * 8 + c) * p.Wo;
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const int w1 = x * N + j - p.off;
                if (w1 >= 0 && w1 < p.Wo) atomicAdd(&trow[w1], st.out[c][j] - unbias);
            }
        }
    }
    __syncthreads();

    // ---- epilogue ---------------------------------------------------------------------
    if (p.y) { // this layer's accumulators, rows of Wo consecutive values
        const int rows_here = p.Ho - r0 < f.R ? p.Ho - r0 : f.R;
        const int row_ints = 8 * p.Wo;
        for (int idx = tid; idx < rows_here * row_ints; idx += nthreads) {
            const int k = idx / row_ints;
            const int t = idx - k * row_ints;
            const int c = t / p.Wo, w1 = t - c * p.Wo;
            if (co0 + c < p.Co) p.y[(((int64_t)n * p.Co + co0 + c) * p.Ho + r0 + k) * p.Wo + w1] = s_acc[idx];
        }
    }
    if (!f.has_next) return; // workgroup-uniform

    // the next layer's packed activation words of this tile's channels
    const PackActArgs &nx = f.nx;
    uint32_t *cells = nx.apk;
    // channels of the tile that exist in the next layer's cells (whole quads: zero words beyond Co)
    const int c_cells = 4 * nx.Cq - co0 < 8 ? 4 * nx.Cq - co0 : 8;
    // word index of (chunk, channel of the tile, padded row, word); four channel words per cell
    auto cell_word = [&](int ch, int c, int hp, int xw) -> int64_t {
        const int cg = co0 + c;
        return ((ch * nx.chunk_stride + (((int64_t)n * nx.Cq + (cg >> 2)) * nx.Hp + hp) * nx.Xs + xw) << 2) + (cg & 3);
    };
    // rows of the next layer's input that this workgroup completes
    int rows_out = 0, hn0 = 0;
    if (f.pool) {
        hn0 = r0 >> 1;
        rows_out = (r0 + 1 < p.Ho && hn0 < nx.H) ? 1 : 0;
    } else {
        hn0 = r0;
        rows_out = p.Ho - r0 < f.R ? p.Ho - r0 : f.R;
    }
    const int per_row = nx.chunks * c_cells * nx.Xs;
    for (int idx = tid; idx < rows_out * per_row; idx += nthreads) {
        const int k = idx / per_row;
        int t = idx - k * per_row;
        const int xw = t % nx.Xs;
        t /= nx.Xs;
        const int c = t % c_cells, ch = t / c_cells;
        uint32_t word = 0;
        if (co0 + c < nx.C && xw > 0) {
            const int e0 = (xw - 1) * nx.N - ch * nx.Kp;
            for (int j = 0; j < nx.N; ++j) {
                const int i = e0 + j;
                if (i < 0 || i >= nx.W) continue;
                int32_t a;
                if (f.pool) {
                    const int32_t *t0 = s_acc + c * p.Wo + 2 * i;
                    const int32_t *t1 = t0 + 8 * p.Wo;
                    a = max(max(t0[0], t0[1]), max(t1[0], t1[1]));
                } else {
                    a = s_acc[(k * 8 + c) * p.Wo + i];
                }
                a = min(max(a, 0) >> f.shift, f.qmax);
                word += (uint32_t)a << (nx.S * j);
            }
        }
        cells[cell_word(ch, c, hn0 + k + nx.pad, xw)] = word;
    }
    // zero padding rows above the first and below the last input row
    if (nx.pad > 0 && (rg == 0 || rg == groups_per_img - 1)) {
        const int count = nx.pad * per_row;
        for (int side = 0; side < 2; ++side) {
            if (side == 0 ? rg != 0 : rg != groups_per_img - 1) continue;
            const int first = side == 0 ? 0 : nx.H + nx.pad;
            for (int idx = tid; idx < count; idx += nthreads) {
                const int k = idx / per_row;
                int t = idx - k * per_row;
                const int xw = t % nx.Xs;
                t /= nx.Xs;
                cells[cell_word(t / c_cells, t % c_cells, first + k, xw)] = 0u;
            }
        }
    }
    if (blockIdx.x == 0)
        for (int gi = tid; gi < nx.toff_entries; gi += nthreads) write_offset_entry(nx, gi);
}

} // namespace

size_t conv2d_fused_lds(const FusedLayerArgs &f)
{
    return ((size_t)f.c.terms_pad * 8 + (size_t)f.R * 8 * f.c.Wo) * 4;
}

hipError_t launch_conv2d_fused(const FusedLayerArgs &f, bool any_signed, hipStream_t stream)
{
    const int waves = f.R * f.segs * f.ksplit;
    if (waves < 1 || waves > 16) return hipErrorInvalidValue;
    const size_t lds = conv2d_fused_lds(f);
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    const int64_t groups = (int64_t)f.c.Nimg * ((f.c.Ho + f.R - 1) / f.R) * f.n_tiles;
    if (groups <= 0 || groups > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 g((unsigned)groups), b((unsigned)(waves * 64));
    switch (f.c.N) {
#define HIKONV_FUSED(NV)                                                                        \
    case NV:                                                                                    \
        if (any_signed && f.split_terms >= 4)                                                   \
            hipLaunchKernelGGL((k_conv2d_fused<NV, true, true>), g, b, lds, stream, f);         \
        else if (any_signed)                                                                    \
            hipLaunchKernelGGL((k_conv2d_fused<NV, true, false>), g, b, lds, stream, f);        \
        else if (f.split_terms >= 4)                                                            \
            hipLaunchKernelGGL((k_conv2d_fused<NV, false, true>), g, b, lds, stream, f);        \
        else                                                                                    \
            hipLaunchKernelGGL((k_conv2d_fused<NV, false, false>), g, b, lds, stream, f);       \
        break;
        HIKONV_FUSED(1) HIKONV_FUSED(2) HIKONV_FUSED(3) HIKONV_FUSED(4)
#undef HIKONV_FUSED
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace hikonv

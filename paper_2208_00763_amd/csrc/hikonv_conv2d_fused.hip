// One kernel per layer of a chain (Section "Complete model evaluation": a layer is the
// convolution followed by activation and pooling): the packed layer convolution whose store
// stage applies the next operator's ReLU, requantisation and optional 2x2 max-pool and writes
// the result as the NEXT layer's packed activation words (Eq. inpack; features are packed at
// run time - here by the workgroup that produced them), so that neither the int32
// accumulators nor a separate packing pass touch HBM between two layers.
//
// A workgroup owns R consecutive output rows of one image (an even number with pooling, so
// that pooled rows are complete inside it) and a tile of eight output channels (two whole
// 4-channel cells of the next layer's layout).  A wave holds as many whole rows as fit its 64
// lanes (or one 63-block segment of a long row), a lane one packed block; the waves of the
// workgroup divide (rows, segments, slices of the term range) among themselves:
//   pack      optional: when the layer's input is not packed yet, the workgroup first packs
//             the C x (R + Kh - 1) input rows it needs into LDS from the bit-dense (or
//             one-value-per-byte) tensor (Eq. inpack; runtime feature packing by the consumer,
//             cooperatively, once per workgroup instead of once per lane and term);
//   stage     the tile's B words go to LDS once per workgroup, the int32 tile [R][8][Wo] is cleared;
//   multiply  as in k_conv2d_pipe: one 16-byte read brings the A words of four terms (from
//             LDS, or from the packed activations in global memory with three loads in
//             flight), B words come as broadcast LDS reads, Acc += A * B over M terms before
//             a split (Theorem 3, "DNN Convolution Extension");
//   split     high part to the next lane (DPP), N fields per channel (Eq. output_split, bias form);
//   reduce    every wave adds its partial int32 sums into the LDS tile (the slices of the term
//             range meet there);
//   epilogue  every wave then works from the tile: the accumulators go to y if the caller
//             wants them, and the packed words of the next layer are built:
//             q = min(qmax, max(acc, 0) >> shift) of the (pooled) values, N' of them shifted
//             to their slices, stored in the next layer's cell layout; the workgroups at the
//             image's top and bottom also write the zero padding rows of their channels, the
//             first workgroup the next layer's term-offset table.
#include "hikonv_conv2d_kernel.h"

namespace hikonv {
namespace {

constexpr int kFusedBatch = 3; // activation cells (term groups) a lane requests before it multiplies (measured on the
                               // nine-layer chain: 2, 3, 4, 6, 8 -> 77.5, 76.8, 78.5, 78.1, 80.8 us)

// GROUP_SPLITS: the plan allows at least four terms between splits, which then fall on the
// boundaries of term groups (f.split_terms, a multiple of 4); else a split may follow any term.
// PACK_IN: the activation words are packed here, into LDS, from the raw input f.in describes.
template <int N, bool ANY_SIGNED, bool GROUP_SPLITS, bool PACK_IN>
__global__ __launch_bounds__(1024) void k_conv2d_fused(FusedLayerArgs f)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t s_mem[];
    const Conv2dArgs &p = f.c;
    const int R = f.rpw * f.wr;            // output rows of the workgroup
    const int R_in = R + p.Kh - 1;         // input rows they read (row stride 1)
    const int Cq = (p.C + 3) >> 2;
    uint32_t *s_w = s_mem;                                                          // [terms_pad][8]
    int32_t *s_acc = reinterpret_cast<int32_t *>(s_mem + (size_t)p.terms_pad * 8); // [R][8][Wo]
    uint32_t *s_a = s_mem + (size_t)p.terms_pad * 8 + (((size_t)R * 8 * p.Wo + 3) & ~(size_t)3); // [chunks][Cq][R_in][Xs][4]
    const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = nthreads >> 6;
    // workgroup -> (image, row group, channel tile), tile fastest: neighbours share the activation rows
    const int groups_per_img = (p.Ho + R - 1) / R;
    uint32_t v = blockIdx.x;
    const int tile = (int)(v % (uint32_t)f.n_tiles);
    v /= (uint32_t)f.n_tiles;
    const int n = (int)(v / (uint32_t)groups_per_img);
    const int rg = (int)(v - (uint32_t)n * (uint32_t)groups_per_img);
    const int r0 = rg * R;
    const int co0 = tile * 8;
    // wave -> (slice of the term range, segment of the row, wave row); lane -> (row of the wave, word)
    const int ks = wave % f.ksplit;
    const int seg = (wave / f.ksplit) % f.segs;
    const int wrow = wave / (f.ksplit * f.segs);
    int rw = 0, xi_raw = lane;
    if (f.segs > 1) {
        xi_raw = seg * 63 + lane;
    } else {
        rw = (int)((uint32_t)lane / (uint32_t)p.Xs);
        xi_raw = lane - rw * p.Xs;
    }
    const int rl = wrow * f.rpw + rw;      // row inside the workgroup's group
    const int ho = r0 + rl;
    const bool active = rw < f.rpw && ho < p.Ho && xi_raw < p.Xs;
    const bool halo = f.segs > 1 ? lane == 0 : xi_raw == 0; // a row's zero word, or the block before a segment
    const int xi = active ? xi_raw : 0;

    // this wave's slice of the term groups; group gi = (channel quad * Kh + kernel row) * chunks + chunk
    const int groups = p.terms / 4;
    const int per = (groups + f.ksplit - 1) / f.ksplit;
    const int g_begin = ks * per;
    const int g_end = g_begin + per < groups ? g_begin + per : groups;
    // 16-byte cell of this lane for group gi: in the packed activations in global memory (plain
    // arithmetic, no read of the offset table, which another kernel has just written), or in LDS
    const int64_t in_row = (int64_t)n * p.img_rows + (int64_t)(active ? ho : 0) * p.stride;
    const char *a_base = reinterpret_cast<const char *>(p.apk) + (in_row * p.Xs + xi) * 16;
    const int rl_a = active ? rl : 0;
    auto load_cell = [&](int gi) -> uint4 {
        const uint32_t q = (uint32_t)gi / (uint32_t)p.chunks, ch = (uint32_t)gi - q * (uint32_t)p.chunks;
        const uint32_t cq = q / (uint32_t)p.Kh, kh = q - cq * (uint32_t)p.Kh;
        if (PACK_IN) return *reinterpret_cast<const uint4 *>(&s_a[((((ch * Cq + cq) * R_in) + rl_a + kh) * p.Xs + xi) * 4]);
        return *reinterpret_cast<const uint4 *>(a_base + 16u * (uint32_t)(ch * p.chunk_stride + ((int64_t)cq * p.Hp + kh) * p.Xs));
    };
    auto request = [&](uint4 (&cell)[kFusedBatch], int g0) {
#pragma unroll
        for (int b = 0; b < kFusedBatch; ++b) {
            const int gi = g0 + b < g_end ? g0 + b : g_end - 1; // past the end: the last group again, not used
            cell[b] = load_cell(gi < 0 ? 0 : gi);
        }
    };
    // from global memory the first cells are requested before anything else: their round trip
    // overlaps the staging below
    uint4 cell[kFusedBatch];
    if (!PACK_IN) request(cell, g_begin);

    // stage the tile's B words (eight per term, contiguous in memory), clear the int32 tile
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(p.wp + ((int64_t)tile * p.terms_pad) * 8);
        uint4 *dst = reinterpret_cast<uint4 *>(s_w);
        for (int i = tid; i < p.terms_pad * 2; i += nthreads) dst[i] = src[i];
        const int tile_ints = R * 8 * p.Wo;
        for (int i = tid; i < tile_ints; i += nthreads) s_acc[i] = 0;
    }
    if (PACK_IN) {
        // Rows (chunk, quad, input row) are dealt to the waves, the 4*Xs words of a row to the
        // lanes (word xw of the quad's channel u).  A lane reads the 32-bit window that holds its
        // N containers (two dwords, funnel shift), clears the containers outside the row and
        // shifts the N values to their slices.
        //  - What a row needs (dword and bit of its first container in the tensor, its chunk's
        //    delay, whether it lies inside the image) is worked out once per wave, lane b for the
        //    wave's b-th row, and handed to all lanes with a lane read: no division per word.
        //  - The windows of kPackBatch rows are requested together, with clamped dword indices so
        //    that no branch separates the loads (a clamped dword only holds containers of
        //    elements outside the row, which are cleared; the host checks that the tensor is a
        //    whole number of dwords and that bit offsets inside an image fit 32 bits).
        constexpr int kPackBatch = 8;
        const PackActArgs &in = f.in;
        const int rows_a = p.chunks * Cq * R_in;
        const int cbits = in.c, vb = in.b;
        const int plane_bits = (int)((int64_t)in.H * in.row_bytes * 8);  // bits between channels of the source
        const int last = (int)((((int64_t)in.Nimg * in.Csrc * in.H * in.row_bytes) >> 2) - 1); // last dword of the tensor
        const uint32_t *xd = static_cast<const uint32_t *>(in.x);
        for (int first = wave; first < rows_a; first += nwaves * 64) { // 64 rows of this wave at a time
            // lane b: row first + b*nwaves
            int d_dw, d_sh, d_delay, d_quad;
            {
                const int row_l = first + lane * nwaves;
                const int row = row_l < rows_a ? row_l : first;
                const int r = row % R_in;
                const int t = row / R_in;
                const int cq = t % Cq, ch = t / Cq;
                const int h = r0 * p.stride + r - in.pad;  // source row (outside the image: zero padding)
                const bool row_ok = h >= 0 && h < in.H;
                const int64_t bit0 = ((((int64_t)n * in.Csrc + cq * 4) * in.H + (row_ok ? h : 0)) * in.row_bytes) * 8;
                d_dw = (int)(bit0 >> 5);
                d_sh = (int)(bit0 & 31);
                d_delay = ch * in.Kp;
                d_quad = row_ok ? cq * 4 : in.C;           // first channel of the quad; in.C: no channel of it exists
            }
            const int rows_w = (rows_a - first + nwaves - 1) / nwaves < 64 ? (rows_a - first + nwaves - 1) / nwaves : 64;
            // Work items of the wave: (row b of its rows_w rows, pass ei over the row's 4*Xs words, 64 words a
            // pass), rows fastest; kPackBatch items are loaded together whether they are rows of one pass or
            // passes over one row (a layer with few channels has a single row per wave and many passes).
            const int passes = (4 * p.Xs + 63) >> 6;
            const int items = rows_w * passes;
            for (int i0 = 0; i0 < items; i0 += kPackBatch) {
                uint32_t w0[kPackBatch], w1[kPackBatch], shb[kPackBatch];
                int lo[kPackBatch], hi[kPackBatch];
#pragma unroll
                for (int b = 0; b < kPackBatch; ++b) {
                    const int item = i0 + b < items ? i0 + b : i0; // past the end: the batch's first item again, not stored
                    const int ei = (int)((uint32_t)item / (uint32_t)rows_w), bb = item - ei * rows_w; // wave-uniform
                    const int e = lane + 64 * ei;                       // every lane takes part; e >= 4*Xs stores nothing
                    const int u = e & 3, xw = e >> 2;
                    const bool word_ok = e < 4 * p.Xs && xw > 0;
                    const int lane_bits = u * plane_bits + (xw - 1) * N * cbits;
                    const int r_dw = __builtin_amdgcn_readlane(d_dw, bb), r_sh = __builtin_amdgcn_readlane(d_sh, bb);
                    const int r_delay = __builtin_amdgcn_readlane(d_delay, bb), r_quad = __builtin_amdgcn_readlane(d_quad, bb);
                    const int e0 = (xw - 1) * N - r_delay;             // first element of the word
                    const bool ok = word_ok && r_quad + u < in.C;
                    lo[b] = e0 < 0 ? -e0 : 0;
                    hi[b] = ok ? (in.W - e0 < N ? in.W - e0 : N) : 0;
                    const int bit = r_sh + (ok ? lane_bits - r_delay * cbits : 0); // from the row's first dword; may be negative
                    const int d = r_dw + (bit >> 5);                   // floor shift
                    const int d0 = d < 0 ? 0 : (d > last ? last : d), d1 = d + 1 < 0 ? 0 : (d + 1 > last ? last : d + 1);
                    w0[b] = xd[d0];
                    w1[b] = xd[d1];
                    shb[b] = (uint32_t)bit & 31u;
                }
#pragma unroll
                for (int b = 0; b < kPackBatch; ++b) {
                    if (i0 + b >= items) break; // wave-uniform
                    const int item = i0 + b;
                    const int ei = (int)((uint32_t)item / (uint32_t)rows_w), bb = item - ei * rows_w;
                    const int e = lane + 64 * ei;
                    const int u = e & 3, xw = e >> 2;
                    const uint32_t raw = funnel_shr(w1[b], w0[b], shb[b]);
                    uint32_t a = 0;
#pragma unroll
                    for (int j = 0; j < N; ++j) {
                        int32_t val;
                        if (in.bipolar)
                            val = cbits == 8 ? ((int8_t)(raw >> (8 * j)) > 0 ? 1 : -1) : (((raw >> (j * cbits)) & 1u) ? 1 : -1);
                        else
                            val = in.a_signed ? __builtin_amdgcn_sbfe((int)raw, j * cbits, vb)
                                              : (int32_t)__builtin_amdgcn_ubfe(raw, j * cbits, vb);
                        if (j >= lo[b] && j < hi[b]) a += (uint32_t)val << (p.S * j);
                    }
                    if (e < 4 * p.Xs) s_a[((size_t)(first + bb * nwaves) * p.Xs + xw) * 4 + u] = a;
                }
            }
        }
    }
    __syncthreads();

    SplitState<N, 8, ANY_SIGNED, true> st;
    st.init(p.S);
    int since = 0, nsplit = 0;
    for (int g0 = g_begin; g0 < g_end; g0 += kFusedBatch) {
        if (PACK_IN || g0 > g_begin) request(cell, g0);
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

    // ---- epilogue: tile rows are dealt to the waves, the columns or words of a row to the lanes ----
    const int rows_here = p.Ho - r0 < R ? p.Ho - r0 : R;
    if (p.y) { // this layer's accumulators
        for (int row = wave; row < rows_here * 8; row += nwaves) {
            const int k = row >> 3, c = row & 7;
            if (co0 + c >= p.Co) continue;
            int32_t *yrow = p.y + (((int64_t)n * p.Co + co0 + c) * p.Ho + r0 + k) * p.Wo;
            const int32_t *trow = s_acc + row * p.Wo;
            for (int w1 = lane; w1 < p.Wo; w1 += 64) yrow[w1] = trow[w1];
        }
    }
    if (!f.has_next) return; // workgroup-uniform

    // the next layer's packed activation words of this tile's channels
    const PackActArgs &nx = f.nx;
    uint32_t *cells = nx.apk;
    // channels of the tile that exist in the next layer's cells (whole quads: zero words beyond Co)
    const int c_cells = 4 * nx.Cq - co0 < 8 ? 4 * nx.Cq - co0 : 8;
    // word index of (chunk, channel of the tile, padded row, word 0); four channel words per cell
    auto cell_row = [&](int ch, int c, int hp) -> int64_t {
        const int cg = co0 + c;
        return ((ch * nx.chunk_stride + (((int64_t)n * nx.Cq + (cg >> 2)) * nx.Hp + hp) * nx.Xs) << 2) + (cg & 3);
    };
    // rows of the next layer's input that this workgroup completes
    int rows_out, hn0;
    if (f.pool) {
        hn0 = r0 >> 1;
        rows_out = rows_here >> 1;
        if (hn0 + rows_out > nx.H) rows_out = nx.H - hn0;
    } else {
        hn0 = r0;
        rows_out = rows_here;
    }
    const int rows_n = rows_out * nx.chunks * c_cells;
    for (int row = wave; row < rows_n; row += nwaves) {
        const int c = row % c_cells;
        const int t = row / c_cells;
        const int ch = t % nx.chunks, k = t / nx.chunks;
        uint32_t *dst = cells + cell_row(ch, c, hn0 + k + nx.pad);
        const bool real = co0 + c < nx.C;
        const int32_t *t0 = s_acc + ((f.pool ? 2 * k : k) * 8 + c) * p.Wo;
        for (int xw = lane; xw < nx.Xs; xw += 64) {
            uint32_t word = 0;
            if (real && xw > 0) {
                const int e0 = (xw - 1) * nx.N - ch * nx.Kp;
                for (int j = 0; j < nx.N; ++j) {
                    const int i = e0 + j;
                    if (i < 0 || i >= nx.W) continue;
                    int32_t a;
                    if (f.pool) {
                        const int32_t *u0 = t0 + 2 * i, *u1 = u0 + 8 * p.Wo;
                        a = max(max(u0[0], u0[1]), max(u1[0], u1[1]));
                    } else {
                        a = t0[i];
                    }
                    a = min(max(a, 0) >> f.shift, f.qmax);
                    word += (uint32_t)a << (nx.S * j);
                }
            }
            dst[(int64_t)xw << 2] = word;
        }
    }
    // zero padding rows above the first and below the last input row
    if (nx.pad > 0) {
        for (int side = 0; side < 2; ++side) {
            if (side == 0 ? rg != 0 : rg != groups_per_img - 1) continue; // workgroup-uniform
            const int first = side == 0 ? 0 : nx.H + nx.pad;
            const int rows_z = nx.pad * nx.chunks * c_cells;
            for (int row = wave; row < rows_z; row += nwaves) {
                const int c = row % c_cells;
                const int t = row / c_cells;
                uint32_t *dst = cells + cell_row(t % nx.chunks, c, first + t / nx.chunks);
                for (int xw = lane; xw < nx.Xs; xw += 64) dst[(int64_t)xw << 2] = 0u;
            }
        }
    }
    if (blockIdx.x == 0)
        for (int gi = tid; gi < nx.toff_entries; gi += nthreads) write_offset_entry(nx, gi);
}

} // namespace

// dynamic LDS bytes: B words of the tile, int32 tile, and the packed input rows when they are packed here
size_t conv2d_fused_lds(const FusedLayerArgs &f)
{
    const size_t R = (size_t)f.rpw * f.wr;
    size_t words = (size_t)f.c.terms_pad * 8 + ((R * 8 * f.c.Wo + 3) & ~(size_t)3);
    if (f.pack_input) words += (size_t)f.c.chunks * ((f.c.C + 3) / 4) * (R + f.c.Kh - 1) * f.c.Xs * 4;
    return words * 4;
}

hipError_t launch_conv2d_fused(const FusedLayerArgs &f, bool any_signed, hipStream_t stream)
{
    const int waves = f.wr * f.segs * f.ksplit;
    const int R = f.rpw * f.wr;
    if (waves < 1 || waves > 16 || f.rpw < 1 || (f.segs > 1 && f.rpw != 1) || f.rpw * f.c.Xs > 64 * (f.segs > 1 ? f.segs : 1))
        return hipErrorNotSupported;
    if (f.pool && (R & 1)) return hipErrorNotSupported;
    const size_t lds = conv2d_fused_lds(f);
    if (lds > 64 * 1024) return hipErrorNotSupported;
    const int64_t groups = (int64_t)f.c.Nimg * ((f.c.Ho + R - 1) / R) * f.n_tiles;
    if (groups <= 0 || groups > 0x7fffffffLL) return hipErrorNotSupported;
    dim3 g((unsigned)groups), b((unsigned)(waves * 64));
    const bool gs = f.split_terms >= 4, pk = f.pack_input != 0;
    switch (f.c.N) {
#define HIKONV_FUSED4(NV, SG)                                                                            \
    if (gs && pk) hipLaunchKernelGGL((k_conv2d_fused<NV, SG, true, true>), g, b, lds, stream, f);        \
    else if (gs) hipLaunchKernelGGL((k_conv2d_fused<NV, SG, true, false>), g, b, lds, stream, f);        \
    else if (pk) hipLaunchKernelGGL((k_conv2d_fused<NV, SG, false, true>), g, b, lds, stream, f);        \
    else hipLaunchKernelGGL((k_conv2d_fused<NV, SG, false, false>), g, b, lds, stream, f);
#define HIKONV_FUSED(NV)                                                                                 \
    case NV:                                                                                             \
        if (any_signed) { HIKONV_FUSED4(NV, true) } else { HIKONV_FUSED4(NV, false) }                    \
        break;
        HIKONV_FUSED(1) HIKONV_FUSED(2) HIKONV_FUSED(3) HIKONV_FUSED(4)
#undef HIKONV_FUSED
#undef HIKONV_FUSED4
    default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

} // namespace hikonv

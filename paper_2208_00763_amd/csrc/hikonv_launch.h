// Host-visible kernel argument blocks and launcher prototypes (internal to libhikonv.so).
#ifndef HIKONV_LAUNCH_H
#define HIKONV_LAUNCH_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hikonv_internal.h"

namespace hikonv {

struct Conv1dArgs {
    const uint32_t *x;       // input buffer (4-byte aligned), rows back to back
    int64_t total_dwords;    // whole dwords in the buffer
    int64_t total_bytes;     // bytes in the buffer
    int64_t row_stride_bits; // bits from one row's element 0 to the next row's
    int64_t rows, len;
    int c, b;                // container bits, value bits
    const uint8_t *g;        // taps bytes
    int taps, w_signed;
    int N, Kp, S, chunks;    // plan
    int shift_m;             // taps-1 for VALID output, 0 for FULL
    int64_t out_len;
    int64_t n_blocks;        // packed blocks per row
    int CH;                  // wave-chunks of 63 blocks per wave
    int64_t tiles_per_row;
    int aligned_runs;        // streaming kernel, staged stores: 1 = a wave owns an output interval whose
                             // ends fall on 128-byte lines of y (it recomputes a few blocks at its start)
    int64_t run_outputs;     // aligned runs: outputs per interval (a multiple of 32)
    int y_phase;             // aligned runs: (y / 4) mod align_outputs, position of y inside its aligned unit
    int align_outputs;       // aligned runs: outputs per aligned unit (32 = 128 bytes), a power of two
    int32_t *y;
    // requantising kernels: q = min(qmax, max(y, 0) >> shift) in c_out-bit containers
    uint32_t *rq_out;        // [rows][rq_row_dwords]
    int64_t rq_row_dwords;
    int64_t rq_run_outputs;  // outputs per wave run (whole output dwords)
    int rq_shift, rq_qmax, rq_c_out;
};

int conv1d_tile_chunks(int N, int64_t n_blocks);
hipError_t launch_conv1d_packed(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream);
hipError_t launch_conv1d_unpacked(const Conv1dArgs &a, bool a_signed, hipStream_t stream);
// streaming variant (no workgroup barrier) for N <= 12 and N*c <= 32
bool conv1d_fast_applicable(const Conv1dArgs &a);
int64_t conv1d_fast_runs_per_row(const Conv1dArgs &a);
int64_t conv1d_fast_run_outputs(const Conv1dArgs &a); // outputs per line-aligned interval
hipError_t launch_conv1d_fast(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream);
// one lane = one aligned output quad, blocks walked inside the lane (no LDS, no lane exchange)
bool conv1d_window_applicable(const Conv1dArgs &a);
hipError_t launch_conv1d_window(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream);
// requantised bit-dense output: packed (streaming kernel for N <= 12 and N*c <= 32, a slow
// general kernel for the other plans up to N = 32) and baseline
int64_t conv1d_requant_run_outputs(int N, int c, int c_out);
hipError_t launch_conv1d_requant(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream);
hipError_t launch_conv1d_requant_unpacked(const Conv1dArgs &a, bool a_signed, hipStream_t stream);
// requantised output, container-aligned 16-bit slices (K = 1, N = 2): same containers in and out, sums within a slice
bool conv1d_requant_aligned_applicable(const Conv1dArgs &a, bool a_signed, int bits_w);
int conv1d_requant_aligned_slice(const Conv1dArgs &a, bool any_signed, int bits_w); // slice width the kernel uses: 16, or 4 (one-bit unsigned operands)
hipError_t launch_conv1d_requant_aligned(const Conv1dArgs &a, bool a_signed, bool any_signed, int bits_w, hipStream_t stream);

// ---- 2-D ---------------------------------------------------------------------------

// Terms per group of the pipelined layer kernel: packed weights and the offset table are
// zero-padded to a multiple of it, and splits happen after a multiple of it.
#ifndef HIKONV_TERM_GROUP
#define HIKONV_TERM_GROUP 4
#endif
constexpr int kTermGroup = HIKONV_TERM_GROUP;

// source of the activations k_pack_act packs: INT8 / bit-dense rows, or the previous layer's
// int32 accumulators, requantised (and max-pooled) on the way
constexpr int kPackFromAcc = 100;

struct PackActArgs {
    const void *x;           // NC(D)HW activations, INT8 or bit-dense rows
    int D, Dp, pad_d;        // source depth, padded depth of the packed rows, depth padding (1, 1, 0 for 2-D)
    int phases;              // column phases packed as separate channels (polyphase stride), else 1
    int pad_w_mat;           // horizontal padding materialised in the packed rows (polyphase), else 0
    int Csrc, Wsrc;          // source channels and row length (C = Csrc*phases packed channels of W elements)
    int Kd;                  // kernel depth (offset table)
    const int32_t *acc;      // kPackFromAcc: [Nimg][C][acc_H][acc_W] accumulators of the producing layer
    int acc_H, acc_W, pool, shift, qmax; // kPackFromAcc: q = min(qmax, max(acc, 0) >> shift) after 2x2 max-pool if pool
    int x_format, c, b, a_signed, bipolar;
    int64_t row_bytes;       // bytes per W-row of x (bit-dense: padded; INT8: W)
    int Nimg, C, H, W, pad;
    int N, Kp, S, chunks;    // plan
    int Hp, Xs;              // padded rows (H + 2 pad), words per packed row (1 zero word + blocks)
    uint32_t *apk;           // [chunks][Nimg][Cq][Dp][Hp][Xs][4]: the words of four channels side by side
    int32_t *toff;           // [toff_entries] byte offset (unsigned) of each term group's activation cells (0 beyond the groups)
    int toff_entries, groups, Kh; // table entries, term groups (4 channels of a quad x one kernel row and chunk)
    int Cq;                  // channel quads: ceil(C / 4)
    int64_t chunk_stride;    // 16-byte cells between chunk planes of apk
    int rows_per_block;      // k_pack_act_rows: packed rows per workgroup (set by the launcher)
};
hipError_t launch_pack_act(const PackActArgs &a, hipStream_t stream);

struct PackWArgs {
    const uint8_t *w;        // [Co][Csrc][Kh][Kwsrc], one value per byte (Kh counts depth x height kernel rows)
    int phases, Csrc, Kwsrc; // polyphase: packed channel c = source channel c / phases, column phase c % phases;
                             // tap j of a phase is source tap j*phases + phase (zero beyond Kwsrc)
    int Co, C, Kh, Kw, w_signed, bipolar;
    int Kp, S, chunks;
    int n_cog;               // ceil(Co / 8)
    int terms_pad;           // C*Kh*chunks rounded up to the pipeline group (zero words beyond)
    uint32_t *wp;            // [n_cog][terms_pad][8]
};
hipError_t launch_pack_weights(const PackWArgs &a, hipStream_t stream);

struct Conv2dArgs {
    const uint32_t *apk;     // packed activations
    const uint32_t *wp;      // packed weights, group-of-8 layout
    int Nimg, C, Ho, Wo1;    // Ho = output rows per (image, channel), all depth slices; Wo1 = stride-1 output width
    int Ho2d;                // output rows per depth slice (= Ho for a 2-D layer)
    int64_t img_rows;        // packed input rows per image (channels x padded depth x padded height)
    int64_t d_rows;          // packed input rows between the inputs of consecutive output depth slices
    int stride_w;            // column decimation applied when storing (1 when the phases are packed separately)
    int Kh, stride, off;     // stride between input rows of consecutive output rows; off = Kw - 1 - pad:
                             // output w sits at row-convolution index w + off
    int Hp, Xs, X;           // packed rows per image-channel, words per row, blocks per row
    int N, S, chunks, M;     // plan; M = products accumulated per split
    int terms;               // 4*ceil(C/4)*Kh*chunks, in the order (quad, kernel row, chunk, channel of the quad)
    int terms_pad;           // = terms (a multiple of 4: channels come in quads, zero weights beyond the real channels)
    int pipelined;           // 1: k_conv2d_pipe, 0: k_conv2d_packed
    int ksplit;              // waves of a workgroup sharing one row group (1, 2 or 4)
    int split_terms;         // terms between splits in the pipelined kernels (multiple of 4)
    int split_terms_any;     // terms between splits in the plain kernel
    const int32_t *toff;     // [terms/4 + 8] byte offset (unsigned) of every term group's 16-byte activation cells, 0 beyond
    uint32_t apk_bytes;      // size of the packed activations (bounds of the buffer loads)
    int Kp;                  // taps per B word
    int Co, cog0;            // output channels to write, first weight group
    int64_t chunk_stride;    // 16-byte cells between chunk planes of apk
    int rows_per_wave, segs; // lane mapping
    int tiles_x, tiles_y;    // row-group blocks x channel tiles; the grid is 1-D (see tile_of_workgroup)
    int per_xcd;             // ceil(tiles_x*tiles_y / 8), 0 = plain order
    int sreg;                // 1: k_conv2d_sreg (weights in scalar registers), 0: the LDS-staged kernels
    int Lr;                  // k_conv2d_sreg, segs == 0: lanes per row (blocks that hold input values)
    int64_t wave_rows;       // total rows = Nimg*Ho
    int Wo;                  // strided output width
    int32_t *y;              // [Nimg][Co][Ho][Wo]
    int stores64;            // 1: the caller asks for stores with 64-bit addresses
    int fast_store;          // 1: every lane's output lies less than 2^31 bytes after the output row of its wave's
                             // first lane (same channel): stores through buffer offsets (set by the launcher)
};
hipError_t launch_conv2d_packed(const Conv2dArgs &a, bool wide, bool any_signed, int co_tile,
                                hipStream_t stream);

// One kernel per layer of a chain: the packed layer whose store stage writes the next layer's
// packed activation words (ReLU, requantisation, optional 2x2 max-pool on the way).
struct FusedLayerArgs {
    Conv2dArgs c;        // this layer; y may be null (the accumulators are then not stored)
    int rpw, wr;         // whole rows per wave (1 when a row is cut into segments), waves in the row direction;
                         // the workgroup owns rpw*wr output rows (an even number with pooling)
    int n_tiles, segs;   // channel tiles of eight; 63-block segments per row (1: the row fits a wave)
    int ksplit;          // waves that divide the term range of one (rows, segment)
    int split_terms;     // terms between splits rounded down to whole term groups (0: fewer than 4 allowed)
    int shift, qmax, pool;
    int has_next;        // 0: plain layer (y only)
    int pack_input;      // 1: the activation words are packed in the kernel, into LDS, from `in`
    PackActArgs in;      // pack_input: this layer's raw input (INT8 or bit-dense) and packing geometry
    PackActArgs nx;      // has_next: geometry and buffers of the next layer's packed activations
};
size_t conv2d_fused_lds(const FusedLayerArgs &f); // dynamic LDS bytes (at most 64 KiB)
hipError_t launch_conv2d_fused(const FusedLayerArgs &f, bool any_signed, hipStream_t stream);

// plans this kernel covers: 32x32+64 multiply, at most three taps per B word and no more
// high segments than own segments, a whole number of term groups between splits
inline bool conv2d_sreg_applicable(int N, int Kp, int split_terms, bool wide)
{
    if (!wide || N < 1 || N > 8 || Kp < 1 || Kp > 3 || Kp - 1 > N) return false;
    if (split_terms < kTermGroup) return false;
    return true;
}

struct Conv2dDirectArgs {
    const uint8_t *x, *w;
    int a_signed, w_signed;
    int Nimg, C, H, W, Co, Kh, Kw, stride, pad, Ho, Wo;
    int32_t *y;
};
hipError_t launch_conv2d_unpacked(const Conv2dDirectArgs &a, hipStream_t stream);

struct EpilogueArgs {
    const int32_t *acc;
    int Nimg, C, H, W, shift, qmax, pool, Ho, Wo;
    int out_format, c;       // container bits when bit-dense
    int64_t out_row_bytes;
    uint8_t *out;
};
hipError_t launch_epilogue(const EpilogueArgs &a, hipStream_t stream);

// ---- misc --------------------------------------------------------------------------
hipError_t launch_compact(const uint8_t *x, int64_t rows, int64_t len, int bits, int bipolar,
                          uint32_t *out, int64_t row_dwords, hipStream_t stream);
hipError_t launch_check_range(const uint8_t *x, int64_t count, int lo, int hi, int is_signed, int bipolar,
                              uint32_t *violations, hipStream_t stream);
hipError_t launch_ubench(int kind, int iters, int blocks, void *buf, size_t bytes, hipStream_t stream);
hipError_t launch_selftest_lane_shift(int32_t *out, hipStream_t stream);

} // namespace hikonv
#endif

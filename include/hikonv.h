/*
 * hikonv.h -- C ABI of the MI355X (gfx950) HiKonv library.
 *
 * HiKonv computes low-bitwidth (1..8 bit, signed or unsigned) 1-D and 2-D
 * convolutions by packing several quantised values into one wide integer word
 * with guard bits, so that one full-width integer multiply yields a run of
 * partial convolution sums, which are then split by shift and mask,
 * sign-corrected and overlap-added across packed blocks.
 *
 * Conventions for every entry point
 *   - Pointers named *_dev are DEVICE pointers owned by the caller; pointers
 *     without that suffix are HOST pointers.  The library never allocates or
 *     frees device memory; scratch space comes from a caller-supplied workspace.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All device work is enqueued asynchronously on it; no call synchronises.
 *   - Return value: HIKONV_OK (0) or a negative HIKONV_E* code.  Nothing is
 *     printed, thrown or aborted.  Values outside the declared bit range are
 *     not detected on the hot path (undefined results, never a fault).
 *   - Outputs are always int32.
 */
#ifndef HIKONV_H
#define HIKONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HIKONV_OK 0
#define HIKONV_EINVAL (-1)       /* bad argument: bits outside 1..8, NULL pointer, negative size ... */
#define HIKONV_EOVERFLOW (-2)    /* a result could exceed int32 for values of the declared range   */
#define HIKONV_ENOPLAN (-3)      /* no (N, K, S) satisfies the constraints                         */
#define HIKONV_EHIP (-4)         /* a HIP call failed; see hikonv_last_hip_error()                 */
#define HIKONV_EWORKSPACE (-5)   /* workspace missing or too small                                 */
#define HIKONV_EUNSUPPORTED (-6) /* valid request that this build has no kernel for                */
#define HIKONV_ESCRATCH (-7)     /* hikonv_conv2d_noalloc: the layer needs more than HIKONV_NOALLOC_SCRATCH_BYTES */

/* Use of the multiplier; selects the guard-bit rule (Section "Maximizing Processing Throughput"). */
#define HIKONV_MODE_SINGLE 0 /* one multiply, F_{N,K}:           G_b = ceil(log2 min(K,N))  */
#define HIKONV_MODE_CONV1D 1 /* blocks overlap-added (Theorem 2): G_b = ceil(log2 taps)      */
#define HIKONV_MODE_DNN 2    /* M products accumulated before a split (Theorem 3)            */

/* signedness argument / flags */
#define HIKONV_A_SIGNED 1 /* activations / f are two's-complement signed */
#define HIKONV_W_SIGNED 2 /* weights / g are two's-complement signed     */
#define HIKONV_BIPOLAR 4  /* 1-bit values mean {-1,+1} (bit 1 = +1), both operands */

/* storage format of activations */
#define HIKONV_FMT_INT8 0     /* one value per byte (int8 if signed, uint8 if unsigned)              */
#define HIKONV_FMT_BITDENSE 1 /* little-endian bit stream per innermost row, value i at bits          */
                              /* [c*i, c*i+c), c = 1,2,4,4,8,8,8,8 for 1..8-bit values; rows padded   */
                              /* to a multiple of 4 bytes (Section "Single convolver architecture":   */
                              /* unused bits of quantised data are discarded in storage)              */

#define HIKONV_FMT_PACKED 2   /* conv2d only: the call's workspace already holds this layer's packed  */
                              /* activations, written by hikonv_epilogue_pack for the same plan and    */
                              /* geometry; x_dev is ignored                                            */

#define HIKONV_OUT_FULL 0  /* len + taps - 1 outputs per row (Eq. pad_f) */
#define HIKONV_OUT_VALID 1 /* y[taps-1 .. len-1]: len - taps + 1 outputs */

/* What the planner optimises (hikonv_plan_t.objective). */
#define HIKONV_OBJ_PAPER_OPS 0     /* Algorithm 1: most low-bit operations per multiply, Eq. (tot_ops); with a  */
                                   /* fixed tap count: most multiply-accumulates per multiply                    */
#define HIKONV_OBJ_MEASURED_COST 1 /* fewest modelled VALU issue slots per output (layers: per multiply-       */
                                   /* accumulate) on gfx950: every candidate                                    */
                                   /* (N, K, S) is priced with per-instruction counts for packing, multiplying, */
                                   /* exchanging, splitting and storing calibrated on MI355X counters, bounded  */
                                   /* below by the slots that fit under the HBM time of its bytes               */

/* Kernel form (hikonv_plan_t.kernel); AUTO lets the library choose (layers: by size). */
#define HIKONV_KERNEL_AUTO 0
#define HIKONV_KERNEL_LDS 1    /* layers: weight words staged in LDS (small layers)                      */
#define HIKONV_KERNEL_SREG 2   /* layers: weight words in scalar registers wherever the plan allows it   */
#define HIKONV_KERNEL_LANES 3  /* hikonv_conv1d: one lane = one packed block, high parts exchanged between */
                               /* neighbouring lanes, outputs staged per wave                             */
#define HIKONV_KERNEL_WINDOW 4 /* hikonv_conv1d: one lane = an aligned group of 4 or 8 outputs, the blocks that */
                               /* cover it multiplied one after the other (AUTO takes it where it applies: */
                               /* at most 7 taps, K = min(taps, N), N in {2,3,4,5,6,8,11})                 */

/* hikonv_plan_t.flags */
#define HIKONV_F_STORES64 1 /* layer kernels: address every output store with 64 bits (the library does this by */
                            /* itself for outputs of 2^31 bytes or more)                                        */

/* The layer kernels (hikonv_conv2d, hikonv_conv3d) hold at most this many slices per lane. */
#define HIKONV_LAYER_MAX_N 8

/*
 * A packing plan.  Request fields are read by hikonv_plan_ex; result fields are
 * written by the planner and read by the convolution entry points, which run
 * exactly the plan they are handed.
 *   Section "Multiplier for Convolution": p, q, L_A, L_B, slice S, guard bits G_b.
 */
typedef struct hikonv_plan_t {
    /* request */
    int32_t bits_a, bits_w;     /* p, q: bitwidths of f (activations) and g (weights), 1..8          */
    int32_t a_signed, w_signed; /* per operand                                                       */
    int32_t bipolar;            /* 1: both operands are {-1,+1}, one bit each in storage (bit 1 = +1); */
                                /* packed as signed slices, 0 in the zero padding                      */
    int32_t L_A, L_B;           /* multiplier input widths in bits                                   */
    int32_t L_acc;              /* width of the product/accumulator register (0 = L_A + L_B)         */
    int32_t mode;               /* HIKONV_MODE_*                                                     */
    int32_t M;                  /* DNN mode: (channel, kernel-row) products accumulated per split;   */
                                /* 0 = let the planner choose                                        */
    int32_t taps;               /* kernel width that must be covered (0 = free: Algorithm 1 picks K) */
    int32_t tight;              /* 0: S = p+q+G_b as in Eq. (slice1) (one more bit where signed data */
                                /* needs it); 1: the smallest S for which every segment sum of the   */
                                /* declared value ranges provably fits (G_b then reports S minus the */
                                /* product width and may be smaller than the paper's)                */
    int32_t objective;          /* HIKONV_OBJ_*                                                      */
    int32_t out_bits;           /* CONV1D mode, measured-cost objective: what the split produces.    */
                                /* 0: int32 outputs (hikonv_conv1d); 1..8: outputs requantised to    */
                                /* this many bits and stored bit-dense (hikonv_conv1d_requant)       */
    int32_t max_N;              /* 0: no limit; else only plans with N <= max_N are considered       */
                                /* (HIKONV_LAYER_MAX_N for plans meant for hikonv_conv2d/conv3d)     */
    int32_t kernel;             /* HIKONV_KERNEL_*; copied through by the planner                    */
    int32_t flags;              /* HIKONV_F_*; copied through by the planner                         */
    /* result */
    int32_t N, K, S, G_b;       /* elements per A word, taps per B word, slice bits, guard bits      */
    int32_t chunks;             /* ceil(taps / K): B words per kernel row (1 if taps == 0)           */
    int32_t ops_per_mul;        /* N*K + (N-1)*(K-1), Eq. (tot_ops)                                  */
    int32_t paper_exact;        /* 1: (N,K,S,G_b) are exactly what Eq. (slice1)-(slice3) and         */
                                /* Algorithm 1 give; 0: adjusted so that every value of the declared */
                                /* ranges is computed exactly (signed corner cases, accumulator fit) */
                                /* or chosen by another objective                                    */
    int32_t stride_elems;       /* elements between the values of neighbouring slices of an A word:  */
                                /* 1 = consecutive elements (Eq. inpack); J > 1 = container-aligned  */
                                /* slices (K = 1, S a multiple of the container width c, J = S / c): */
                                /* slice n of the word for residue r holds element r + n*J, so that  */
                                /* packing is a shift and a mask of the bit-dense input (Theorem 1   */
                                /* has no cross terms when K = 1, so any assignment of elements to   */
                                /* slices is a valid packing)                                        */
    int32_t cost_milli;         /* modelled VALU issue slots per output element x 1000 (CONV1D mode  */
                                /* with fixed taps; 0 where the model does not apply)                */
} hikonv_plan_t;

/*
 * hikonv_plan -- Algorithm 1 ("Optimal Throughput Search") for a single
 * multiplier with both inputs `mult_width` bits wide: finds (N, K) maximising
 * N*K + (N-1)*(K-1) under Eq. (slice2)/(slice3) with S from Eq. (slice1).
 * signedness: OR of HIKONV_A_SIGNED, HIKONV_W_SIGNED, HIKONV_BIPOLAR.
 * out (host) receives the full plan.  Host only; touches no device.
 */
int hikonv_plan(int bits_a, int bits_w, int signedness, int mult_width, hikonv_plan_t *out);

/*
 * hikonv_plan_ex -- the same search for any mode, asymmetric widths, a fixed
 * number of kernel taps (chunked over several B words when they do not fit one)
 * and an accumulator width.  `request` (host): request fields set, result
 * fields ignored.  `out` (host) may alias request.
 */
int hikonv_plan_ex(const hikonv_plan_t *request, hikonv_plan_t *out);

/*
 * With objective = HIKONV_OBJ_MEASURED_COST, mode CONV1D and fixed taps the search
 * of hikonv_plan_ex minimises the modelled cost instead (Algorithm 1's loop with
 * another objective; Section "Maximizing Processing Throughput" states the
 * optimisation for a multiplier whose every use costs the same, which does not hold
 * for a GPU lane that also has to pack and split).  Besides the (N, K, S) of
 * Eq. (slice1)-(slice3) it considers container-aligned slices (stride_elems > 1)
 * when out_bits names an output container as wide as the input's, and with out_bits
 * set it prices the degenerate plan N = K = 1 (one value and one tap per multiply,
 * Theorem 1's smallest case) as the one-product-per-multiply kernel that runs it:
 * where no packed plan is cheaper (8-bit operands, for one) that plan is the answer.
 * In mode DNN with fixed taps the same objective prices a layer plan by the
 * multiply-accumulates it does per issue slot, splits and extra B words included
 * (Section "DNN Convolution Extension": M products accumulate before a split), and
 * searches the exact-interval slices as `tight` does: a narrower slice lets more
 * products accumulate, and on this chip the splits are what a layer pays for.
 * hikonv_plan_cost -- the model's price of a fully specified plan (request and
 * result fields set; out_bits selects the output form): VALU issue slots x 1000
 * per output element (CONV1D) or per low-bit multiply-accumulate (DNN), or a
 * negative HIKONV_E* code.  Host only.
 */
int hikonv_plan_cost(const hikonv_plan_t *plan);

/*
 * hikonv_plan_check -- exact interval check of a fully specified plan: every
 * segment sum, both packed operands and the accumulated product must fit their
 * fields for all values of the declared ranges.  Returns HIKONV_OK,
 * HIKONV_EOVERFLOW (would be inexact) or HIKONV_EINVAL.  Host only.
 */
int hikonv_plan_check(const hikonv_plan_t *plan);

/* Bytes of one bit-dense row of `len` values of `bits` bits (multiple of 4); <0 on bad bits. */
int64_t hikonv_bitdense_row_bytes(int64_t len, int bits);

/*
 * hikonv_compact -- convert [rows][len] one-value-per-byte data to the
 * bit-dense format (the paper's runtime feature compression).  bipolar != 0
 * stores bit 1 for values > 0.  out_dev must hold rows*row_bytes bytes.
 */
int hikonv_compact(const void *x_dev, int64_t rows, int64_t len, int bits, int bipolar,
                   void *out_dev, void *stream);

/*
 * hikonv_check_range -- debugging aid for the convention above that values
 * outside the declared bit range give undefined results: adds to
 * *violations_dev (a device uint32 the caller has set, normally to 0) the
 * number of the `count` one-value-per-byte entries at x_dev that are not a
 * `bits`-bit value of the given signedness ({-1,+1} entries when bipolar).  Bit-dense data
 * cannot be out of range and needs no check.  Asynchronous like every call.
 */
int hikonv_check_range(const void *x_dev, int64_t count, int bits, int is_signed, int bipolar,
                       uint32_t *violations_dev, void *stream);

/*
 * hikonv_conv1d -- packed 1-D convolution (Eq. pad_f, Theorem 2):
 *   y[r][m] = sum_k h_r[m-k] g[k],  h_r = zero extension of row r of x.
 * plan: mode CONV1D, L_A = L_B = 32, taps == `taps`, from hikonv_plan_ex.
 * x_dev: [rows][len] in x_format.  g_dev: `taps` bytes on the device, shared by
 * all rows.  y_dev: [rows][out_len] int32, out_len = len+taps-1 (FULL) or
 * len-taps+1 (VALID, 0 if len < taps).  x_dev must be 4-byte aligned, y_dev
 * 16-byte aligned (HIKONV_EINVAL otherwise); stride_elems must be 1.
 */
int hikonv_conv1d(const hikonv_plan_t *plan, const void *x_dev, int x_format, int64_t rows,
                  int64_t len, const void *g_dev, int taps, int out_mode, int32_t *y_dev,
                  void *stream);

/* Baseline: the same convolution with one v_mad_i32_i24 per low-bit product (no packing). */
int hikonv_conv1d_unpacked(int bits_a, int bits_w, int signedness, const void *x_dev, int x_format,
                           int64_t rows, int64_t len, const void *g_dev, int taps, int out_mode,
                           int32_t *y_dev, void *stream);

/*
 * hikonv_conv1d_requant -- the same convolution with the activation and the
 * requantisation of the next operator fused into the packed kernel, and the
 * result kept compressed (Section "Single convolver architecture": low-bit
 * features stay packed at run time; requantisation rule as in hikonv_epilogue):
 *   q[r][o] = min(qmax, max(y[r][o], 0) >> shift),  0 <= qmax < 2^out_bits.
 * q_dev: [rows] bit-dense rows of out_len values of out_bits bits,
 * hikonv_bitdense_row_bytes(out_len, out_bits) bytes each, 16-byte aligned;
 * bits beyond out_len in a row are written as 0.  Nothing else is written.
 * The call runs the plan it is handed.  Plans with stride_elems = 1 and N <= 12
 * whose N containers fit 32 bits run the streaming kernel; other such plans run a
 * slow general kernel.  A plan with N = K = 1 packs nothing and runs the kernel of
 * hikonv_conv1d_requant_unpacked.
 * Plans with container-aligned slices (stride_elems = S / c > 1, K = 1,
 * chunks = taps; N = 2, S = 16, or for one-bit unsigned values and taps N = 8,
 * S = 4), as hikonv_plan_ex returns them under HIKONV_OBJ_MEASURED_COST with
 * out_bits set, need: input and output containers of the same width c, taps <= 7,
 * a window of 32/c + taps - 1 containers within 64 bits, and
 * taps*max|a|*max|w| within the slice (hikonv_plan_check tells); otherwise
 * HIKONV_EINVAL.
 * N > 32 or more than 8 chunks give HIKONV_EUNSUPPORTED.
 */
int hikonv_conv1d_requant(const hikonv_plan_t *plan, const void *x_dev, int x_format, int64_t rows,
                          int64_t len, const void *g_dev, int taps, int out_mode, int shift, int qmax,
                          int out_bits, void *q_dev, void *stream);

/* Baseline for hikonv_conv1d_requant: one v_mad_i32_i24 per low-bit product, same output. */
int hikonv_conv1d_requant_unpacked(int bits_a, int bits_w, int signedness, const void *x_dev,
                                   int x_format, int64_t rows, int64_t len, const void *g_dev,
                                   int taps, int out_mode, int shift, int qmax, int out_bits,
                                   void *q_dev, void *stream);

/*
 * Weight pre-packing (Section "Basic HiKonv Operations": weights can be packed
 * offline).  For a layer W[Co][C][Kh][Kw] (one value per byte) builds, per
 * (co, ci, kh, chunk), the word B = sum_k g[k] 2^(S k) of the reversed kernel
 * row g = W[co][ci][kh][Kw-1:0] (Eq. I_PRIME).  packed_dev must hold
 * hikonv_packed_weights_bytes() bytes.
 */
size_t hikonv_packed_weights_bytes(const hikonv_plan_t *plan, int Co, int C, int Kh, int Kw);
int hikonv_pack_weights(const hikonv_plan_t *plan, const void *w_dev, int Co, int C, int Kh, int Kw,
                        void *packed_dev, void *stream);

/*
 * hikonv_conv2d -- packed DNN convolution layer (Eq. conv_org, Theorem 3),
 * cross-correlation with zero padding `pad` and `stride`:
 *   O[n][co][h][w] = sum_{ci,kh,kw} Ipad[n][ci][h s+kh][w s+kw] W[co][ci][kh][kw].
 * plan: mode DNN, (L_A,L_B,L_acc) = (32,32,64) or (24,24,32), and
 *   taps == Kw: rows are convolved at column stride 1 and every stride-th result
 *     is stored (0 <= pad <= Kw-1); or
 *   stride > 1 and taps == ceil(Kw/stride) (!= Kw): polyphase form.  The s column
 *     phases of each padded input row are packed as separate channels and phase p
 *     meets the kernel taps p, p+s, p+2s, ... (zero beyond Kw), so that
 *       O[..][w] = sum_p sum_j Ipad_p[w+j] W[..][j s+p],  Ipad_p[i] = Ipad[s i+p]:
 *     a sum of stride-1 row convolutions with ceil(Kw/s) taps, added in the packed
 *     domain like channels are (Theorem 3); M counts (channel, kernel row, phase)
 *     products.  No multiply is spent on discarded columns.  Any pad >= 0.  Not
 *     for {-1,+1} layers.
 * x_dev: NCHW in x_format (bit-dense rows are the W rows).  y_dev: NCHW int32.
 * workspace_dev: at least hikonv_conv2d_workspace_bytes() bytes, 256-byte aligned.
 * hikonv_conv2d packs the raw weights w_dev ([Co][C][Kh][Kw], one per byte) into
 * the workspace on every call; hikonv_conv2d_prepacked takes weights already
 * packed by hikonv_pack_weights (taps == Kw) or hikonv_pack_weights_ex (either
 * form) with the same plan and stride.
 */
size_t hikonv_conv2d_workspace_bytes(const hikonv_plan_t *plan, int N, int C, int H, int W, int Co,
                                     int Kh, int Kw, int stride, int pad, int prepacked);
int hikonv_conv2d(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C, int H,
                  int W, const void *w_dev, int Co, int Kh, int Kw, int stride, int pad,
                  void *workspace_dev, size_t workspace_bytes, int32_t *y_dev, void *stream);
int hikonv_conv2d_prepacked(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C,
                            int H, int W, const void *w_packed_dev, int Co, int Kh, int Kw, int stride,
                            int pad, void *workspace_dev, size_t workspace_bytes, int32_t *y_dev,
                            void *stream);

/*
 * hikonv_conv2d_noalloc -- hikonv_conv2d for callers that cannot allocate device
 * memory and have no workspace to hand over: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * error codes as hikonv_conv2d (raw weights w_dev, packed on every call) without
 * the workspace: packed activations, term offsets and packed weights go to a fixed
 * array of HIKONV_NOALLOC_SCRATCH_BYTES bytes that is part of the library's device
 * code (each GPU the library runs on holds one copy until the process ends).  The
 * call allocates and frees nothing and does not synchronise.
 *   - x_format: HIKONV_FMT_INT8 or HIKONV_FMT_BITDENSE (HIKONV_FMT_PACKED: HIKONV_EINVAL).
 *   - A layer whose hikonv_conv2d_workspace_bytes(..., prepacked = 0) exceeds
 *     HIKONV_NOALLOC_SCRATCH_BYTES returns HIKONV_ESCRATCH; nothing is launched.
 *   - All calls on one GPU share that GPU's array: calls that may overlap on one GPU
 *     (different streams, several host threads) race; calls on one stream are ordered.
 *     The array keeps the last call's contents; every call writes all it reads.
 */
#define HIKONV_NOALLOC_SCRATCH_BYTES (8u << 20)
int hikonv_conv2d_noalloc(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C, int H,
                          int W, const void *w_dev, int Co, int Kh, int Kw, int stride, int pad,
                          int32_t *y_dev, void *stream);

/*
 * Weight pre-packing for any layer form: Kd kernel depth slices (1 for a 2-D
 * layer) and the column stride the layer will be called with (it selects the
 * polyphase form exactly as in hikonv_conv2d: plan->taps == ceil(Kw/stride)).
 * w_dev: [Co][C][Kd][Kh][Kw], one value per byte.
 */
size_t hikonv_packed_weights_bytes_ex(const hikonv_plan_t *plan, int Co, int C, int Kd, int Kh, int Kw,
                                      int stride);
int hikonv_pack_weights_ex(const hikonv_plan_t *plan, const void *w_dev, int Co, int C, int Kd, int Kh,
                           int Kw, int stride, void *packed_dev, void *stream);

/*
 * hikonv_conv3d -- packed three-dimensional convolution layer (the paper notes
 * at the end of Section "General purpose processors" that the DNN extension
 * carries to higher-dimensional convolutions): Eq. conv_org with one more axis,
 *   O[n][co][d][h][w] = sum_{ci,kd,kh,kw} Ipad[n][ci][d s+kd][h s+kh][w s+kw] W[co][ci][kd][kh][kw],
 * zero padding `pad` on all six sides, one stride for the three axes.  Every
 * (ci, kd, kh) input row is one more 1-D row convolution accumulated in the
 * packed domain (Theorem 3 with the kernel depth as a further outer sum); M
 * counts (ci, kd, kh[, phase]) products.  plan as for hikonv_conv2d (both stride
 * forms; not {-1,+1}).  x_dev: NCDHW in x_format (INT8 or BITDENSE).  w_dev:
 * [Co][C][Kd][Kh][Kw] one value per byte when prepacked == 0, else the output of
 * hikonv_pack_weights_ex.  y_dev: NCDHW int32.  workspace as for hikonv_conv2d,
 * sized by hikonv_conv3d_workspace_bytes().
 */
size_t hikonv_conv3d_workspace_bytes(const hikonv_plan_t *plan, int N, int C, int D, int H, int W, int Co,
                                     int Kd, int Kh, int Kw, int stride, int pad, int prepacked);
int hikonv_conv3d(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C, int D, int H,
                  int W, const void *w_dev, int prepacked, int Co, int Kd, int Kh, int Kw, int stride,
                  int pad, void *workspace_dev, size_t workspace_bytes, int32_t *y_dev, void *stream);

/* Baseline: direct layer, one v_mad_i32_i24 per product.  x_dev and w_dev one value per byte. */
int hikonv_conv2d_unpacked(int bits_a, int bits_w, int signedness, const void *x_dev, int N, int C,
                           int H, int W, const void *w_dev, int Co, int Kh, int Kw, int stride, int pad,
                           int32_t *y_dev, void *stream);

/*
 * hikonv_epilogue -- the un-accelerated rest of a layer in the complete-model
 * experiment (Section "Complete model evaluation"): ReLU, requantise
 * q = min(qmax, max(acc,0) >> shift), optional 2x2/stride-2 max-pool, written
 * as the next layer's activations in out_format with out_bits-bit values.
 * acc_dev: NCHW int32.  out_dev: [N][C][Ho][Wo] rows of Wo values.
 */
int hikonv_epilogue(const int32_t *acc_dev, int N, int C, int H, int W, int shift, int qmax, int pool,
                    int out_bits, int out_format, void *out_dev, void *stream);

/*
 * hikonv_epilogue_pack -- the same epilogue (ReLU, q = min(qmax, max(acc,0) >> shift),
 * optional 2x2/stride-2 max-pool) writing its result directly as the packed
 * activation words of the NEXT layer (Section "Basic HiKonv Operations":
 * features are packed at run time - here by their producer, so the next layer
 * needs no packing pass).  acc_dev: NCHW int32 [N][C][H][W].  The next layer is
 * described by its plan (unsigned activations of next_plan->bits_a bits,
 * qmax < 2^bits_a) and its geometry: input [N][C][H'][W'] with H' = H/2, W' = W/2
 * when pool, else H, W.  next_workspace_dev: the workspace later passed to
 * hikonv_conv2d / hikonv_conv2d_prepacked for that layer, which must then be
 * called with x_format = HIKONV_FMT_PACKED and the same plan and geometry.
 */
int hikonv_epilogue_pack(const int32_t *acc_dev, int N, int C, int H, int W, int shift, int qmax, int pool,
                         const hikonv_plan_t *next_plan, int next_Co, int next_Kh, int next_Kw,
                         int next_stride, int next_pad, void *next_workspace_dev,
                         size_t next_workspace_bytes, void *stream);

/*
 * hikonv_conv2d_fused -- one kernel per layer of a chain (Section "Complete model
 * evaluation": a layer is the convolution followed by activation and pooling).  The
 * packed stride-1 layer of hikonv_conv2d_prepacked whose store stage also applies the
 * epilogue of hikonv_epilogue_pack (q = min(qmax, max(acc, 0) >> shift), optional
 * 2x2/stride-2 max-pool) and writes the result directly as the NEXT layer's packed
 * activation words into next_workspace_dev, which that layer then takes with
 * x_format = HIKONV_FMT_PACKED (same next_plan and geometry: input [N][Co][H'][W'],
 * H' = Ho/2, W' = Wo/2 when pool, else Ho, Wo).  Neither the int32 accumulators nor
 * a packing pass touch memory between the two layers.
 *   y_dev: NCHW int32 accumulators of this layer, or NULL to skip storing them.
 *   next_plan NULL: no following layer (y_dev required); shift, qmax, pool and the
 *   next_* arguments are ignored.
 *   x_format INT8 / BITDENSE: where a workgroup's share of the input is small (at
 *   most 2048 packed words: few input channels), or where plan->kernel ==
 *   HIKONV_KERNEL_LDS asks for it and the rows fit its LDS, every workgroup packs
 *   the input rows it needs into LDS itself (one kernel for the whole layer;
 *   workspace_dev is not used and may be NULL); otherwise the input is packed into
 *   workspace_dev by a first kernel, as in hikonv_conv2d (HIKONV_EWORKSPACE if it
 *   is missing).
 *   PACKED: workspace_dev already holds the packed input.
 * Covers plans with (L_A, L_B, L_acc) = (32, 32, 64) and N <= 4, rows of at most
 * 16 (8 with pooling) 63-block segments, and layers whose per-workgroup LDS (the
 * B words of eight output channels, an int32 tile of rows x 8 x Wo) stays within
 * 64 KiB; next plans with unsigned activations; anything else returns
 * HIKONV_EUNSUPPORTED and the caller chains hikonv_conv2d_prepacked and
 * hikonv_epilogue_pack instead.
 */
int hikonv_conv2d_fused(const hikonv_plan_t *plan, const void *x_dev, int x_format, int N, int C, int H,
                        int W, const void *w_packed_dev, int Co, int Kh, int Kw, int pad,
                        void *workspace_dev, size_t workspace_bytes, int32_t *y_dev, int shift, int qmax,
                        int pool, const hikonv_plan_t *next_plan, int next_Co, int next_Kh, int next_Kw,
                        int next_pad, void *next_workspace_dev, size_t next_workspace_bytes, void *stream);

const char *hikonv_strerror(int code);
int hikonv_last_hip_error(void); /* hipError_t of the most recent failing HIP call in this thread */

#ifdef __cplusplus
}
#endif
#endif /* HIKONV_H */

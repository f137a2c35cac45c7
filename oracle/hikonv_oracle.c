/*
 * HiKonv oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, obviously-correct CPU definitions of everything the HIP path
 * computes.  HiKonv reaches exactly the result of an ordinary convolution
 * (Theorems 1-3 of the paper are equalities), so the oracle is the ordinary
 * definition written out as loops, accumulated in int64 and narrowed to int32
 * only after a range check.  There is no packing, blocking, fusion or
 * reordering here, and no code is shared with the HIP library.
 *
 * Only tests, the smoke check and the cpu_baseline leg of the benchmark may
 * call into this file.
 *
 * Pins (see tests/test_oracle_pins.py): numpy.convolve / torch conv2d /
 * torch max_pool2d on CPU, brute-force Python loops on tiny shapes, the
 * paper's worked F_{3,2} example, linearity and shift invariants.
 * Unpinned by the paper (it defines none of them): the requantisation rule,
 * the {-1,+1} value set of "binary" layers, and the bit-dense container
 * layout; they are pinned only by the definitions written here.
 */
#include <stdint.h>
#include <stddef.h>
#include <limits.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of threads the parallel loops below will use (1 without OpenMP). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * 1-D convolution, Section "1-D Convolution", Eq. (pad_f0) and Eq. (pad_f):
 *   h = zero extension of f,   y[m] = sum_{k=0}^{K-1} h[m-k] * g[k].
 * mode 0 (FULL):  m = 0 .. len+K-2          (len+K-1 outputs per row)
 * mode 1 (VALID): m = K-1 .. len-1          (len-K+1 outputs per row, 0 if len<K)
 * f is [rows][len], the kernel g[K] is shared by all rows, y is
 * [rows][out_len].  Values are one per byte: read as uint8 when the operand's
 * `*_unsigned` flag is set (so unsigned 8-bit values 0..255 are representable),
 * as int8 otherwise.  Returns 0, or -1 if a sum does not fit int32.
 */
static inline int64_t byte_value(const int8_t *p, int64_t i, int is_unsigned)
{
    return is_unsigned ? (int64_t)(uint8_t)p[i] : (int64_t)p[i];
}

int oracle_conv1d(const int8_t *f, int f_unsigned, int64_t rows, int64_t len,
                  const int8_t *g, int g_unsigned, int K, int mode, int32_t *y)
{
    int64_t m_first = (mode == 1) ? (int64_t)K - 1 : 0;
    int64_t m_last = (mode == 1) ? len - 1 : len + K - 2;   /* inclusive */
    int64_t out_len = m_last - m_first + 1;
    int bad = 0;
    if (out_len <= 0) return 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t r = 0; r < rows; ++r) {
        const int8_t *fr = f + r * len;
        int32_t *yr = y + r * out_len;
        for (int64_t m = m_first; m <= m_last; ++m) {
            int64_t acc = 0;
            for (int k = 0; k < K; ++k) {
                int64_t n = m - k;
                int64_t h = (n >= 0 && n < len) ? byte_value(fr, n, f_unsigned) : 0;
                acc += h * byte_value(g, k, g_unsigned);
            }
            if (acc > INT32_MAX || acc < INT32_MIN) bad |= 1;
            yr[m - m_first] = (int32_t)acc;
        }
    }
    return bad ? -1 : 0;
}

/*
 * DNN convolution layer, Section "DNN Convolution Extension", Eq. (conv_org),
 * extended with zero padding `pad` on all four sides (zero extension as in
 * Eq. (pad_f0)) and an output stride:
 *   O[n][co][h][w] = sum_{ci,kh,kw} Ipad[n][ci][h*s+kh][w*s+kw] * W[co][ci][kh][kw]
 * with Ho = (H + 2*pad - Kh)/s + 1, Wo likewise.  This is a cross-correlation
 * (the kernel is not flipped).  x is NCHW, w is [Co][C][Kh][Kw], y is NCHW.
 * Returns 0, or -1 if a sum does not fit int32.
 */
int oracle_conv2d(const int8_t *x, int x_unsigned, int N, int C, int H, int W,
                  const int8_t *w, int w_unsigned, int Co, int Kh, int Kw,
                  int stride, int pad, int32_t *y)
{
    int Ho = (H + 2 * pad - Kh) / stride + 1;
    int Wo = (W + 2 * pad - Kw) / stride + 1;
    int bad = 0;
    if (H + 2 * pad < Kh || W + 2 * pad < Kw) return 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : bad)
    for (int n = 0; n < N; ++n) {
        for (int co = 0; co < Co; ++co) {
            for (int h = 0; h < Ho; ++h) {
                for (int wo = 0; wo < Wo; ++wo) {
                    int64_t acc = 0;
                    for (int ci = 0; ci < C; ++ci) {
                        for (int kh = 0; kh < Kh; ++kh) {
                            for (int kw = 0; kw < Kw; ++kw) {
                                int ih = h * stride + kh - pad;
                                int iw = wo * stride + kw - pad;
                                int64_t v = 0;
                                if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                                    v = byte_value(x, (((int64_t)n * C + ci) * H + ih) * W + iw, x_unsigned);
                                acc += v * byte_value(w, (((int64_t)co * C + ci) * Kh + kh) * Kw + kw, w_unsigned);
                            }
                        }
                    }
                    if (acc > INT32_MAX || acc < INT32_MIN) bad |= 1;
                    y[(((int64_t)n * Co + co) * Ho + h) * Wo + wo] = (int32_t)acc;
                }
            }
        }
    }
    return bad ? -1 : 0;
}

/*
 * Three-dimensional convolution layer: the paper notes that the DNN extension carries
 * over to higher-dimensional convolutions (end of Section "General purpose processors");
 * the definition is Eq. (conv_org) with one more spatial axis, zero padding `pad` on all
 * six sides and one output stride for the three axes:
 *   O[n][co][d][h][w] = sum_{ci,kd,kh,kw} Ipad[n][ci][d*s+kd][h*s+kh][w*s+kw] * W[co][ci][kd][kh][kw]
 * with Do = (D + 2*pad - Kd)/s + 1, Ho, Wo likewise (cross-correlation, kernel not
 * flipped).  x is NCDHW, w is [Co][C][Kd][Kh][Kw], y is NCDHW.
 * Returns 0, or -1 if a sum does not fit int32.
 */
int oracle_conv3d(const int8_t *x, int x_unsigned, int N, int C, int D, int H, int W,
                  const int8_t *w, int w_unsigned, int Co, int Kd, int Kh, int Kw,
                  int stride, int pad, int32_t *y)
{
    int Do = (D + 2 * pad - Kd) / stride + 1;
    int Ho = (H + 2 * pad - Kh) / stride + 1;
    int Wo = (W + 2 * pad - Kw) / stride + 1;
    int bad = 0;
    if (D + 2 * pad < Kd || H + 2 * pad < Kh || W + 2 * pad < Kw) return 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : bad)
    for (int n = 0; n < N; ++n) {
        for (int co = 0; co < Co; ++co) {
            for (int d = 0; d < Do; ++d) {
                for (int h = 0; h < Ho; ++h) {
                    for (int wo = 0; wo < Wo; ++wo) {
                        int64_t acc = 0;
                        for (int ci = 0; ci < C; ++ci) {
                            for (int kd = 0; kd < Kd; ++kd) {
                                for (int kh = 0; kh < Kh; ++kh) {
                                    for (int kw = 0; kw < Kw; ++kw) {
                                        int id = d * stride + kd - pad;
                                        int ih = h * stride + kh - pad;
                                        int iw = wo * stride + kw - pad;
                                        int64_t v = 0;
                                        if (id >= 0 && id < D && ih >= 0 && ih < H && iw >= 0 && iw < W)
                                            v = byte_value(x, ((((int64_t)n * C + ci) * D + id) * H + ih) * W + iw,
                                                           x_unsigned);
                                        acc += v * byte_value(w, ((((int64_t)co * C + ci) * Kd + kd) * Kh + kh) * Kw + kw,
                                                              w_unsigned);
                                    }
                                }
                            }
                        }
                        if (acc > INT32_MAX || acc < INT32_MIN) bad |= 1;
                        y[((((int64_t)n * Co + co) * Do + d) * Ho + h) * Wo + wo] = (int32_t)acc;
                    }
                }
            }
        }
    }
    return bad ? -1 : 0;
}

/*
 * Activation + requantisation between layers of the complete-model experiment
 * (Section "Complete model evaluation": all calculations in integers).  The
 * paper gives no rule; the reading used here is
 *   q = min(qmax, max(acc, 0) >> shift)
 * i.e. ReLU, an arithmetic right shift by a fixed per-layer amount, and a
 * clamp to the unsigned range [0, qmax].
 */
void oracle_relu_requant(const int32_t *acc, int64_t count, int shift, int qmax, int8_t *q)
{
    for (int64_t i = 0; i < count; ++i) {
        int64_t v = acc[i];
        if (v < 0) v = 0;
        v >>= shift;
        if (v > qmax) v = qmax;
        q[i] = (int8_t)v;
    }
}

/* 2x2 max pooling, stride 2, on NCHW int8 (odd trailing row/column dropped). */
void oracle_maxpool2x2(const int8_t *x, int N, int C, int H, int W, int8_t *y)
{
    int Ho = H / 2, Wo = W / 2;
    for (int64_t nc = 0; nc < (int64_t)N * C; ++nc) {
        for (int h = 0; h < Ho; ++h) {
            for (int w = 0; w < Wo; ++w) {
                int8_t best = x[(nc * H + 2 * h) * W + 2 * w];
                for (int dh = 0; dh < 2; ++dh)
                    for (int dw = 0; dw < 2; ++dw) {
                        int8_t v = x[(nc * H + 2 * h + dh) * W + 2 * w + dw];
                        if (v > best) best = v;
                    }
                y[(nc * Ho + h) * Wo + w] = best;
            }
        }
    }
}

/*
 * Bit-dense ("compressed") storage of low-bitwidth values, Section "Single
 * convolver architecture" (unused bits discarded).  The container layout is
 * this build's own definition: each row of `len` values is a little-endian bit
 * stream in which value i occupies bits [c*i, c*i+c) with container width
 * c = 1,2,4,4,8,8,8,8 for b = 1..8 bits; the value's low b bits are stored
 * (two's complement for signed values) and the remaining c-b bits are zero.
 * Rows are padded with zero bits to a multiple of 4 bytes.
 */
int oracle_container_bits(int bits)
{
    static const int c[9] = {0, 1, 2, 4, 4, 8, 8, 8, 8};
    return (bits >= 1 && bits <= 8) ? c[bits] : 0;
}

int64_t oracle_bitdense_row_bytes(int64_t len, int bits)
{
    int64_t nbits = len * oracle_container_bits(bits);
    return ((nbits + 31) / 32) * 4;
}

void oracle_bitdense_pack(const int8_t *v, int64_t rows, int64_t len, int bits, uint8_t *out)
{
    int c = oracle_container_bits(bits);
    int64_t rb = oracle_bitdense_row_bytes(len, bits);
    for (int64_t i = 0; i < rows * rb; ++i) out[i] = 0;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t i = 0; i < len; ++i) {
            unsigned field = (unsigned)(uint8_t)v[r * len + i] & ((1u << bits) - 1u);
            for (int t = 0; t < bits; ++t) {
                int64_t bit = i * c + t;
                if ((field >> t) & 1u) out[r * rb + bit / 8] |= (uint8_t)(1u << (bit % 8));
            }
        }
    }
}

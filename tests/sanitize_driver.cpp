// Host-only driver built with -fsanitize=address,undefined -fno-sanitize-recover by
// tests/test_sanitizers.py: it links the planner (csrc/hikonv_plan.cpp) and the C oracle and
// walks the planner's whole request space and the oracle's edge shapes, so that any
// out-of-bounds access, shift beyond a type's width or signed overflow aborts the run.
// The oracle results are also checked against values fixed by hand and by exactly sized
// heap buffers (an access one element outside any of them is an ASan error).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/hikonv.h"

extern "C" {
int oracle_conv1d(const int8_t *f, int f_unsigned, int64_t rows, int64_t len, const int8_t *g, int g_unsigned, int K,
                  int mode, int32_t *y);
int oracle_conv2d(const int8_t *x, int x_unsigned, int N, int C, int H, int W, const int8_t *w, int w_unsigned, int Co,
                  int Kh, int Kw, int stride, int pad, int32_t *y);
int oracle_conv3d(const int8_t *x, int x_unsigned, int N, int C, int D, int H, int W, const int8_t *w, int w_unsigned,
                  int Co, int Kd, int Kh, int Kw, int stride, int pad, int32_t *y);
void oracle_relu_requant(const int32_t *acc, int64_t count, int shift, int qmax, int8_t *q);
void oracle_maxpool2x2(const int8_t *x, int N, int C, int H, int W, int8_t *y);
int64_t oracle_bitdense_row_bytes(int64_t len, int bits);
void oracle_bitdense_pack(const int8_t *v, int64_t rows, int64_t len, int bits, uint8_t *out);
}

static void fail(const char *what)
{
    std::fprintf(stderr, "sanitize_driver: %s\n", what);
    std::exit(3);
}

static uint64_t lcg(uint64_t &s)
{
    s = s * 6364136223846793005ull + 1442695040888963407ull;
    return s >> 33;
}

static long planner_sweep()
{
    static const int widths[][3] = {{27, 18, 0}, {32, 32, 64}, {24, 24, 32}, {64, 64, 0}, {1, 1, 0}, {64, 1, 128}, {8, 64, 16}};
    static const int conv_taps[] = {1, 2, 3, 5, 7, 16, 63, 64};
    static const int dnn_m[] = {1, 7, 170, 1 << 20};
    long ok = 0, calls = 0;
    hikonv_plan_t out;
    for (int p = 1; p <= 8; ++p)
        for (int q = 1; q <= 8; ++q)
            for (int sg = 0; sg < 4; ++sg)
                for (const auto &w : widths)
                    for (int tight = 0; tight < 2; ++tight)
                        for (int obj = 0; obj < 2; ++obj) {
                            hikonv_plan_t in = {};
                            in.bits_a = p;
                            in.bits_w = q;
                            in.a_signed = sg & 1;
                            in.w_signed = sg >> 1;
                            in.L_A = w[0];
                            in.L_B = w[1];
                            in.L_acc = w[2];
                            in.tight = tight;
                            in.objective = obj;
                            in.mode = HIKONV_MODE_SINGLE;
                            for (int taps : {0, 3}) {
                                in.taps = taps;
                                ++calls;
                                if (hikonv_plan_ex(&in, &out) == HIKONV_OK) ok += hikonv_plan_check(&out) == HIKONV_OK;
                            }
                            in.mode = HIKONV_MODE_CONV1D;
                            for (int taps : conv_taps)
                                for (int ob : {0, p}) {
                                    in.taps = taps;
                                    in.out_bits = ob;
                                    ++calls;
                                    if (hikonv_plan_ex(&in, &out) == HIKONV_OK) {
                                        ok += hikonv_plan_check(&out) == HIKONV_OK;
                                        (void)hikonv_plan_cost(&out);
                                    }
                                }
                            in.out_bits = 0;
                            in.mode = HIKONV_MODE_DNN;
                            for (int taps : {1, 3, 7, 64})
                                for (int m : dnn_m)
                                    for (int max_n : {0, 8}) {
                                        in.taps = taps;
                                        in.M = m;
                                        in.max_N = max_n;
                                        ++calls;
                                        if (hikonv_plan_ex(&in, &out) == HIKONV_OK) ok += hikonv_plan_check(&out) == HIKONV_OK;
                                    }
                            in.max_N = 0;
                        }
    // M chosen by the planner (512 trials per call): a thinner grid
    for (int p = 1; p <= 8; p += 3)
        for (int q = 1; q <= 8; q += 2)
            for (int sg = 0; sg < 4; ++sg)
                for (int wide = 0; wide < 2; ++wide)
                    for (int taps : {1, 3, 5}) {
                        hikonv_plan_t in = {};
                        in.bits_a = p;
                        in.bits_w = q;
                        in.a_signed = sg & 1;
                        in.w_signed = sg >> 1;
                        in.L_A = in.L_B = wide ? 32 : 24;
                        in.L_acc = wide ? 64 : 32;
                        in.mode = HIKONV_MODE_DNN;
                        in.taps = taps;
                        in.max_N = HIKONV_LAYER_MAX_N;
                        ++calls;
                        if (hikonv_plan_ex(&in, &out) == HIKONV_OK) ok += hikonv_plan_check(&out) == HIKONV_OK;
                    }
    // {-1,+1} plans and the headline entry point
    for (int width : {24, 27, 32, 64}) {
        ++calls;
        if (hikonv_plan(1, 1, HIKONV_BIPOLAR, width, &out) == HIKONV_OK) ok += 1;
        for (int b = 1; b <= 8; ++b)
            for (int sg = 0; sg < 4; ++sg) {
                ++calls;
                if (hikonv_plan(b, b, sg, width, &out) == HIKONV_OK) ok += 1;
            }
    }
    // plans handed in by a caller: every field combination the check must survive
    uint64_t s = 1;
    for (int i = 0; i < 200000; ++i) {
        hikonv_plan_t pl = {};
        int32_t *f = reinterpret_cast<int32_t *>(&pl);
        for (size_t k = 0; k < sizeof(pl) / 4; ++k) f[k] = (int32_t)(lcg(s) % 70) - 2;
        (void)hikonv_plan_check(&pl);
        (void)hikonv_plan_cost(&pl);
    }
    std::printf("planner: %ld requests, %ld plans found and accepted by hikonv_plan_check\n", calls, ok);
    if (ok < calls / 4) fail("implausibly few plans");
    return ok;
}

static void oracle_edges()
{
    // 1-D: the worked F_{3,2} example (f = 11, 9, 7 reversed order is the paper's; here the plain values)
    {
        const int8_t f[3] = {7, 9, 11}, g[2] = {2, 3};
        std::vector<int32_t> y(4);
        if (oracle_conv1d(f, 1, 1, 3, g, 1, 2, 0, y.data()) != 0) fail("conv1d rc");
        const int32_t want[4] = {14, 39, 49, 33};
        for (int i = 0; i < 4; ++i)
            if (y[i] != want[i]) fail("conv1d worked example");
    }
    uint64_t s = 7;
    for (int len : {1, 2, 3, 17, 64})
        for (int K : {1, 2, 3, 7, 64})
            for (int mode = 0; mode < 2; ++mode)
                for (int uns = 0; uns < 2; ++uns) {
                    const int rows = 3;
                    const int out_len = mode ? (len - K + 1 > 0 ? len - K + 1 : 0) : len + K - 1;
                    std::vector<int8_t> f((size_t)rows * len), g(K);
                    for (auto &v : f) v = (int8_t)lcg(s);
                    for (auto &v : g) v = (int8_t)lcg(s);
                    std::vector<int32_t> y((size_t)rows * out_len);
                    if (oracle_conv1d(f.data(), uns, rows, len, g.data(), uns, K, mode, y.data()) != 0) fail("conv1d rc");
                    // a delta kernel returns the row itself (shifted): detects flipped or offset indexing
                    std::vector<int8_t> d(K, 0);
                    d[K - 1] = 1;
                    if (oracle_conv1d(f.data(), uns, rows, len, d.data(), 0, K, mode, y.data()) != 0) fail("conv1d rc");
                    for (int r = 0; r < rows; ++r)
                        for (int o = 0; o < out_len; ++o) {
                            const int m = o + (mode ? K - 1 : 0), n = m - (K - 1);
                            const int32_t want = n >= 0 && n < len ? (uns ? (int32_t)(uint8_t)f[(size_t)r * len + n] : (int32_t)f[(size_t)r * len + n]) : 0;
                            if (y[(size_t)r * out_len + o] != want) fail("conv1d delta kernel");
                        }
                }
    // 2-D / 3-D: all-ones input and kernel count the taps inside the image (padding, stride, ragged sizes)
    for (int H : {1, 4, 7})
        for (int W : {1, 5, 9})
            for (int Kk : {1, 3, 5})
                for (int stride : {1, 2, 3})
                    for (int pad : {0, 1, 2}) {
                        if (H + 2 * pad < Kk || W + 2 * pad < Kk) continue;
                        const int N = 2, C = 3, Co = 2;
                        const int Ho = (H + 2 * pad - Kk) / stride + 1, Wo = (W + 2 * pad - Kk) / stride + 1;
                        std::vector<int8_t> x((size_t)N * C * H * W, 1), w((size_t)Co * C * Kk * Kk, 1);
                        std::vector<int32_t> y((size_t)N * Co * Ho * Wo);
                        if (oracle_conv2d(x.data(), 0, N, C, H, W, w.data(), 0, Co, Kk, Kk, stride, pad, y.data()) != 0)
                            fail("conv2d rc");
                        for (int h = 0; h < Ho; ++h)
                            for (int ww = 0; ww < Wo; ++ww) {
                                int cnt = 0;
                                for (int kh = 0; kh < Kk; ++kh)
                                    for (int kw = 0; kw < Kk; ++kw) {
                                        const int ih = h * stride + kh - pad, iw = ww * stride + kw - pad;
                                        cnt += ih >= 0 && ih < H && iw >= 0 && iw < W;
                                    }
                                if (y[(size_t)h * Wo + ww] != cnt * C) fail("conv2d tap count");
                            }
                        const int D = 3;
                        if (D + 2 * pad < Kk) continue;
                        const int Do = (D + 2 * pad - Kk) / stride + 1;
                        std::vector<int8_t> x3((size_t)N * C * D * H * W, 1), w3((size_t)Co * C * Kk * Kk * Kk, 1);
                        std::vector<int32_t> y3((size_t)N * Co * Do * Ho * Wo);
                        if (oracle_conv3d(x3.data(), 0, N, C, D, H, W, w3.data(), 0, Co, Kk, Kk, Kk, stride, pad, y3.data()) != 0)
                            fail("conv3d rc");
                    }
    // overflow report instead of a wrapped sum: 2^24 products of 127 * 127 do not fit int32
    {
        const int C = 1 << 15, Kk = 23;     // 2^15 * 529 * 16129 > 2^31
        std::vector<int8_t> x((size_t)C * Kk * Kk, 127), w((size_t)C * Kk * Kk, 127);
        int32_t y = 0;
        if (oracle_conv2d(x.data(), 0, 1, C, Kk, Kk, w.data(), 0, 1, Kk, Kk, 1, 0, &y) == 0) fail("conv2d overflow not reported");
    }
    // epilogue pieces on exactly sized buffers, extreme values
    {
        const int32_t acc[6] = {INT32_MIN, -1, 0, 15, 16, INT32_MAX};
        int8_t q[6];
        for (int shift : {0, 1, 31}) oracle_relu_requant(acc, 6, shift, 15, q);
        oracle_relu_requant(acc, 6, 0, 15, q);
        const int8_t want[6] = {0, 0, 0, 15, 15, 15};
        for (int i = 0; i < 6; ++i)
            if (q[i] != want[i]) fail("relu_requant");
        for (int H : {1, 2, 5})
            for (int W : {1, 2, 7}) {
                std::vector<int8_t> x((size_t)2 * H * W), y((size_t)2 * (H / 2) * (W / 2));
                for (auto &v : x) v = (int8_t)(lcg(s) & 15);
                oracle_maxpool2x2(x.data(), 1, 2, H, W, y.data());
            }
        for (int bits = 1; bits <= 8; ++bits)
            for (int len : {0, 1, 7, 8, 9, 31, 32, 33, 100}) {
                std::vector<int8_t> v((size_t)2 * len);
                for (auto &e : v) e = (int8_t)lcg(s);
                std::vector<uint8_t> out((size_t)2 * oracle_bitdense_row_bytes(len, bits));
                oracle_bitdense_pack(v.data(), 2, len, bits, out.data());
            }
    }
    std::printf("oracle: edge shapes ran clean\n");
}

int main()
{
    planner_sweep();
    oracle_edges();
    std::printf("sanitize_driver: ok\n");
    return 0;
}

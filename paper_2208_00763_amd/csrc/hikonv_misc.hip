// Small kernels around the hot path: runtime feature compression to the bit-dense format,
// the un-accelerated layer epilogue of the complete-model experiment, roofline
// micro-benchmarks, and a lane-exchange self check.
#include "hikonv_device.h"
#include "../../include/hikonv_bench.h"
#include "hikonv_launch.h"

namespace hikonv {
namespace {

// one thread per output dword of the bit-dense stream
__global__ __launch_bounds__(256) void k_compact(const uint8_t *x, int64_t rows, int64_t len, int b, int c,
                                                 int bipolar, uint32_t *out, int64_t row_dwords)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * row_dwords) return;
    const int64_t r = idx / row_dwords, j = idx % row_dwords;
    const int per = 32 / c;
    const uint32_t vmask = (1u << b) - 1u;
    uint32_t word = 0;
    for (int t = 0; t < per; ++t) {
        int64_t i = j * per + t;
        if (i < len) {
            uint8_t v = x[r * len + i];
            uint32_t f = bipolar ? ((int8_t)v > 0 ? 1u : 0u) : ((uint32_t)v & vmask);
            word |= f << (t * c);
        }
    }
    out[idx] = word;
}

// Runtime feature compression, streaming form (Section "Single convolver architecture": the
// unused bits of quantised features are dropped in storage).  Rows whose bytes start on dword
// boundaries (x and len multiples of 4).  A thread turns 16 consecutive values (one 16-byte
// load; 32 values for one-bit containers) into 16*C bits with a few shift-or steps per input
// dword and stores them as one 16/8/4-byte vector; grid.y walks the rows, so nothing is divided.
typedef uint32_t u32x4_dw4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2_dw4 __attribute__((ext_vector_type(2), aligned(4)));

// the C-bit containers of the four byte values of w, gathered into the low 4*C bits
template <int C>
__device__ __forceinline__ uint32_t gather_bytes(uint32_t w, uint32_t vmask4, int bipolar)
{
    if (bipolar) {
        // bit 1 for values > 0 (as int8): some low bit set and the sign bit clear
        const uint32_t nz = ((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) & 0x80808080u;
        w = (nz & ~w) >> 7;
    } else {
        w &= vmask4;
    }
    if (C == 8) return w;
    if (C == 4) {
        w = (w | (w >> 4)) & 0x00ff00ffu;
        return (w | (w >> 8)) & 0xffffu;
    }
    if (C == 2) {
        w = (w | (w >> 6)) & 0x000f000fu;
        return (w | (w >> 12)) & 0xffu;
    }
    // C == 1: bit 0 of byte i goes to bit 28 + i of the product (all partial products fall on distinct bits)
    return ((w & 0x01010101u) * 0x10204080u) >> 28;
}

template <int C>
__global__ __launch_bounds__(256) void k_compact_rows(const uint8_t *x, int64_t rows, int len, int b, int bipolar,
                                                      uint32_t *out, int row_dwords)
{
    constexpr int IN_DW = C == 1 ? 8 : 4;           // input dwords per thread
    constexpr int OUT_DW = IN_DW * C / 8;           // output dwords per thread: 1, 1, 2, 4
    const uint32_t vmask4 = ((1u << b) - 1u) * 0x01010101u;
    const int q = blockIdx.x * 256 + threadIdx.x;   // this thread's group of IN_DW*4 values in the row
    const int i0 = q * IN_DW * 4;
    if (i0 >= len) return;
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) {
        const uint8_t *row = x + r * len;
        uint32_t in[IN_DW];
        if (i0 + IN_DW * 4 <= len) {
#pragma unroll
            for (int v = 0; v < IN_DW / 4; ++v) {
                const u32x4_dw4 t = *reinterpret_cast<const u32x4_dw4 *>(row + i0 + 16 * v);
                in[4 * v] = t.x, in[4 * v + 1] = t.y, in[4 * v + 2] = t.z, in[4 * v + 3] = t.w;
            }
        } else {
#pragma unroll
            for (int d = 0; d < IN_DW; ++d) {
                uint32_t w = 0;
                for (int t = 0; t < 4; ++t)
                    if (i0 + 4 * d + t < len) w |= (uint32_t)row[i0 + 4 * d + t] << (8 * t);
                in[d] = w;
            }
        }
        uint32_t o[OUT_DW];
#pragma unroll
        for (int k = 0; k < OUT_DW; ++k) {
            uint32_t word = 0;
#pragma unroll
            for (int d = 0; d < IN_DW / OUT_DW; ++d)
                word |= gather_bytes<C>(in[k * (IN_DW / OUT_DW) + d], vmask4, bipolar) << (4 * C * d);
            o[k] = word;
        }
        uint32_t *dst = out + r * (int64_t)row_dwords + (int64_t)q * OUT_DW;
        const int left = row_dwords - q * OUT_DW;   // dwords of the row from here on (>= 1)
        if (OUT_DW == 4 && left >= 4) {
            *reinterpret_cast<u32x4_dw4 *>(dst) = u32x4_dw4{o[0], o[1], o[2], o[3]};
        } else if (OUT_DW == 2 && left >= 2) {
            *reinterpret_cast<u32x2_dw4 *>(dst) = u32x2_dw4{o[0], o[1]};
        } else {
#pragma unroll
            for (int k = 0; k < OUT_DW; ++k)
                if (k < left) dst[k] = o[k];
        }
    }
}

// ReLU + requantise (+ 2x2 max-pool).  grid.y walks the output rows (image, channel, row), a
// thread makes one output dword (bit-dense) or four output bytes (one value per byte); one
// 32-bit division per thread finds the row's plane.
template <bool POOL, bool BITDENSE>
__global__ __launch_bounds__(256) void k_epilogue(EpilogueArgs p)
{
    const int per = BITDENSE ? 32 / p.c : 4;         // values per thread
    const int j = blockIdx.x * 256 + threadIdx.x;    // this thread's unit in the row
    const int w0 = j * per;
    if (w0 >= p.Wo) return;
    const uint32_t total_rows = (uint32_t)p.Nimg * p.C * p.Ho;
    for (uint32_t row = blockIdx.y; row < total_rows; row += gridDim.y) {
        const uint32_t nc = row / (uint32_t)p.Ho;
        const int h = (int)(row - nc * (uint32_t)p.Ho);
        const int32_t *src = p.acc + (int64_t)nc * p.H * p.W + (POOL ? (int64_t)(2 * h) * p.W : (int64_t)h * p.W);
        uint32_t word = 0;
        for (int t = 0; t < per; ++t) {
            const int w = w0 + t;
            if (w >= p.Wo) break;
            int32_t v;
            if (POOL) {
                const int32_t *s0 = src + 2 * w;
                v = max(max(s0[0], s0[1]), max(s0[p.W], s0[p.W + 1]));
            } else {
                v = src[w];
            }
            v = min(max(v, 0) >> p.shift, p.qmax);
            word |= (uint32_t)v << (t * (BITDENSE ? p.c : 8));
        }
        if (BITDENSE) {
            reinterpret_cast<uint32_t *>(p.out + (int64_t)row * p.out_row_bytes)[j] = word;
        } else {
            uint8_t *dst = p.out + (int64_t)row * p.Wo + w0;
            for (int t = 0; t < 4 && w0 + t < p.Wo; ++t) dst[t] = (uint8_t)(word >> (8 * t));
        }
    }
}

// ---- micro-benchmarks --------------------------------------------------------------
template <int KIND>
__global__ __launch_bounds__(256) void k_ubench_valu(int iters, uint32_t *buf, uint32_t s1, uint32_t s2)
{
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;
    uint32_t a[8];
    uint64_t w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = t * 2654435761u + i * 40503u + s1;
        w[i] = ((uint64_t)a[i] << 32) | (a[i] ^ 0x9e3779b9u);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                // One named instruction per slot, written as the instruction itself so that the rate
                // printed next to a mnemonic is that instruction's; every chain feeds on its neighbour.
                const int nb = (i + 1) & 7;
                if (KIND == HIKONV_UB_MAD_U32_U24)
                    asm volatile("v_mad_u32_u24 %0, %0, %1, %2" : "+v"(a[i]) : "v"(a[nb]), "v"(s2));
                if (KIND == HIKONV_UB_MAD_I32_I24)
                    asm volatile("v_mad_i32_i24 %0, %0, %1, %2" : "+v"(a[i]) : "v"(a[nb]), "v"(s2));
                if (KIND == HIKONV_UB_MAD_U64_U32) {
                    uint64_t carry;
                    asm volatile("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(w[i]), "=s"(carry) : "v"((uint32_t)w[nb]), "v"(s1));
                }
                if (KIND == HIKONV_UB_MAD_I64_I32) {
                    uint64_t carry;
                    asm volatile("v_mad_i64_i32 %0, %1, %2, %3, %0" : "+v"(w[i]), "=s"(carry) : "v"((uint32_t)w[nb]), "v"(s1));
                }
                if (KIND == HIKONV_UB_MUL_LO_U32) asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(a[i]) : "v"(a[nb]));
                if (KIND == HIKONV_UB_BFE_U32) asm volatile("v_bfe_u32 %0, %1, %2, %3" : "=v"(a[i]) : "v"(a[nb]), "v"(s2), "v"(s1 + 20u));
                if (KIND == HIKONV_UB_LSHR_B64) asm volatile("v_lshrrev_b64 %0, %1, %2" : "=v"(w[i]) : "v"(s2), "v"(w[nb]));
                if (KIND == HIKONV_UB_DPP_MOV)
                    asm volatile("v_mov_b32_dpp %0, %1 wave_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(a[i]) : "v"(a[nb]));
                if (KIND == HIKONV_UB_ADD_U32) asm volatile("v_add_u32 %0, %0, %1" : "+v"(a[i]) : "v"(a[nb]));
                if (KIND == HIKONV_UB_ADD_U64) asm volatile("v_lshl_add_u64 %0, %0, 0, %1" : "+v"(w[i]) : "v"(w[nb]));
                if (KIND == HIKONV_UB_ALIGNBIT) asm volatile("v_alignbit_b32 %0, %0, %1, %2" : "+v"(a[i]) : "v"(a[nb]), "v"(s2));
                if (KIND == HIKONV_UB_AND_B32) asm volatile("v_and_b32 %0, %0, %1" : "+v"(a[i]) : "v"(a[nb]));
                if (KIND == HIKONV_UB_ASHR_I64) asm volatile("v_ashrrev_i64 %0, %1, %2" : "=v"(w[i]) : "v"(s2), "v"(w[nb]));
                if (KIND == HIKONV_UB_BFE_I32) asm volatile("v_bfe_i32 %0, %1, %2, %3" : "=v"(a[i]) : "v"(a[nb]), "v"(s2), "v"(s1 + 20u));
                // dependent chains: every slot works on the same accumulator (run with one wave per SIMD,
                // the time per slot is the instruction's dependent-issue latency)
                if (KIND == HIKONV_UB_CHAIN_MAD_I64_I32) {
                    uint64_t carry;
                    asm volatile("v_mad_i64_i32 %0, %1, %2, %3, %0" : "+v"(w[0]), "=s"(carry) : "v"(a[1]), "v"(s1));
                }
                if (KIND == HIKONV_UB_CHAIN_MAD_I32_I24) asm volatile("v_mad_i32_i24 %0, %0, %1, %2" : "+v"(a[0]) : "v"(a[1]), "v"(s2));
            }
        }
    }
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += a[i] + (uint32_t)w[i] + (uint32_t)(w[i] >> 32);
    buf[t] = sum;
}

__global__ __launch_bounds__(256) void k_ubench_write(int4 *dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int4 v = make_int4(threadIdx.x, blockIdx.x, 3, 4);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = v;
}

__global__ __launch_bounds__(256) void k_ubench_write_nt(int4 *dst, int64_t n16)
{
    typedef int32_t v4i __attribute__((ext_vector_type(4)));
    const int64_t stride = (int64_t)gridDim.x * 256;
    const v4i v = {(int)threadIdx.x, (int)blockIdx.x, 3, 4};
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(v, reinterpret_cast<v4i *>(dst) + i);
}

// Plain writes of values that differ from store to store: every int32 is a hash of its position,
// cut to `value_bits` low bits (the time to write a buffer depends on what is written: int32
// words that are mostly zero bits, such as the outputs of a 1-bit convolution, move slower than
// varied ones).
__global__ __launch_bounds__(256) void k_ubench_write_varied(int4 *dst, int64_t n16, int value_bits)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    const uint32_t mask = value_bits >= 32 ? 0xffffffffu : (1u << value_bits) - 1u;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        const uint32_t h = (uint32_t)i * 2654435761u;
        dst[i] = make_int4((int)(h & mask), (int)((h >> 7 ^ h * 3u) & mask), (int)((h >> 13 ^ h * 5u) & mask),
                           (int)((h >> 19 ^ h * 7u) & mask));
    }
}

// The store pattern of the streaming 1-D kernel without its arithmetic: every wave owns one
// contiguous run of 47 lines of 128 bytes and writes it with six line-aligned 1 KB stores.
__global__ __launch_bounds__(256) void k_ubench_write_runs(int4 *dst, int64_t n16)
{
    typedef int32_t v4i __attribute__((ext_vector_type(4)));
    constexpr int kRunQuads = 47 * 8;
    const int lane = threadIdx.x & 63;
    const int64_t run = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const v4i v = {(int)threadIdx.x, (int)blockIdx.x, 3, 4};
    for (int64_t r = run; r * kRunQuads < n16; r += (int64_t)gridDim.x * 4) {
        const int64_t q0 = r * kRunQuads;
        for (int q = lane; q < kRunQuads && q0 + q < n16; q += 64)
            __builtin_nontemporal_store(v, reinterpret_cast<v4i *>(dst) + q0 + q);
    }
}

__global__ __launch_bounds__(256) void k_ubench_copy(const int4 *src, int4 *dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void k_ubench_read(const int4 *src, int64_t n16, int *sink)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    int acc = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        int4 v = src[i];
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x7fffffff) sink[0] = acc; // practically never: keeps the loads alive
}

// Counts the bytes of a one-value-per-byte buffer that lie outside the declared value range:
// [lo, hi] as signed bytes, or, for {-1,+1} data, anything but -1 and +1.  One atomic per wave.
__global__ void __launch_bounds__(256) k_check_range(const uint8_t *x, int64_t count, int lo, int hi, int is_signed,
                                                      int bipolar, uint32_t *violations)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    uint32_t bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
        const int v = is_signed ? (int)(int8_t)x[i] : (int)x[i];
        bad += bipolar ? (v != 1 && v != -1) : (v < lo || v > hi);
    }
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_down(bad, off, 64);
    if ((threadIdx.x & 63) == 0 && bad) atomicAdd(violations, bad);
}

__global__ void k_selftest_lane_shift(int32_t *out)
{
    out[threadIdx.x] = (int32_t)lane_shr1((uint32_t)(threadIdx.x + 100));
}

} // namespace

hipError_t launch_compact(const uint8_t *x, int64_t rows, int64_t len, int bits, int bipolar, uint32_t *out,
                          int64_t row_dwords, hipStream_t stream)
{
    const int64_t total = rows * row_dwords;
    if (total <= 0) return hipSuccess;
    const int c = container_bits(bits);
    // streaming form: every row starts on a dword boundary and positions inside a row fit 32 bits
    if ((reinterpret_cast<uintptr_t>(x) & 3) == 0 && (len & 3) == 0 && len < (1LL << 30)) {
        const int per_thread = c == 1 ? 32 : 16;
        dim3 g((unsigned)ceil_div(len, (int64_t)256 * per_thread), (unsigned)(rows < 65535 ? rows : 65535));
        switch (c) {
        case 1: hipLaunchKernelGGL(k_compact_rows<1>, g, dim3(256), 0, stream, x, rows, (int)len, bits, bipolar, out, (int)row_dwords); break;
        case 2: hipLaunchKernelGGL(k_compact_rows<2>, g, dim3(256), 0, stream, x, rows, (int)len, bits, bipolar, out, (int)row_dwords); break;
        case 4: hipLaunchKernelGGL(k_compact_rows<4>, g, dim3(256), 0, stream, x, rows, (int)len, bits, bipolar, out, (int)row_dwords); break;
        default: hipLaunchKernelGGL(k_compact_rows<8>, g, dim3(256), 0, stream, x, rows, (int)len, bits, bipolar, out, (int)row_dwords); break;
        }
        return hipGetLastError();
    }
    const int64_t grid = ceil_div(total, 256);
    if (grid > 0x7fffffffLL) return hipErrorNotSupported;
    hipLaunchKernelGGL(k_compact, dim3((unsigned)grid), dim3(256), 0, stream, x, rows, len, bits, c, bipolar, out,
                       row_dwords);
    return hipGetLastError();
}

hipError_t launch_check_range(const uint8_t *x, int64_t count, int lo, int hi, int is_signed, int bipolar,
                              uint32_t *violations, hipStream_t stream)
{
    if (count <= 0) return hipSuccess;
    const int64_t want = ceil_div(count, 256 * 16);
    const unsigned grid = (unsigned)(want < 1 ? 1 : want > 8192 ? 8192 : want);
    hipLaunchKernelGGL(k_check_range, dim3(grid), dim3(256), 0, stream, x, count, lo, hi, is_signed, bipolar, violations);
    return hipGetLastError();
}

hipError_t launch_epilogue(const EpilogueArgs &a, hipStream_t stream)
{
    const bool bitdense = a.out_format == HIKONV_FMT_BITDENSE;
    const int64_t units = bitdense ? a.out_row_bytes / 4 : ceil_div(a.Wo, 4);
    const int64_t rows = (int64_t)a.Nimg * a.C * a.Ho;
    if (rows <= 0 || units <= 0) return hipSuccess;
    if (rows >= (1LL << 31) || a.Wo >= (1 << 30)) return hipErrorNotSupported;
    dim3 g((unsigned)ceil_div(units, 256), (unsigned)(rows < 65535 ? rows : 65535));
    if (a.pool && bitdense)
        hipLaunchKernelGGL((k_epilogue<true, true>), g, dim3(256), 0, stream, a);
    else if (a.pool)
        hipLaunchKernelGGL((k_epilogue<true, false>), g, dim3(256), 0, stream, a);
    else if (bitdense)
        hipLaunchKernelGGL((k_epilogue<false, true>), g, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((k_epilogue<false, false>), g, dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_ubench(int kind, int iters, int blocks, void *buf, size_t bytes, hipStream_t stream)
{
    dim3 g((unsigned)blocks), b(256);
    uint32_t *u = static_cast<uint32_t *>(buf);
    switch (kind) {
#define HIKONV_UB_CASE(K)                                                                      \
    case K:                                                                                    \
        if (bytes < (size_t)blocks * 256 * 4) return hipErrorNotSupported;                     \
        hipLaunchKernelGGL((k_ubench_valu<K>), g, b, 0, stream, iters, u, 3u, 1u);             \
        break;
        HIKONV_UB_CASE(HIKONV_UB_MAD_U32_U24)
        HIKONV_UB_CASE(HIKONV_UB_MAD_U64_U32)
        HIKONV_UB_CASE(HIKONV_UB_MUL_LO_U32)
        HIKONV_UB_CASE(HIKONV_UB_BFE_U32)
        HIKONV_UB_CASE(HIKONV_UB_LSHR_B64)
        HIKONV_UB_CASE(HIKONV_UB_DPP_MOV)
        HIKONV_UB_CASE(HIKONV_UB_ADD_U32)
        HIKONV_UB_CASE(HIKONV_UB_MAD_I32_I24)
        HIKONV_UB_CASE(HIKONV_UB_MAD_I64_I32)
        HIKONV_UB_CASE(HIKONV_UB_ADD_U64)
        HIKONV_UB_CASE(HIKONV_UB_ALIGNBIT)
        HIKONV_UB_CASE(HIKONV_UB_AND_B32)
        HIKONV_UB_CASE(HIKONV_UB_ASHR_I64)
        HIKONV_UB_CASE(HIKONV_UB_BFE_I32)
        HIKONV_UB_CASE(HIKONV_UB_CHAIN_MAD_I64_I32)
        HIKONV_UB_CASE(HIKONV_UB_CHAIN_MAD_I32_I24)
#undef HIKONV_UB_CASE
    case HIKONV_UB_HBM_WRITE:
        hipLaunchKernelGGL(k_ubench_write, g, b, 0, stream, static_cast<int4 *>(buf), (int64_t)(bytes / 16));
        break;
    case HIKONV_UB_HBM_WRITE_NT:
        hipLaunchKernelGGL(k_ubench_write_nt, g, b, 0, stream, static_cast<int4 *>(buf), (int64_t)(bytes / 16));
        break;
    case HIKONV_UB_HBM_WRITE_VARIED:
        if (iters < 1 || iters > 32) return hipErrorInvalidValue;
        hipLaunchKernelGGL(k_ubench_write_varied, g, b, 0, stream, static_cast<int4 *>(buf), (int64_t)(bytes / 16), iters);
        break;
    case HIKONV_UB_HBM_WRITE_RUNS:
        hipLaunchKernelGGL(k_ubench_write_runs, g, b, 0, stream, static_cast<int4 *>(buf), (int64_t)(bytes / 16));
        break;
    case HIKONV_UB_HBM_COPY: {
        const int64_t half16 = (int64_t)(bytes / 32);
        hipLaunchKernelGGL(k_ubench_copy, g, b, 0, stream, static_cast<const int4 *>(buf),
                           static_cast<int4 *>(buf) + half16, half16);
        break;
    }
    case HIKONV_UB_HBM_READ:
        if (bytes < 32) return hipErrorNotSupported;
        hipLaunchKernelGGL(k_ubench_read, g, b, 0, stream, static_cast<const int4 *>(buf) + 1,
                           (int64_t)(bytes / 16) - 1, static_cast<int *>(buf));
        break;
    default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

hipError_t launch_selftest_lane_shift(int32_t *out, hipStream_t stream)
{
    hipLaunchKernelGGL(k_selftest_lane_shift, dim3(1), dim3(64), 0, stream, out);
    return hipGetLastError();
}

} // namespace hikonv

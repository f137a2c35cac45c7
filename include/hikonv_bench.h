/*
 * hikonv_bench.h -- measurement and self-check entry points of libhikonv.so that are not
 * part of the convolution interface: roofline micro-benchmarks (integer VALU issue rate,
 * HBM bandwidth) and a lane-exchange layout check.  Used by bench.py and the tests.
 * Conventions as in hikonv.h.
 */
#ifndef HIKONV_BENCH_H
#define HIKONV_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Roofline micro-benchmarks.  kind: HIKONV_UB_*.  Launches one kernel on
 * `stream`; the caller times it.  For VALU kinds every lane of `blocks` x 256
 * threads issues iters x 64 dependent-chain-free instructions of the kind;
 * buf_dev (>= 4*blocks*256 bytes) receives a checksum so nothing is optimised
 * away.  For HBM kinds buf_dev holds `bytes` bytes (copy: first half -> second).
 */
#define HIKONV_UB_MAD_U32_U24 0
#define HIKONV_UB_MAD_U64_U32 1
#define HIKONV_UB_MUL_LO_U32 2
#define HIKONV_UB_BFE_U32 3
#define HIKONV_UB_LSHR_B64 4
#define HIKONV_UB_DPP_MOV 5
#define HIKONV_UB_ADD_U32 6
#define HIKONV_UB_MAD_I32_I24 7
#define HIKONV_UB_MAD_I64_I32 8
#define HIKONV_UB_ADD_U64 9
#define HIKONV_UB_ALIGNBIT 10
#define HIKONV_UB_AND_B32 11
#define HIKONV_UB_ASHR_I64 12
#define HIKONV_UB_BFE_I32 13
#define HIKONV_UB_CHAIN_MAD_I64_I32 14 /* one dependent chain per lane: with one wave per SIMD the time per slot is the latency */
#define HIKONV_UB_CHAIN_MAD_I32_I24 15
#define HIKONV_UB_HBM_WRITE 16
#define HIKONV_UB_HBM_COPY 17
#define HIKONV_UB_HBM_READ 18
#define HIKONV_UB_HBM_WRITE_NT 19 /* write with the non-temporal hint */
#define HIKONV_UB_HBM_WRITE_RUNS 20 /* non-temporal, one contiguous 6016-byte run per wave (the 1-D kernel's store pattern) */
#define HIKONV_UB_HBM_WRITE_VARIED 21 /* plain writes of int32 values that vary from word to word, `iters` (1..32) low bits of a hash of the position */
int hikonv_ubench(int kind, int iters, int blocks, void *buf_dev, size_t bytes, void *stream);

/* Lane-exchange self check: out_dev[i] (64 ints) = value lane i receives from lane i-1 (lane 0: 0). */
int hikonv_selftest_lane_shift(int32_t *out_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HIKONV_BENCH_H */

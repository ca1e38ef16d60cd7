/*
 * sqp_test_hooks.h -- test and benchmark hooks of libsqp.so.  NOT part of the product ABI
 * (that is sqp.h): process-wide switches that override the launch plan the library would
 * pick, plan queries that need no GPU, and two calibration kernels for the benchmark.  None
 * is thread-safe; a test sets a switch, makes its calls and resets it (0 / -1 = automatic).
 */
#ifndef SQP_TEST_HOOKS_H
#define SQP_TEST_HOOKS_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif
#pragma GCC visibility push(default) /* the library is built with hidden visibility: these are its exports */

/* Weight-streaming path (M <= 64 rows) of sqp_w4a16_gemm. */
void sqp_debug_set_decode_max_m(int m);            /* rows up to which that path is used (default 64) */
void sqp_debug_set_decode_split(int split);        /* force the number of K parts; 0 = automatic */
void sqp_debug_set_decode_plan(int nw, int split); /* force strips per workgroup and K parts; (0, 0) = automatic */
void sqp_debug_set_decode_kw(int kw);              /* 1 = never two waves per strip; 0 = automatic */
void sqp_debug_set_decode_kp(int kp);              /* two chunks per iteration (twice the waves): 0 = automatic, 1 = never, 2 = wherever built */
void sqp_debug_set_decode_slice(int mode);         /* column-slice kernel (M <= 16, groups of 128): 0 = automatic, -1 = never,
                                                      1 = always with 32-column slices, 2 = always with 64-column slices */
/* Which kernel a call would take: -1 = the strip kernel below, 0 / 1 = the column-slice kernel
 * with 32- / 64-column slices.  Host arithmetic only. */
int sqp_debug_decode_slice_choice(int M, int N, int K, int group);
/* The plan the heuristic picks for a shape: strips per workgroup, K parts, k-steps per chunk
 * (0 = the generic one-thread-per-element kernel).  Host arithmetic only. */
void sqp_debug_decode_plan(int M, int N, int K, int group, int *nw, int *split, int *kspg);

/* Tiled matrix-core path (M > 64). */
void sqp_debug_set_prefill_tiles(int mode);        /* 0 = automatic, 1 = full tiles only, 2 = half-width tiles only */
void sqp_debug_set_prefill_shape(int shape);       /* 0 = automatic, 1 = 128 x 512 full tiles, 2 = 256 x 256 */
void sqp_debug_set_prefill_ksplit(int k);          /* -1 = automatic, 0 or 1 = never, k >= 2 = k parts */
/* The tile plan for a shape on a chip of `cus` compute units: full tiles of the first launch,
 * half-width tiles of the second, K parts.  Host arithmetic only. */
void sqp_debug_prefill_plan(int M, int N, int K, int cus, long *full, long *half, int *ksplit);

/* Calibration kernels for the benchmark: a plain device copy of `bytes` (a multiple of 16)
 * whose traffic is known, and a loop of nothing but independent 32x32x16 fp16 matrix
 * instructions (data: 64 KiB of fp16 on the device, out: blocks * 256 floats; flops of the
 * launch = blocks * 4 * iters * 16 * 32768). */
int sqp_debug_plain_copy(const void *src, void *dst, size_t bytes, void *stream);
/* A plain streaming read of `bytes` (a multiple of 16; whole passes of 8 x blocks x 256 x 16 bytes
 * are read, the rest is skipped) by `blocks` workgroups of 256 threads, with (nt != 0) or without
 * the non-temporal hint; sink: 4 bytes.  The rate depends on the grid: three workgroups per
 * compute unit (768) read faster than thousands. */
int sqp_debug_read_probe(const void *src, size_t bytes, int nt, int blocks, void *sink, void *stream);
int sqp_debug_mfma_ceiling(const void *data, float *out, int blocks, int iters, void *stream);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif /* SQP_TEST_HOOKS_H */

/*
 * sqp.h -- C ABI of the SmoothQuant+ W4A16 linear-layer library for AMD MI355X (gfx950).
 *
 * The operations are those of arXiv 2312.03788: per-channel smoothing (Eq. 5, Eq. 6),
 * group-wise asymmetric 4-bit weight quantisation (Eq. 1, Sec 2.2) and the quantised
 * linear layer Y = X * W_hat with FP16 input/output and INT4 weights (Eq. 3, Fig. 7).
 *
 * Conventions for every entry point
 *   - Orientation follows Eq. 2: X is [M x K] (tokens x input channels), W is [K x N]
 *     (input channels x output channels), Y is [M x N]; all row-major, last index
 *     contiguous.
 *   - Every pointer is a DEVICE pointer owned by the caller and must be 16-byte aligned
 *     (the fp64 outputs of the loss calls: 8-byte).  fp16 data is IEEE binary16.  The
 *     library allocates no device memory, frees none, and keeps no caller memory except
 *     the workspace pointer handed to sqp_set_workspace.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     only enqueued; no call synchronises the device or allocates, so every call may be
 *     recorded into a HIP graph.
 *   - Return value: SQP_OK (0), or a negative error code, in which case nothing was
 *     enqueued.  sqp_status_string() names a code.
 *   - Shape rules: M, N, K > 0; N % 8 == 0; K % 8 == 0; group % 8 == 0, group >= 8,
 *     K % group == 0; every tensor has fewer than 2^31 elements.
 *
 * Storage format of a quantised weight (what sqp_quantize_pack writes and
 * sqp_dequantize / sqp_w4a16_gemm read):
 *   packed[K/8][N]      uint32; word (j, n) holds the 4-bit codes of input channels
 *                       k = 8j .. 8j+7 of output column n, the code of k = 8j+i in bits
 *                       [4i+3 : 4i] (lowest nibble = lowest k).
 *   scales[K/group][N]  fp16 step size Delta of group t = k / group, column n.
 *   zeros [K/group][N]  uint8 zero point Z in [0, 15] of the same group.
 */
#ifndef SQP_H
#define SQP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#pragma GCC visibility push(default) /* the library is built with hidden visibility: these are its exports */

#define SQP_OK 0
#define SQP_ERR_NULL (-1)    /* a required pointer is NULL */
#define SQP_ERR_SHAPE (-2)   /* a shape rule above is violated */
#define SQP_ERR_ALIGN (-3)   /* a pointer is not 16-byte aligned */
#define SQP_ERR_ARG (-4)     /* alpha outside [0, 1] or not finite */
#define SQP_ERR_LAUNCH (-5)  /* the HIP runtime reported an error at launch */
#define SQP_ERR_WORKSPACE (-6) /* the workspace is too small for the launch plan of this shape */

const char *sqp_status_string(int status);

/* Smoothing factor of Eq. 6:  s[j] = max_t|x_cal[t][j]|^alpha / max_n|w[j][n]|^(1-alpha),
 * j = input channel.  Both maxima are floored at 1e-5 (Eq. 6 is 0 or infinite on a dead
 * channel); the quotient is evaluated in fp64 and rounded once to fp32.
 *   x_cal [T][K] fp16  calibration activations (Sec 2.2: per-channel maxima over the
 *                      calibration tokens)
 *   w     [K][N] fp16  the unsmoothed weight
 *   s     [K]    fp32  out; also used as scratch while the call runs
 * alpha in [0, 1]. */
int sqp_smooth_scales(int T, int K, int N, float alpha, const void *x_cal, const void *w,
                      float *s, void *stream);

/* Activation side of Eq. 5:  x_out[m][j] = fp16(x[m][j] / s[j]), fp32 divide, one rounding.
 * x, x_out [M][K] fp16 (may alias), s [K] fp32. */
int sqp_smooth_apply_x(int M, int K, const void *x, const float *s, void *x_out, void *stream);

/* Weight side of Eq. 5:  w_out[j][n] = fp16(s[j] * w[j][n]), fp32 multiply, one rounding.
 * w, w_out [K][N] fp16 (may alias), s [K] fp32. */
int sqp_smooth_apply_w(int K, int N, const void *w, const float *s, void *w_out, void *stream);

/* The merged gate/up projection of a LlamaMLP block with its activation fused (Fig. 5: the
 * block whose smoothing factors are folded into the preceding layers).  packed/scales/zeros
 * hold the quantised merged weight [K][N] whose columns alternate (gate j, up j)
 * (sqp_interleave_gate_up); the result is
 *   y[m][j] = fp16( SiLU(g) * u ),  g, u = the fp32 sums of Eq. 3 for columns 2j and 2j+1,
 * y [M][N/2] fp16.  N % 16 == 0; group 32, 64 or a multiple of 128.  Otherwise as sqp_w4a16_gemm. */
int sqp_w4a16_gemm_silu_mul(int M, int N, int K, int group, const void *x, const uint32_t *packed,
                            const void *scales, const uint8_t *zeros, void *y, void *stream);

/* LlamaRMSNorm: y[m][j] = fp16( x[m][j] / sqrt(mean_j x[m][j]^2 + eps) * gamma[j] ), fp32
 * arithmetic.  gamma [H] fp16 may already contain the division by the smoothing factor of the
 * layers it feeds (Sec 2.2: fused into post_attention_layernorm; fold it with
 * sqp_smooth_apply_x on the 1 x H weight).  x, y [M][H] fp16, H % 8 == 0, 0 <= eps < 1. */
int sqp_rmsnorm(int M, int H, const void *x, const void *gamma, float eps, void *y, void *stream);

/* w_out[k][n] = fp16(w[k][n] / s[n]): divides the OUTPUT columns of a layer by the smoothing
 * factor of the layer it feeds (Sec 2.2: down_proj's factor fused into up_proj's weights).
 * w, w_out [K][N] fp16 (may alias), s [N] fp32, N % 8 == 0. */
int sqp_scale_columns(int K, int N, const void *w, const float *s, void *w_out, void *stream);

/* w_out [K][2I] with column 2j = w_gate[.][j] and column 2j+1 = w_up[.][j] (exact copies), the
 * merged layout sqp_w4a16_gemm_silu_mul expects.  w_gate, w_up [K][I] fp16, I % 8 == 0. */
int sqp_interleave_gate_up(int K, int I, const void *w_gate, const void *w_up, void *w_out, void *stream);

/* Orientation helper: w_nk [N][K] fp16 (one row per output feature, as checkpoints store a
 * linear layer) -> w_kn [K][N] fp16, the orientation of Eq. 2 (X W with W of shape Ci x Co) that
 * every other entry point takes.  Exact copy of the values; the buffers must not overlap. */
int sqp_transpose_nk(int N, int K, const void *w_nk, void *w_kn, void *stream);

/* Group-wise asymmetric 4-bit quantisation of Eq. 1 along K (Sec 2.2) and packing.
 * For each column n and group t (rows t*group .. (t+1)*group-1):
 *   lo = min(min w, 0), hi = max(max w, 0)           (range widened to contain 0)
 *   Delta = fp16((hi - lo) / 15), replaced by 2^-24 if that is zero
 *   Z = clamp(round(-lo / Delta), 0, 15)
 *   code = clamp(round(w / Delta) + Z, 0, 15)        round = half-to-even, fp32 divide
 * w [K][N] fp16 (already smoothed); packed/scales/zeros as described above (out). */
int sqp_quantize_pack(int N, int K, int group, const void *w, uint32_t *packed, void *scales,
                      uint8_t *zeros, void *stream);

/* Second line of Eq. 1:  w_hat[k][n] = fp16((code - Z) * Delta).  w_hat [K][N] fp16 out. */
int sqp_dequantize(int N, int K, int group, const uint32_t *packed, const void *scales,
                   const uint8_t *zeros, void *w_hat, void *stream);

/* The quantised linear layer of Eq. 3 (Fig. 7: FP16 in, INT4 weights, FP16 out):
 *   y[m][n] = fp16( sum_k x[m][k] * (code[k][n] - Z[k/group][n]) * Delta[k/group][n] )
 * with fp32 accumulation and one rounding to fp16 at the end.  The result is
 * run-to-run deterministic.  x [M][K] fp16, y [M][N] fp16 out (must not alias x).
 * Rows M <= 64 take the weight-streaming (memory-bound) path, larger M the tiled
 * matrix-core path.  When the output has too few tiles to occupy the chip, the launch plan
 * splits the inner dimension across workgroups and passes fp32 partial sums through the
 * workspace set with sqp_set_workspace (with few rows, or few rows and a short K, groups of 128
 * run a kernel that splits K inside each workgroup instead and uses no workspace:
 * sqp_w4a16_gemm_workspace_bytes() is 0 for those shapes):
 *   - no workspace set: the plan without a split runs (same result within the tolerance of
 *     Eq. 3's fp32 accumulation, slower on narrow layers);
 *   - workspace smaller than sqp_w4a16_gemm_workspace_bytes() of the shape:
 *     SQP_ERR_WORKSPACE, nothing enqueued.
 * Calls that use the workspace must not overlap on the device (order them on one stream, or
 * with events): they share its tickets and partial sums. */
int sqp_w4a16_gemm(int M, int N, int K, int group, const void *x, const uint32_t *packed,
                   const void *scales, const uint8_t *zeros, void *y, void *stream);

/* Bytes of workspace the launch plan of sqp_w4a16_gemm / sqp_w4a16_gemm_silu_mul uses for
 * this shape on the current device: 0 if the plan does not split the inner dimension,
 * otherwise 512 KB of tickets plus the fp32 partial sums.  Host arithmetic only. */
size_t sqp_w4a16_gemm_workspace_bytes(int M, int N, int K, int group);

/* Hands the library a caller-owned device buffer for the partial sums of Eq. 3's split
 * launches on the CURRENT device (process-wide, one per device; the library keeps only the
 * pointer).  The call enqueues one kernel on `stream` that zeroes the ticket area (the first
 * 512 KB); GEMM calls must be ordered after it.  Every split launch leaves the tickets zero
 * again, so the buffer is set once; after an aborted launch set it again.  The caller keeps
 * the buffer alive until it sets another one or none: (NULL, 0) removes it.
 * Errors: SQP_ERR_ALIGN; SQP_ERR_WORKSPACE if bytes <= 512 KB.  Not to be called while
 * another thread is inside a GEMM call. */
int sqp_set_workspace(void *dev_ptr, size_t bytes, void *stream);

/* Quantisation loss of one layer, Eq. 4:  *loss = || x w - x_hat w_hat ||_F^2  with
 * w_hat the dequantised weights of (packed, scales, zeros) (Eq. 1) - the quantity the search
 * over the smoothing strength alpha minimises (Sec 2.2, Eq. 6), for one layer.  Both products
 * are accumulated together in fp32 (the difference is formed before any rounding to fp16),
 * the squares are summed in fp64 in a fixed order (run-to-run deterministic).
 *   x     [M][K] fp16  calibration activations        w [K][N] fp16  the unsmoothed weight
 *   x_hat [M][K] fp16  smoothed activations (Eq. 5)   packed/scales/zeros: quantised smoothed weight
 *   scratch  device, at least sqp_quant_loss_scratch_doubles(M, N) doubles, overwritten
 *   loss     device, one double (out)
 * All device pointers (scratch and loss 8-byte aligned); nothing is allocated. */
long sqp_quant_loss_scratch_doubles(int M, int N);
int sqp_quant_loss(int M, int N, int K, int group, const void *x, const void *w, const void *x_hat,
                   const uint32_t *packed, const void *scales, const uint8_t *zeros, double *scratch,
                   double *loss, void *stream);

/* sqp_w4a16_gemm for callers that cannot allocate device memory and own no workspace: code
 * recorded under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, kernels, launch plans and results as sqp_w4a16_gemm with a sufficient
 * workspace set (bit-identical), but the tickets and partial sums of split launches live in a
 * static device array of the library: 512 KB + SQP_STATIC_PARTIAL_BYTES per device, held
 * until the process ends.  The call allocates nothing and ignores sqp_set_workspace.
 *   - A shape whose plan needs more partial sums than SQP_STATIC_PARTIAL_BYTES
 *     (sqp_w4a16_gemm_workspace_bytes(shape) - 512 KB) is refused with SQP_ERR_WORKSPACE,
 *     nothing enqueued.  The library's own plans stay below the limit for every shape.
 *   - The first call on a device looks the array up and enqueues one extra kernel that zeroes
 *     its tickets; make that call outside a graph capture.
 *   - All calls on one device share the array: calls that overlap on the device race (order
 *     them on one stream or with events), as do overlaps with nothing else in this library. */
#define SQP_STATIC_PARTIAL_BYTES ((size_t)48 << 20)
int sqp_w4a16_gemm_static(int M, int N, int K, int group, const void *x, const uint32_t *packed,
                          const void *scales, const uint8_t *zeros, void *y, void *stream);

/* Search of the smoothing strength for one layer (Sec 2.2: alpha is chosen on a grid to
 * minimise the quantisation loss of Eq. 4; the paper's grid is 0, 0.05, ..., 1).  The
 * per-channel maxima of Eq. 6 do not depend on alpha and are computed once; then for each
 * alphas[i], in order:  s = Eq. 6,  x_hat = x_cal / s and w_s = s * w (Eq. 5),  w_s quantised
 * (Eq. 1),  loss[i] = Eq. 4 on the calibration rows.  *best = index of the smallest loss (the
 * lowest index on ties).  Every step is the kernel of the corresponding entry point above, so
 * loss[i] equals what those calls would give, bit for bit.
 *   alphas   HOST array of n_alpha values in [0, 1], 1 <= n_alpha <= 4096
 *   x_cal [T][K] fp16, w [K][N] fp16                                    (in)
 *   amax [2K] fp32, s [K] fp32, x_hat [T][K] fp16, w_s [K][N] fp16, packed / scales / zeros of
 *   the layer's shape, scratch (sqp_quant_loss_scratch_doubles(T, N) doubles): device work
 *   buffers, overwritten; on return they hold the last alpha's values
 *   loss [n_alpha] fp64 device (out), best: one int, device (out)
 * Nothing is allocated and nothing synchronises; errors as for the single calls. */
int sqp_alpha_search(int T, int N, int K, int group, int n_alpha, const float *alphas, const void *x_cal,
                     const void *w, float *amax, float *s, void *x_hat, void *w_s, uint32_t *packed,
                     void *scales, uint8_t *zeros, double *scratch, double *loss, int *best, void *stream);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif /* SQP_H */

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
 *   - Every pointer is a DEVICE pointer owned by the caller and must be 16-byte aligned.
 *     fp16 data is IEEE binary16.  The library never frees or keeps caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     only enqueued; no call synchronises the device.
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

#define SQP_OK 0
#define SQP_ERR_NULL (-1)    /* a required pointer is NULL */
#define SQP_ERR_SHAPE (-2)   /* a shape rule above is violated */
#define SQP_ERR_ALIGN (-3)   /* a pointer is not 16-byte aligned */
#define SQP_ERR_ARG (-4)     /* alpha outside [0, 1] or not finite */
#define SQP_ERR_LAUNCH (-5)  /* the HIP runtime reported an error at launch */
#define SQP_ERR_WORKSPACE (-6) /* the library could not obtain its device workspace */

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
 * matrix-core path (with the inner dimension split across workgroups when the output has
 * too few tiles to occupy the chip).  Some shapes use a library-owned device workspace
 * (128 MB of fp32 partial sums per device) that is allocated on first use (so the first
 * such call may allocate; concurrent calls on different streams that both need it are
 * serialised by the caller). */
int sqp_w4a16_gemm(int M, int N, int K, int group, const void *x, const uint32_t *packed,
                   const void *scales, const uint8_t *zeros, void *y, void *stream);

/* Quantisation loss of one layer, Eq. 4:  *loss = || x w - x_hat w_hat ||_F^2  with
 * w_hat the dequantised weights of (packed, scales, zeros) (Eq. 1) - the quantity the search
 * over the smoothing strength alpha minimises (Sec 2.2, Eq. 6), for one layer.  Both products
 * are accumulated together in fp32 (the difference is formed before any rounding to fp16),
 * the squares are summed in fp64 in a fixed order (run-to-run deterministic).
 *   x     [M][K] fp16  calibration activations        w [K][N] fp16  the unsmoothed weight
 *   x_hat [M][K] fp16  smoothed activations (Eq. 5)   packed/scales/zeros: quantised smoothed weight
 *   scratch  device, at least sqp_quant_loss_scratch_doubles(M, N) doubles, overwritten
 *   loss     device, one double (out)
 * All device pointers; nothing is allocated. */
long sqp_quant_loss_scratch_doubles(int M, int N);
int sqp_quant_loss(int M, int N, int K, int group, const void *x, const void *w, const void *x_hat,
                   const uint32_t *packed, const void *scales, const uint8_t *zeros, double *scratch,
                   double *loss, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SQP_H */

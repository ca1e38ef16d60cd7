/*
 * sqp_oracle.c -- CPU oracle for the SmoothQuant+ W4A16 linear-layer path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * statement of what the GPU library must compute.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it; the product
 * (the HIP library and its Python binding) never does.  It shares no source,
 * header, table or helper with the GPU path.
 *
 * Every function follows one passage of the paper (arXiv 2312.03788):
 *   Eq. 1   uniform asymmetric 4-bit quantisation (codes, step size, dequant)
 *   Eq. 2/3 the (quantised) linear layer Y = X * W_hat
 *   Eq. 4   quantisation loss
 *   Eq. 5   per-channel smoothing  Y = (X diag(s)^-1)(diag(s) W)
 *   Eq. 6   smoothing factor s_j = max|X_j|^alpha / max|W_j|^(1-alpha)
 *   Sec 2.2 group-wise quantisation, group size 128 (others allowed)
 *   Sec 2.3 / Fig. 7: FP16 in, FP16 out, INT4 weights.
 * Where the paper is silent the reading taken is stated at the function.
 *
 * Orientation follows Eq. 2: X is [T x Ci] (here M x K), W is [Ci x Co]
 * (here K x N, N contiguous).  fp16 values travel as uint16_t bit patterns.
 *
 * Pins (tests marked "not gpu"): exhaustive fp16 conversion against numpy,
 * closed-form groups, pack bijection, Eq. 5 identity in fp64, the alpha = 0
 * and alpha = 1 special cases of Eq. 6, round-to-nearest error bound,
 * brute-force tiny GEMMs against numpy float64.  No function here is
 * "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ fp16 */

/* IEEE binary16 bit pattern -> float, exact. */
float orc_h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu;
    uint32_t m = h & 0x3ffu;
    float v;
    if (e == 0) {
        v = ldexpf((float)m, -24);            /* zero and subnormals */
    } else if (e == 31) {
        uint32_t u = 0x7f800000u | (m << 13); /* inf / nan */
        memcpy(&v, &u, 4);
    } else {
        uint32_t u = ((e + 112u) << 23) | (m << 13);
        memcpy(&v, &u, 4);
    }
    if (sign) v = -v;
    return v;
}

/* float -> IEEE binary16 bit pattern, round-to-nearest-even, subnormals kept. */
uint16_t orc_f2h(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u | ((a >> 13) & 0x3ffu)); /* nan */
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7c00u);                       /* >= 65536 or inf */
    uint32_t e = a >> 23;
    if (e >= 113) {                            /* normal half range (before rounding) */
        uint32_t h = ((e - 112u) << 10) | ((a >> 13) & 0x3ffu);
        uint32_t rem = a & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) h++; /* carry may reach inf: correct */
        return (uint16_t)(sign | h);
    }
    /* result is subnormal (or rounds up to the smallest normal) */
    uint32_t shift = 126u - e;                 /* value / 2^-24 = mant >> shift */
    if (shift > 24) return sign;               /* below 2^-25: zero */
    uint32_t mant = (a & 0x7fffffu) | 0x800000u;
    uint32_t r = mant >> shift;
    uint32_t rem = mant & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (r & 1u))) r++;
    return (uint16_t)(sign | r);
}

void orc_h2f_array(size_t n, const uint16_t *h, float *f)
{
    for (size_t i = 0; i < n; i++) f[i] = orc_h2f(h[i]);
}

void orc_f2h_array(size_t n, const float *f, uint16_t *h)
{
    for (size_t i = 0; i < n; i++) h[i] = orc_f2h(f[i]);
}

/* ------------------------------------------------------------- smoothing */

/* max_t |X[t][j]| for every input channel j (Sec 2.2: per-channel activation
 * maxima over the calibration tokens).  x is [T][K]. */
void orc_absmax_x(int T, int K, const uint16_t *x, float *ax)
{
    for (int j = 0; j < K; j++) ax[j] = 0.0f;
    for (int t = 0; t < T; t++)
        for (int j = 0; j < K; j++) {
            float v = fabsf(orc_h2f(x[(size_t)t * K + j]));
            if (v > ax[j]) ax[j] = v;
        }
}

/* max_n |W[j][n]| for every input channel j: Eq. 6's max|W_j|, taken over all
 * outputs fed by input channel j (Fig. 4: weights are smoothed over the input
 * channel dimension).  w is [K][N]. */
void orc_absmax_w(int K, int N, const uint16_t *w, float *aw)
{
    for (int j = 0; j < K; j++) {
        float m = 0.0f;
        for (int n = 0; n < N; n++) {
            float v = fabsf(orc_h2f(w[(size_t)j * N + n]));
            if (v > m) m = v;
        }
        aw[j] = m;
    }
}

/* Eq. 6.  Reading for a dead channel (a maximum of 0, on which Eq. 6 is 0 or
 * infinite): both maxima are floored at 1e-5 first.  Evaluated in fp64 and
 * rounded once to fp32. */
void orc_smooth_factor(int K, float alpha, const float *ax, const float *aw, float *s)
{
    double a = (double)alpha;
    for (int j = 0; j < K; j++) {
        float fx = ax[j] > 1e-5f ? ax[j] : 1e-5f;
        float fw = aw[j] > 1e-5f ? aw[j] : 1e-5f;
        s[j] = (float)(pow((double)fx, a) / pow((double)fw, 1.0 - a));
    }
}

/* Eq. 6 from the calibration activations and the unsmoothed weight. */
void orc_smooth_scales(int T, int K, int N, float alpha, const uint16_t *xcal,
                       const uint16_t *w, float *s)
{
    float *ax = (float *)malloc(sizeof(float) * (size_t)K);
    float *aw = (float *)malloc(sizeof(float) * (size_t)K);
    orc_absmax_x(T, K, xcal, ax);
    orc_absmax_w(K, N, w, aw);
    orc_smooth_factor(K, alpha, ax, aw, s);
    free(ax);
    free(aw);
}

/* Eq. 5, activation side: X_hat[m][j] = X[m][j] / s[j]; fp32 divide, one
 * rounding to fp16 (the layer's input stays FP16, Fig. 7). */
void orc_smooth_apply_x(int M, int K, const uint16_t *x, const float *s, uint16_t *xo)
{
    for (int m = 0; m < M; m++)
        for (int j = 0; j < K; j++)
            xo[(size_t)m * K + j] = orc_f2h(orc_h2f(x[(size_t)m * K + j]) / s[j]);
}

/* Eq. 5, weight side: W_hat[j][n] = s[j] * W[j][n]; fp32 multiply, one
 * rounding to fp16 (Sec 2.3: the smoothed model is an FP16 model). */
void orc_smooth_apply_w(int K, int N, const uint16_t *w, const float *s, uint16_t *wo)
{
    for (int j = 0; j < K; j++)
        for (int n = 0; n < N; n++)
            wo[(size_t)j * N + n] = orc_f2h(s[j] * orc_h2f(w[(size_t)j * N + n]));
}

/* ------------------------------------------------- quantise / pack / dequant */

static int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

/* Eq. 1 applied to one group of `group` consecutive input channels of one
 * output column (Sec 2.2: group-wise, the group axis read as the input-channel
 * axis K).  Readings where Eq. 1 is silent:
 *   - the range is widened to contain 0, so that Z lands in [0,15]; identical
 *     to Eq. 1 whenever min <= 0 <= max;
 *   - the step is computed in fp32, rounded once to fp16, and the ROUNDED step
 *     is what Z, the codes and the dequantised weights are computed with;
 *   - a zero step (constant-zero group) is replaced by 2^-24;
 *   - Z = round(-lo / step), the choice that maps lo to code 0;
 *   - round() is round-half-to-even.
 * Writes the fp16 step, the zero point and `group` codes (0..15). */
static void quant_group(int group, const uint16_t *w, size_t stride,
                        uint16_t *step16, uint8_t *zero, uint8_t *codes)
{
    float wmin = orc_h2f(w[0]), wmax = wmin;
    for (int i = 1; i < group; i++) {
        float v = orc_h2f(w[(size_t)i * stride]);
        if (v < wmin) wmin = v;
        if (v > wmax) wmax = v;
    }
    float lo = wmin < 0.0f ? wmin : 0.0f;
    float hi = wmax > 0.0f ? wmax : 0.0f;
    float d32 = (hi - lo) / 15.0f;
    uint16_t d16 = orc_f2h(d32);
    if ((d16 & 0x7fffu) == 0) d16 = 0x0001u;
    float d = orc_h2f(d16);
    int z = clampi((int)rintf(-lo / d), 0, 15);
    for (int i = 0; i < group; i++) {
        float v = orc_h2f(w[(size_t)i * stride]);
        codes[i] = (uint8_t)clampi((int)rintf(v / d) + z, 0, 15);
    }
    *step16 = d16;
    *zero = (uint8_t)z;
}

/* Group-wise 4-bit quantisation of W[K][N] (Eq. 1, Sec 2.2) and packing:
 * word packed[j][n] holds the codes of k = 8j .. 8j+7 of column n, the code of
 * k = 8j+i in bits [4i+3 : 4i].  scales/zeros are [K/group][N]. */
void orc_quantize_pack(int N, int K, int group, const uint16_t *w, uint32_t *packed,
                       uint16_t *scales, uint8_t *zeros)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)group);
    for (int t = 0; t < K / group; t++)
        for (int n = 0; n < N; n++) {
            const uint16_t *w0 = w + (size_t)t * group * N + n;
            quant_group(group, w0, (size_t)N, &scales[(size_t)t * N + n],
                        &zeros[(size_t)t * N + n], codes);
            for (int j = 0; j < group / 8; j++) {
                uint32_t word = 0;
                for (int i = 0; i < 8; i++) word |= (uint32_t)codes[8 * j + i] << (4 * i);
                packed[((size_t)t * (group / 8) + j) * N + n] = word;
            }
        }
    free(codes);
}

/* code of weight (k, n) */
static int code_at(const uint32_t *packed, int N, int k, int n)
{
    return (int)((packed[(size_t)(k >> 3) * N + n] >> (4 * (k & 7))) & 0xfu);
}

/* Eq. 1, second line: w_hat = (code - Z) * step, as an fp16 value.  The fp32
 * product of a 5-bit integer and an 11-bit significand is exact, so this is a
 * single rounding. */
void orc_dequantize(int N, int K, int group, const uint32_t *packed, const uint16_t *scales,
                    const uint8_t *zeros, uint16_t *w_hat)
{
    for (int k = 0; k < K; k++)
        for (int n = 0; n < N; n++) {
            int t = k / group;
            float d = orc_h2f(scales[(size_t)t * N + n]);
            int z = zeros[(size_t)t * N + n];
            w_hat[(size_t)k * N + n] = orc_f2h((float)(code_at(packed, N, k, n) - z) * d);
        }
}

/* Unpack to one byte per code, [K][N] (test helper for the pack bijection). */
void orc_unpack(int N, int K, const uint32_t *packed, uint8_t *codes)
{
    for (int k = 0; k < K; k++)
        for (int n = 0; n < N; n++) codes[(size_t)k * N + n] = (uint8_t)code_at(packed, N, k, n);
}

/* ------------------------------------------------------------------- GEMM */

/* Eq. 3 as its definition: y[m][n] = sum_k x[m][k] * w_hat[k][n] with w_hat the
 * fp16 dequantised weight of Eq. 1; every product is exact in fp64 and the sum
 * runs in fp64 in plain k order.  Also returns t[m][n] = sum_k |x * w_hat|,
 * the magnitude the parity tolerance is stated against. */
void orc_w4a16_gemm_ref(int M, int N, int K, int group, const uint16_t *x,
                        const uint32_t *packed, const uint16_t *scales, const uint8_t *zeros,
                        double *y, double *t)
{
#pragma omp parallel
    {
        double *col = (double *)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; n++) {
            for (int k = 0; k < K; k++) {
                int g = k / group;
                float d = orc_h2f(scales[(size_t)g * N + n]);
                int z = zeros[(size_t)g * N + n];
                col[k] = (double)orc_h2f(orc_f2h((float)(code_at(packed, N, k, n) - z) * d));
            }
            for (int m = 0; m < M; m++) {
                double acc = 0.0, mag = 0.0;
                for (int k = 0; k < K; k++) {
                    double p = (double)orc_h2f(x[(size_t)m * K + k]) * col[k];
                    acc += p;
                    mag += fabs(p);
                }
                y[(size_t)m * N + n] = acc;
                if (t) t[(size_t)m * N + n] = mag;
            }
        }
        free(col);
    }
}

/* The same layer in the precision the method names (fp32 accumulate, one
 * rounding to fp16 at the end; Fig. 7: FP16 out).  Sequential k order.  This
 * is the variant the benchmark times as the CPU baseline. */
void orc_w4a16_gemm_f32(int M, int N, int K, int group, const uint16_t *x,
                        const uint32_t *packed, const uint16_t *scales, const uint8_t *zeros,
                        uint16_t *y)
{
    float *xf = (float *)malloc(sizeof(float) * (size_t)M * K);
    for (size_t i = 0; i < (size_t)M * K; i++) xf[i] = orc_h2f(x[i]);
#pragma omp parallel
    {
        float *col = (float *)malloc(sizeof(float) * (size_t)K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; n++) {
            for (int k = 0; k < K; k++) {
                int g = k / group;
                float d = orc_h2f(scales[(size_t)g * N + n]);
                int z = zeros[(size_t)g * N + n];
                col[k] = orc_h2f(orc_f2h((float)(code_at(packed, N, k, n) - z) * d));
            }
            for (int m = 0; m < M; m++) {
                float acc = 0.0f;
                for (int k = 0; k < K; k++) acc += xf[(size_t)m * K + k] * col[k];
                y[(size_t)m * N + n] = orc_f2h(acc);
            }
        }
        free(col);
    }
    free(xf);
}

/* Eq. 4: E = || X W - X_hat W_hat ||_2^2 in fp64.  W and W_hat are fp16 [K][N];
 * X_hat is the activation that multiplies W_hat (X itself for plain rounding,
 * X diag(s)^-1 after smoothing, Eq. 5). */
double orc_quant_loss(int M, int N, int K, const uint16_t *x, const uint16_t *w,
                      const uint16_t *x_hat, const uint16_t *w_hat)
{
    double e = 0.0;
#pragma omp parallel for reduction(+ : e) schedule(static)
    for (int n = 0; n < N; n++)
        for (int m = 0; m < M; m++) {
            double a = 0.0, b = 0.0;
            for (int k = 0; k < K; k++) {
                a += (double)orc_h2f(x[(size_t)m * K + k]) * (double)orc_h2f(w[(size_t)k * N + n]);
                b += (double)orc_h2f(x_hat[(size_t)m * K + k]) *
                     (double)orc_h2f(w_hat[(size_t)k * N + n]);
            }
            e += (a - b) * (a - b);
        }
    return e;
}

/* Threads the OpenMP loops above will use (reported beside the CPU baseline). */
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

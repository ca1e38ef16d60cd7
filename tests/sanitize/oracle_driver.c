/* Runs every function of the CPU oracle on small ragged shapes with exactly sized heap buffers;
 * built with AddressSanitizer and UndefinedBehaviorSanitizer by tests/test_host_sanitizers.py, so
 * that any out-of-bounds access or undefined operation in the oracle aborts the run. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

float orc_h2f(uint16_t h);
uint16_t orc_f2h(float f);
void orc_h2f_array(size_t n, const uint16_t *h, float *f);
void orc_f2h_array(size_t n, const float *f, uint16_t *h);
void orc_absmax_x(int T, int K, const uint16_t *x, float *ax);
void orc_absmax_w(int K, int N, const uint16_t *w, float *aw);
void orc_smooth_factor(int K, float alpha, const float *ax, const float *aw, float *s);
void orc_smooth_scales(int T, int K, int N, float alpha, const uint16_t *xcal, const uint16_t *w, float *s);
void orc_smooth_apply_x(int M, int K, const uint16_t *x, const float *s, uint16_t *xo);
void orc_smooth_apply_w(int K, int N, const uint16_t *w, const float *s, uint16_t *wo);
void orc_quantize_pack(int N, int K, int group, const uint16_t *w, uint32_t *packed, uint16_t *scales, uint8_t *zeros);
void orc_dequantize(int N, int K, int group, const uint32_t *packed, const uint16_t *scales, const uint8_t *zeros, uint16_t *w_hat);
void orc_unpack(int N, int K, const uint32_t *packed, uint8_t *codes);
void orc_w4a16_gemm_ref(int M, int N, int K, int group, const uint16_t *x, const uint32_t *packed, const uint16_t *scales,
                        const uint8_t *zeros, double *y, double *t);
void orc_w4a16_gemm_f32(int M, int N, int K, int group, const uint16_t *x, const uint32_t *packed, const uint16_t *scales,
                        const uint8_t *zeros, uint16_t *y);
double orc_quant_loss(int M, int N, int K, const uint16_t *x, const uint16_t *w, const uint16_t *x_hat, const uint16_t *w_hat);
int orc_num_threads(void);

static uint32_t rng_state = 12345u;
static float rnd(void)  /* uniform in [-1, 1) */
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return (float)(rng_state >> 8) / 8388608.0f - 1.0f;
}

static int run(int T, int M, int K, int N, int group)
{
    size_t kn = (size_t)K * N, groups = (size_t)(K / group) * N;
    uint16_t *xcal = malloc(sizeof(uint16_t) * T * K), *x = malloc(sizeof(uint16_t) * M * K), *w = malloc(sizeof(uint16_t) * kn);
    uint16_t *xs = malloc(sizeof(uint16_t) * M * K), *ws = malloc(sizeof(uint16_t) * kn), *what = malloc(sizeof(uint16_t) * kn);
    uint16_t *scales = malloc(sizeof(uint16_t) * groups), *y16 = malloc(sizeof(uint16_t) * M * N);
    uint8_t *zeros = malloc(groups), *codes = malloc(kn);
    uint32_t *packed = malloc(sizeof(uint32_t) * (K / 8) * N);
    float *s = malloc(sizeof(float) * K), *ax = malloc(sizeof(float) * K), *aw = malloc(sizeof(float) * K), *s2 = malloc(sizeof(float) * K);
    double *y = malloc(sizeof(double) * M * N), *t = malloc(sizeof(double) * M * N);
    for (size_t i = 0; i < (size_t)T * K; i++) xcal[i] = orc_f2h(rnd() * ((i % K) == 3 ? 50.0f : 1.0f));
    for (size_t i = 0; i < (size_t)M * K; i++) x[i] = orc_f2h(rnd());
    for (size_t i = 0; i < kn; i++) w[i] = orc_f2h(0.05f * rnd());
    for (int k = 0; k < K; k++) w[(size_t)k * N] = 0;       /* a constant-zero column: the step floor */
    orc_absmax_x(T, K, xcal, ax);
    orc_absmax_w(K, N, w, aw);
    orc_smooth_factor(K, 0.5f, ax, aw, s2);
    orc_smooth_scales(T, K, N, 0.5f, xcal, w, s);
    int bad = 0;
    for (int k = 0; k < K; k++) bad += s[k] != s2[k];
    orc_smooth_apply_x(M, K, x, s, xs);
    orc_smooth_apply_w(K, N, w, s, ws);
    orc_quantize_pack(N, K, group, ws, packed, scales, zeros);
    orc_dequantize(N, K, group, packed, scales, zeros, what);
    orc_unpack(N, K, packed, codes);
    for (size_t i = 0; i < kn; i++) bad += codes[i] > 15;
    for (size_t i = 0; i < groups; i++) bad += zeros[i] > 15;
    orc_w4a16_gemm_ref(M, N, K, group, xs, packed, scales, zeros, y, t);
    orc_w4a16_gemm_f32(M, N, K, group, xs, packed, scales, zeros, y16);
    for (size_t i = 0; i < (size_t)M * N; i++) bad += !(t[i] >= 0.0) || y[i] != y[i];
    double e = orc_quant_loss(M, N, K, x, w, xs, what);
    bad += !(e >= 0.0);
    float f[3] = {1.0f, -2.5f, 65504.0f};
    uint16_t h[3];
    orc_f2h_array(3, f, h);
    orc_h2f_array(3, h, f);
    bad += f[1] != -2.5f || orc_h2f(h[2]) != 65504.0f;
    free(xcal); free(x); free(w); free(xs); free(ws); free(what); free(scales); free(y16); free(zeros); free(codes);
    free(packed); free(s); free(ax); free(aw); free(s2); free(y); free(t);
    return bad;
}

int main(void)
{
    int bad = 0;
    bad += run(5, 3, 128, 8, 128);
    bad += run(7, 1, 256, 24, 32);
    bad += run(3, 4, 48, 16, 24);
    bad += run(9, 2, 64, 8, 8);
    bad += run(4, 5, 256, 40, 256);
    if (orc_num_threads() < 1) bad++;
    printf("oracle sanitizer run: %d inconsistencies\n", bad);
    return bad != 0;
}

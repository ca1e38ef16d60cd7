// Companion kernels of the W4A16 layer: smoothing factors (Eq. 6), smoothing of
// activations and weights (Eq. 5), group-wise 4-bit quantise + pack and dequantise
// (Eq. 1, Sec 2.2) of arXiv 2312.03788.  All are single streaming passes, bound by HBM
// bandwidth; every result here is defined bit-exactly (IEEE fp32 divide/multiply, one
// round-to-nearest-even to fp16), so no fast-math and no FMA contraction in this file.
#include "sqp_common.h"

#pragma clang fp contract(off)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Streaming accesses to the weight, every byte of which is touched once per call: the
// non-temporal hint lets them pass through the caches (a plain read probe streams 12-15 %
// faster with it on this chip; measured here: weight abs-max +7 %, weight scaling +4 %; no gain
// for quantise + pack, and a loss for the much smaller activation tensor, which stay plain).
__device__ __forceinline__ uint4 load_stream(const uint4 *p)
{
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(uint4 *p, const uint4 &v)
{
    __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(p));
}

namespace {

__device__ __forceinline__ float h2f_lo(uint32_t v) { return (float)__builtin_bit_cast(h16x2, v).x; }
__device__ __forceinline__ float h2f_hi(uint32_t v) { return (float)__builtin_bit_cast(h16x2, v).y; }
__device__ __forceinline__ uint32_t pack_h2(float a, float b)
{
    h16x2 r;
    r.x = (h16)a;
    r.y = (h16)b;
    return __builtin_bit_cast(uint32_t, r);
}

// ------------------------------------------------------------------ Eq. 6

__global__ void fill_zero_u32(uint32_t *p, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// max_t |x[t][j]|, accumulated into ax_bits[j] as the bit pattern of a non-negative
// float (unsigned order == float order there), so the atomic max is order-independent.
// Block: 32 column-octets x 8 row lanes.
__global__ void __launch_bounds__(256) absmax_x_kernel(int T, int K, const uint4 *x, uint32_t *ax_bits)
{
    __shared__ float red[8][256];
    const int oct = threadIdx.x & 31, rl = threadIdx.x >> 5;
    const int koct = blockIdx.x * 32 + oct;  // column octet
    const int KO = K >> 3;
    float m[8];
#pragma unroll
    for (int i = 0; i < 8; i++) m[i] = 0.0f;
    if (koct < KO) {
        for (int t = blockIdx.y * 8 + rl; t < T; t += 8 * gridDim.y) {
            uint4 v = x[(size_t)t * KO + koct];
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; i++) {
                m[2 * i] = fmaxf(m[2 * i], fabsf(h2f_lo(w[i])));
                m[2 * i + 1] = fmaxf(m[2 * i + 1], fabsf(h2f_hi(w[i])));
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; i++) red[rl][oct * 8 + i] = m[i];
    __syncthreads();
    const int col = blockIdx.x * 256 + threadIdx.x;
    if (col < K) {
        float r = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; i++) r = fmaxf(r, red[i][threadIdx.x]);
        atomicMax(&ax_bits[col], __builtin_bit_cast(uint32_t, r));
    }
}

__device__ __forceinline__ float smooth_factor_of(float ax, float aw, float alpha)
{
    ax = ax > 1e-5f ? ax : 1e-5f;
    aw = aw > 1e-5f ? aw : 1e-5f;
    const double a = (double)alpha;
    return (float)(pow((double)ax, a) / pow((double)aw, 1.0 - a));
}

// One block per input channel j: aw = max_n |w[j][n]|.  FACTOR: then Eq. 6 with ax read from
// s[j] (left there by absmax_x_kernel) and s[j] overwritten with the factor; otherwise aw is
// stored to s[j].
template <bool FACTOR>
__global__ void __launch_bounds__(256) absmax_w_kernel(int N, float alpha, const uint4 *w, float *s)
{
    __shared__ float red[4];
    const int j = blockIdx.x;
    const int NO = N >> 3;
    const uint4 *row = w + (size_t)j * NO;
    float m = 0.0f;
    for (int o = threadIdx.x; o < NO; o += 256) {
        const uint4 v = load_stream(row + o);
        uint32_t q[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; i++) m = fmaxf(m, fmaxf(fabsf(h2f_lo(q[i])), fabsf(h2f_hi(q[i]))));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float aw = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        s[j] = FACTOR ? smooth_factor_of(s[j], aw, alpha) : aw;
    }
}

// Eq. 6 from stored maxima: amax = [ax (K) | aw (K)].
__global__ void __launch_bounds__(256) smooth_factor_kernel(int K, float alpha, const float *amax, float *s)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j < K) s[j] = smooth_factor_of(amax[j], amax[K + j], alpha);
}

// ------------------------------------------------------------------ Eq. 5

__global__ void __launch_bounds__(256) apply_x_kernel(long total_oct, int KO, const uint4 *x, const float4 *s, uint4 *out)
{
    long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total_oct) return;
    int ko = (int)(i % KO);
    uint4 v = x[i];
    float4 s0 = s[2 * ko], s1 = s[2 * ko + 1];
    uint4 r;
    r.x = pack_h2(h2f_lo(v.x) / s0.x, h2f_hi(v.x) / s0.y);
    r.y = pack_h2(h2f_lo(v.y) / s0.z, h2f_hi(v.y) / s0.w);
    r.z = pack_h2(h2f_lo(v.z) / s1.x, h2f_hi(v.z) / s1.y);
    r.w = pack_h2(h2f_lo(v.w) / s1.z, h2f_hi(v.w) / s1.w);
    out[i] = r;
}

__global__ void __launch_bounds__(256) apply_w_kernel(long total_oct, int NO, const uint4 *w, const float *s, uint4 *out)
{
    long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total_oct) return;
    float sj = s[i / NO];
    uint4 v = load_stream(w + i);
    uint4 r;
    r.x = pack_h2(sj * h2f_lo(v.x), sj * h2f_hi(v.x));
    r.y = pack_h2(sj * h2f_lo(v.y), sj * h2f_hi(v.y));
    r.z = pack_h2(sj * h2f_lo(v.z), sj * h2f_hi(v.z));
    r.w = pack_h2(sj * h2f_lo(v.w), sj * h2f_hi(v.w));
    store_stream(out + i, r);
}

// ------------------------------------------------------------------ Eq. 1
#ifndef SQP_QP_SPLIT128
#define SQP_QP_SPLIT128 2   // threads sharing a group of 128 rows
#endif
#ifndef SQP_QP_SPLIT64
#define SQP_QP_SPLIT64 1
#endif

struct GroupParams {
    float d;     // the fp16-rounded step, as float
    uint16_t d16;
    int z;
};

__device__ __forceinline__ GroupParams group_params(float wmin, float wmax)
{
    float lo = wmin < 0.0f ? wmin : 0.0f;
    float hi = wmax > 0.0f ? wmax : 0.0f;
    float d32 = (hi - lo) / 15.0f;
    h16 dh = (h16)d32;
    uint16_t bits = __builtin_bit_cast(uint16_t, dh);
    if ((bits & 0x7fffu) == 0) bits = 0x0001u;
    GroupParams p;
    p.d16 = bits;
    p.d = (float)__builtin_bit_cast(h16, bits);
    int z = (int)rintf(-lo / p.d);
    p.z = z < 0 ? 0 : (z > 15 ? 15 : z);
    return p;
}

__device__ __forceinline__ uint32_t code_of(float v, const GroupParams &p)
{
    int q = (int)rintf(v / p.d) + p.z;
    q = q < 0 ? 0 : (q > 15 ? 15 : q);
    return (uint32_t)q;
}

// The code of Eq. 1 needs rint(v / d) with the correctly rounded quotient.  A full IEEE
// division per weight makes the kernel ALU-bound, so the quotient is first formed as
// t = v * (1 / d): |t - v/d| <= 2^-23 * |v/d| <= 1.8e-6 (|v/d| <= 15.01 because the group's
// range contains 0), and the rounded quotient lies within 0.9e-6 of v/d.  Unless t is within
// NEAR_TIE of a half-integer, rint(t) is therefore rint of the exact quotient; the rare
// words with such a value are redone with the division (a wave-uniform branch).
constexpr float NEAR_TIE = 4.0e-6f;

__device__ __forceinline__ uint32_t code_fast(float v, float inv, int z, bool &near_tie)
{
    const float t = v * inv;
    const float r = rintf(t);
    near_tie |= fabsf(t - r) >= 0.5f - NEAR_TIE;
    int q = (int)r + z;
    q = q < 0 ? 0 : (q > 15 ? 15 : q);
    return (uint32_t)q;
}

// SPLIT adjacent threads quantise one group of G rows of two adjacent columns, G / SPLIT rows
// each; the weights stay in registers between the min/max pass (exact packed fp16 min/max,
// combined across the SPLIT lanes by shuffles) and the coding pass.  Fewer rows per thread
// mean fewer registers and more waves in flight to overlap the loads of one with the
// arithmetic of another; with SPLIT = 2 a wave still reads whole 128-byte lines (32 column
// pairs of one row per half).  grid: (ceil(SPLIT * N/2 / 256), K/G), block 256.
template <int G, int SPLIT>
__global__ void __launch_bounds__(256) quantize_pack_reg_kernel(int N, const uint32_t *w, uint2 *packed, uint32_t *scales, uint16_t *zeros)
{
    constexpr int R = G / SPLIT;  // rows per thread
    static_assert(R % 8 == 0, "whole packed words per thread");
    const int gid = blockIdx.x * 256 + threadIdx.x;
    const int n2 = gid / SPLIT, part = gid % SPLIT;
    const int N2 = N >> 1;
    // N2 * SPLIT is a multiple of SPLIT, so the SPLIT lanes of a group are in or out together
    if (n2 >= N2) return;
    const int t = blockIdx.y;
    const uint32_t *wp = w + ((size_t)t * G + (size_t)part * R) * N2 + n2;
    uint32_t v[R];
#pragma unroll
    for (int i = 0; i < R; i++) v[i] = wp[(size_t)i * N2];
    h16x2 mn = __builtin_bit_cast(h16x2, v[0]), mx = mn;
#pragma unroll
    for (int i = 1; i < R; i++) {
        const h16x2 c = __builtin_bit_cast(h16x2, v[i]);
        mn = __builtin_elementwise_min(mn, c);
        mx = __builtin_elementwise_max(mx, c);
    }
#pragma unroll
    for (int off = 1; off < SPLIT; off <<= 1) {
        const h16x2 omn = __builtin_bit_cast(h16x2, __shfl_xor(__builtin_bit_cast(int, mn), off, 64));
        const h16x2 omx = __builtin_bit_cast(h16x2, __shfl_xor(__builtin_bit_cast(int, mx), off, 64));
        mn = __builtin_elementwise_min(mn, omn);
        mx = __builtin_elementwise_max(mx, omx);
    }
    const GroupParams p0 = group_params((float)mn.x, (float)mx.x), p1 = group_params((float)mn.y, (float)mx.y);
    if (part == 0) {
        scales[(size_t)t * N2 + n2] = (uint32_t)p0.d16 | ((uint32_t)p1.d16 << 16);
        zeros[(size_t)t * N2 + n2] = (uint16_t)(p0.z | (p1.z << 8));
    }
    const float inv0 = 1.0f / p0.d, inv1 = 1.0f / p1.d;
    uint2 *pp = packed + ((size_t)t * (G / 8) + (size_t)part * (R / 8)) * N2 + n2;
#pragma unroll
    for (int j = 0; j < R / 8; j++) {
        uint32_t w0 = 0, w1 = 0;
        bool near_tie = false;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            w0 |= code_fast(h2f_lo(v[8 * j + i]), inv0, p0.z, near_tie) << (4 * i);
            w1 |= code_fast(h2f_hi(v[8 * j + i]), inv1, p1.z, near_tie) << (4 * i);
        }
        if (__builtin_amdgcn_ballot_w64(near_tie) != 0ull) {
            w0 = 0;
            w1 = 0;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                w0 |= code_of(h2f_lo(v[8 * j + i]), p0) << (4 * i);
                w1 |= code_of(h2f_hi(v[8 * j + i]), p1) << (4 * i);
            }
        }
        pp[(size_t)j * N2] = make_uint2(w0, w1);
    }
}

// Groups of 128 rows, the configuration of every benchmark layer: a block of 256 threads
// quantises 128 rows x 256 columns.  Thread (part = tid / 32, oct = tid % 32) holds rows
// 16 part .. 16 part + 15 of columns 8 oct .. 8 oct + 7 in registers (16 loads of 16 bytes; a
// wave's load covers two rows x 512 contiguous bytes).  Column minima and maxima (exact packed
// fp16 min / max) meet in LDS; the step, the zero point and the reciprocal step of column
// 8 oct + part are then computed by thread (part, oct) alone (three IEEE divisions per column,
// not per thread and column) and handed to the other parts through LDS.  Coding pass, per
// weight: t = fma(w, 1 / Delta, Z) -- within 1.9e-6 of (correctly rounded w / Delta) + Z
// wherever the code is not clamped, see NEAR_TIE -- then round, clamp to [0, 15] as a float,
// and the eight codes of a word are assembled by a fused multiply-add chain (sum c_i 16^i per
// half word is exact in fp32).  A word containing a value within NEAR_TIE of a rounding tie is
// redone with the division of the definition (wave-uniform branch, about 0.4 % of the words).
__global__ void __launch_bounds__(256) quantize_pack_g128_kernel(int N, const uint4 *__restrict__ w, uint32_t *__restrict__ packed,
                                                                 uint16_t *__restrict__ scales, uint8_t *__restrict__ zeros)
{
    __shared__ uint4 red[8][2][32];     // [part][min | max][oct]: 8 KB
    __shared__ float par_d[256], par_inv[256], par_z[256];  // per column of the block
    const int oct = threadIdx.x & 31, part = threadIdx.x >> 5;
    const int NO = N >> 3;
    const int o = blockIdx.x * 32 + oct;
    const bool in = o < NO;
    const int t = blockIdx.y;
    const uint4 *wp = w + ((size_t)t * 128 + (size_t)part * 16) * NO + (in ? o : 0);
    uint4 v[16];
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = load_stream(wp + (size_t)i * NO);
    h16x2 mn[4], mx[4];
    {
        const uint32_t q[4] = {v[0].x, v[0].y, v[0].z, v[0].w};
#pragma unroll
        for (int c = 0; c < 4; c++) mn[c] = mx[c] = __builtin_bit_cast(h16x2, q[c]);
    }
#pragma unroll
    for (int i = 1; i < 16; i++) {
        const uint32_t q[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const h16x2 e = __builtin_bit_cast(h16x2, q[c]);
            mn[c] = __builtin_elementwise_min(mn[c], e);
            mx[c] = __builtin_elementwise_max(mx[c], e);
        }
    }
    auto as_u4 = [](const h16x2 (&a)[4]) {
        return make_uint4(__builtin_bit_cast(uint32_t, a[0]), __builtin_bit_cast(uint32_t, a[1]),
                          __builtin_bit_cast(uint32_t, a[2]), __builtin_bit_cast(uint32_t, a[3]));
    };
    red[part][0][oct] = as_u4(mn);
    red[part][1][oct] = as_u4(mx);
    __syncthreads();
    {
        // thread (part, oct): column 8 oct + part, i.e. half (part & 1) of dword (part >> 1) of the octet
        const uint32_t *rmn = reinterpret_cast<const uint32_t *>(&red[0][0][oct]) + (part >> 1);
        const uint32_t *rmx = reinterpret_cast<const uint32_t *>(&red[0][1][oct]) + (part >> 1);
        constexpr int PSTRIDE = 2 * 32 * 4;  // dwords between parts
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int pp = 0; pp < 8; pp++) {
            const h16x2 a = __builtin_bit_cast(h16x2, rmn[pp * PSTRIDE]), b = __builtin_bit_cast(h16x2, rmx[pp * PSTRIDE]);
            const float fa = (part & 1) ? (float)a.y : (float)a.x, fb = (part & 1) ? (float)b.y : (float)b.x;
            lo = pp == 0 ? fa : fminf(lo, fa);
            hi = pp == 0 ? fb : fmaxf(hi, fb);
        }
        const GroupParams gp = group_params(lo, hi);
        const int col = oct * 8 + part;
        par_d[col] = gp.d;
        par_inv[col] = 1.0f / gp.d;
        par_z[col] = (float)gp.z;
        const int n = blockIdx.x * 256 + col;
        if (n < N) {
            scales[(size_t)t * N + n] = gp.d16;
            zeros[(size_t)t * N + n] = (uint8_t)gp.z;
        }
    }
    __syncthreads();
    if (!in) return;
    uint32_t *pp0 = packed + ((size_t)t * 16 + (size_t)part * 2) * N + (size_t)o * 8;
#pragma unroll
    for (int j = 0; j < 2; j++) {
        uint32_t word[8];
#pragma unroll
        for (int c = 0; c < 8; c++) {
            const float inv = par_inv[oct * 8 + c], zf = par_z[oct * 8 + c];
            float code[8], worst = 0.f;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const uint4 &row = v[8 * j + i];
                const uint32_t dw = (c >> 1) == 0 ? row.x : ((c >> 1) == 1 ? row.y : ((c >> 1) == 2 ? row.z : row.w));
                const float x = (c & 1) ? h2f_hi(dw) : h2f_lo(dw);
                const float tq = fmaf(x, inv, zf);
                const float r = rintf(tq);
                worst = fmaxf(worst, fabsf(tq - r));
                code[i] = fminf(fmaxf(r, 0.0f), 15.0f);
            }
            const float lo4 = fmaf(fmaf(fmaf(code[3], 16.0f, code[2]), 16.0f, code[1]), 16.0f, code[0]);
            const float hi4 = fmaf(fmaf(fmaf(code[7], 16.0f, code[6]), 16.0f, code[5]), 16.0f, code[4]);
            word[c] = (uint32_t)lo4 | ((uint32_t)hi4 << 16);
            if (__builtin_amdgcn_ballot_w64(worst >= 0.5f - NEAR_TIE) != 0ull) {
                GroupParams gp;
                gp.d = par_d[oct * 8 + c];
                gp.z = (int)zf;
                gp.d16 = 0;
                uint32_t wd = 0;
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    const uint4 &row = v[8 * j + i];
                    const uint32_t dw = (c >> 1) == 0 ? row.x : ((c >> 1) == 1 ? row.y : ((c >> 1) == 2 ? row.z : row.w));
                    wd |= code_of((c & 1) ? h2f_hi(dw) : h2f_lo(dw), gp) << (4 * i);
                }
                word[c] = wd;
            }
        }
        uint4 *dst = reinterpret_cast<uint4 *>(pp0 + (size_t)j * N);
        dst[0] = make_uint4(word[0], word[1], word[2], word[3]);
        dst[1] = make_uint4(word[4], word[5], word[6], word[7]);
    }
}

// Any group size (multiple of 8): the group is read twice.
__global__ void __launch_bounds__(256) quantize_pack_any_kernel(int N, int G, const uint32_t *w, uint2 *packed, uint32_t *scales, uint16_t *zeros)
{
    const int n2 = blockIdx.x * 256 + threadIdx.x;
    const int N2 = N >> 1;
    if (n2 >= N2) return;
    const int t = blockIdx.y;
    const uint32_t *wp = w + (size_t)t * G * N2 + n2;
    uint32_t v0 = wp[0];
    float mn0 = h2f_lo(v0), mx0 = mn0, mn1 = h2f_hi(v0), mx1 = mn1;
    for (int i = 1; i < G; i++) {
        uint32_t v = wp[(size_t)i * N2];
        float a = h2f_lo(v), b = h2f_hi(v);
        mn0 = fminf(mn0, a);
        mx0 = fmaxf(mx0, a);
        mn1 = fminf(mn1, b);
        mx1 = fmaxf(mx1, b);
    }
    GroupParams p0 = group_params(mn0, mx0), p1 = group_params(mn1, mx1);
    scales[(size_t)t * N2 + n2] = (uint32_t)p0.d16 | ((uint32_t)p1.d16 << 16);
    zeros[(size_t)t * N2 + n2] = (uint16_t)(p0.z | (p1.z << 8));
    uint2 *pp = packed + (size_t)t * (G / 8) * N2 + n2;
    for (int j = 0; j < G / 8; j++) {
        uint32_t w0 = 0, w1 = 0;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            uint32_t v = wp[(size_t)(8 * j + i) * N2];
            w0 |= code_of(h2f_lo(v), p0) << (4 * i);
            w1 |= code_of(h2f_hi(v), p1) << (4 * i);
        }
        pp[(size_t)j * N2] = make_uint2(w0, w1);
    }
}

// One thread expands one packed word of two adjacent columns into 8 rows.
// grid: (ceil(N/512), K/8), block 256.
__global__ void __launch_bounds__(256) dequantize_kernel(int N, int words_per_group, const uint2 *packed, const uint32_t *scales, const uint16_t *zeros, uint32_t *w_hat)
{
    const int n2 = blockIdx.x * 256 + threadIdx.x;
    const int N2 = N >> 1;
    if (n2 >= N2) return;
    const int j = blockIdx.y;
    const int t = j / words_per_group;
    uint2 pw = packed[(size_t)j * N2 + n2];
    uint32_t sc = scales[(size_t)t * N2 + n2];
    uint16_t zz = zeros[(size_t)t * N2 + n2];
    float d0 = h2f_lo(sc), d1 = h2f_hi(sc);
    int z0 = zz & 0xff, z1 = zz >> 8;
    uint32_t *out = w_hat + (size_t)j * 8 * N2 + n2;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        int q0 = (int)((pw.x >> (4 * i)) & 15u), q1 = (int)((pw.y >> (4 * i)) & 15u);
        out[(size_t)i * N2] = pack_h2((float)(q0 - z0) * d0, (float)(q1 - z1) * d1);
    }
}

}  // namespace

extern "C" int sqp_smooth_scales(int T, int K, int N, float alpha, const void *x_cal, const void *w, float *s, void *stream)
{
    if (!x_cal || !w || !s) return SQP_ERR_NULL;
    if (T <= 0 || K <= 0 || N <= 0 || (K % 8) || (N % 8)) return SQP_ERR_SHAPE;
    if (sqp_too_big(T, K) || sqp_too_big(K, N)) return SQP_ERR_SHAPE;
    if (sqp_misaligned(x_cal) || sqp_misaligned(w) || sqp_misaligned(s)) return SQP_ERR_ALIGN;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return SQP_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    fill_zero_u32<<<(K + 255) / 256, 256, 0, st>>>((uint32_t *)s, K);
    int gy = (T + 63) / 64;
    if (gy > 64) gy = 64;
    absmax_x_kernel<<<dim3((K + 255) / 256, gy), 256, 0, st>>>(T, K, (const uint4 *)x_cal, (uint32_t *)s);
    absmax_w_kernel<true><<<K, 256, 0, st>>>(N, alpha, (const uint4 *)w, s);
    return sqp_launch_status();
}

// The two halves of sqp_smooth_scales as separate steps (the per-channel maxima do not depend on
// alpha, so a search over alpha computes them once): amax = [max_t|x_cal[t][j]| (K) | max_n|w[j][n]| (K)].
int sqp_channel_absmax(int T, int K, int N, const void *x_cal, const void *w, float *amax, hipStream_t st)
{
    fill_zero_u32<<<(K + 255) / 256, 256, 0, st>>>((uint32_t *)amax, K);
    int gy = (T + 63) / 64;
    if (gy > 64) gy = 64;
    absmax_x_kernel<<<dim3((K + 255) / 256, gy), 256, 0, st>>>(T, K, (const uint4 *)x_cal, (uint32_t *)amax);
    absmax_w_kernel<false><<<K, 256, 0, st>>>(N, 0.0f, (const uint4 *)w, amax + K);
    return sqp_launch_status();
}

int sqp_smooth_factor(int K, float alpha, const float *amax, float *s, hipStream_t st)
{
    smooth_factor_kernel<<<(K + 255) / 256, 256, 0, st>>>(K, alpha, amax, s);
    return sqp_launch_status();
}

extern "C" int sqp_smooth_apply_x(int M, int K, const void *x, const float *s, void *x_out, void *stream)
{
    if (!x || !s || !x_out) return SQP_ERR_NULL;
    if (M <= 0 || K <= 0 || (K % 8) || sqp_too_big(M, K)) return SQP_ERR_SHAPE;
    if (sqp_misaligned(x) || sqp_misaligned(s) || sqp_misaligned(x_out)) return SQP_ERR_ALIGN;
    long total = (long)M * (K / 8);
    apply_x_kernel<<<(unsigned)((total + 255) / 256), 256, 0, (hipStream_t)stream>>>(total, K / 8, (const uint4 *)x, (const float4 *)s, (uint4 *)x_out);
    return sqp_launch_status();
}

extern "C" int sqp_smooth_apply_w(int K, int N, const void *w, const float *s, void *w_out, void *stream)
{
    if (!w || !s || !w_out) return SQP_ERR_NULL;
    if (K <= 0 || N <= 0 || (N % 8) || sqp_too_big(K, N)) return SQP_ERR_SHAPE;
    if (sqp_misaligned(w) || sqp_misaligned(s) || sqp_misaligned(w_out)) return SQP_ERR_ALIGN;
    long total = (long)K * (N / 8);
    apply_w_kernel<<<(unsigned)((total + 255) / 256), 256, 0, (hipStream_t)stream>>>(total, N / 8, (const uint4 *)w, s, (uint4 *)w_out);
    return sqp_launch_status();
}

// fp16 [N][K] (one row per output feature, the orientation checkpoints store) -> [K][N] (the
// orientation of Eq. 2 that every other entry point takes).  64 x 64 tile per workgroup through
// LDS: 16-byte reads along K, 16-byte writes along N; the LDS row stride of 66 halves keeps the
// 2-byte column reads of a wave on different banks.  grid: (K/64 rounded up, N/64 rounded up).
__global__ void __launch_bounds__(256) transpose_nk_kernel(int N, int K, const h16 *__restrict__ in, h16 *__restrict__ out)
{
    __shared__ h16 tile[64][66];
    const int k0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    const int r = threadIdx.x >> 3, c8 = (threadIdx.x & 7) * 8;
#pragma unroll
    for (int rr = 0; rr < 64; rr += 32) {
        const int n = n0 + r + rr, k = k0 + c8;
        h16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (n < N && k < K) v = *reinterpret_cast<const h16x8 *>(in + (size_t)n * K + k);  // K % 8 == 0
#pragma unroll
        for (int i = 0; i < 8; i++) tile[r + rr][c8 + i] = v[i];
    }
    __syncthreads();
#pragma unroll
    for (int rr = 0; rr < 64; rr += 32) {
        const int k = k0 + r + rr, n = n0 + c8;
        if (k < K && n < N) {                                                              // N % 8 == 0
            h16x8 v;
#pragma unroll
            for (int i = 0; i < 8; i++) v[i] = tile[c8 + i][r + rr];
            *reinterpret_cast<h16x8 *>(out + (size_t)k * N + n) = v;
        }
    }
}

extern "C" int sqp_transpose_nk(int N, int K, const void *w_nk, void *w_kn, void *stream)
{
    if (!w_nk || !w_kn) return SQP_ERR_NULL;
    if (N <= 0 || K <= 0 || (N % 8) || (K % 8) || sqp_too_big(K, N)) return SQP_ERR_SHAPE;
    if (sqp_misaligned(w_nk) || sqp_misaligned(w_kn)) return SQP_ERR_ALIGN;
    if ((N + 63) / 64 > 65535) return SQP_ERR_SHAPE;
    transpose_nk_kernel<<<dim3((K + 63) / 64, (N + 63) / 64), 256, 0, (hipStream_t)stream>>>(N, K, (const h16 *)w_nk, (h16 *)w_kn);
    return sqp_launch_status();
}

extern "C" int sqp_quantize_pack(int N, int K, int group, const void *w, uint32_t *packed, void *scales, uint8_t *zeros, void *stream)
{
    if (!w || !packed || !scales || !zeros) return SQP_ERR_NULL;
    int rc = sqp_check_quant_shape(N, K, group);
    if (rc) return rc;
    if (K / group > 65535) return SQP_ERR_SHAPE;
    if (sqp_misaligned(w) || sqp_misaligned(packed) || sqp_misaligned(scales) || sqp_misaligned(zeros)) return SQP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    dim3 grid((N / 2 + 255) / 256, K / group);
    dim3 grid2((N + 255) / 256, K / group);  // two threads per column pair
    const uint32_t *wp = (const uint32_t *)w;
    uint2 *pp = (uint2 *)packed;
    uint32_t *sp = (uint32_t *)scales;
    uint16_t *zp = (uint16_t *)zeros;
    switch (group) {
        case 32: quantize_pack_reg_kernel<32, 1><<<grid, 256, 0, st>>>(N, wp, pp, sp, zp); break;
        case 64: quantize_pack_reg_kernel<64, SQP_QP_SPLIT64><<<SQP_QP_SPLIT64 == 2 ? grid2 : grid, 256, 0, st>>>(N, wp, pp, sp, zp); break;
        case 128:
            quantize_pack_g128_kernel<<<dim3((N + 255) / 256, K / 128), 256, 0, st>>>(N, (const uint4 *)w, packed, (uint16_t *)scales, zeros);
            break;
        default: quantize_pack_any_kernel<<<grid, 256, 0, st>>>(N, group, wp, pp, sp, zp); break;
    }
    return sqp_launch_status();
}

extern "C" int sqp_dequantize(int N, int K, int group, const uint32_t *packed, const void *scales, const uint8_t *zeros, void *w_hat, void *stream)
{
    if (!packed || !scales || !zeros || !w_hat) return SQP_ERR_NULL;
    int rc = sqp_check_quant_shape(N, K, group);
    if (rc) return rc;
    if (K / 8 > 65535) return SQP_ERR_SHAPE;
    if (sqp_misaligned(packed) || sqp_misaligned(scales) || sqp_misaligned(zeros) || sqp_misaligned(w_hat)) return SQP_ERR_ALIGN;
    dim3 grid((N / 2 + 255) / 256, K / 8);
    dequantize_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(N, group / 8, (const uint2 *)packed, (const uint32_t *)scales, (const uint16_t *)zeros, (uint32_t *)w_hat);
    return sqp_launch_status();
}

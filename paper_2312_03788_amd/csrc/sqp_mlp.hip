// Companion kernels of the offline fusion on a LlamaMLP block (Sec 2.2 and Fig. 5 of
// arXiv 2312.03788): the smoothing factor of gate_proj / up_proj is divided into the weight of
// the RMSNorm in front of them, the one of down_proj into up_proj's output columns, so that no
// separate division of the activations runs at inference time.
//   sqp_rmsnorm             LlamaRMSNorm with a (possibly folded) fp16 weight
//   sqp_scale_columns       w[k][n] / s[n]: fold a smoothing factor into the producing layer
//   sqp_interleave_gate_up  merged gate+up weight with gate j / up j in adjacent columns, the
//                           layout whose GEMM epilogue forms SiLU(gate) * up
// All three are single streaming passes (HBM-bound, 16-byte accesses).
#include "sqp_common.h"

namespace {

__device__ __forceinline__ float lo_of(uint32_t v) { return (float)__builtin_bit_cast(h16x2, v).x; }
__device__ __forceinline__ float hi_of(uint32_t v) { return (float)__builtin_bit_cast(h16x2, v).y; }
__device__ __forceinline__ uint32_t pack2(float a, float b)
{
    h16x2 r;
    r.x = (h16)a;
    r.y = (h16)b;
    return __builtin_bit_cast(uint32_t, r);
}

// One workgroup per row: sum of squares in fp32 (per-thread partial over 8-element pieces,
// wave shuffles, then the 4 wave sums in a fixed order), then y = fp16(x * r * gamma) with
// r = 1 / sqrt(mean + eps).  The row is read twice (the second read hits the cache).
__global__ void __launch_bounds__(256) rmsnorm_kernel(int H8, float inv_h, float eps, const uint4 *__restrict__ x,
                                                      const uint4 *__restrict__ gamma, uint4 *__restrict__ y)
{
    __shared__ float red[4];
    const uint4 *xr = x + (size_t)blockIdx.x * H8;
    float ss = 0.f;
    for (int i = threadIdx.x; i < H8; i += 256) {
        const uint4 v = xr[i];
        const float a0 = lo_of(v.x), a1 = hi_of(v.x), a2 = lo_of(v.y), a3 = hi_of(v.y);
        const float a4 = lo_of(v.z), a5 = hi_of(v.z), a6 = lo_of(v.w), a7 = hi_of(v.w);
        ss += ((a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3)) + ((a4 * a4 + a5 * a5) + (a6 * a6 + a7 * a7));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float total = (red[0] + red[1]) + (red[2] + red[3]);
    const float r = 1.0f / sqrtf(total * inv_h + eps);
    uint4 *yr = y + (size_t)blockIdx.x * H8;
    for (int i = threadIdx.x; i < H8; i += 256) {
        const uint4 v = xr[i], g = gamma[i];
        uint4 o;
        o.x = pack2(lo_of(v.x) * r * lo_of(g.x), hi_of(v.x) * r * hi_of(g.x));
        o.y = pack2(lo_of(v.y) * r * lo_of(g.y), hi_of(v.y) * r * hi_of(g.y));
        o.z = pack2(lo_of(v.z) * r * lo_of(g.z), hi_of(v.z) * r * hi_of(g.z));
        o.w = pack2(lo_of(v.w) * r * lo_of(g.w), hi_of(v.w) * r * hi_of(g.w));
        yr[i] = o;
    }
}

// The same with the row held in registers between the two passes (rows of up to 2048 NI halves):
// the input is read once.  The sum of squares is formed in the same order as above, so both
// kernels give the same bits.
template <int NI>
__global__ void __launch_bounds__(256) rmsnorm_reg_kernel(int H8, float inv_h, float eps, const uint4 *__restrict__ x,
                                                          const uint4 *__restrict__ gamma, uint4 *__restrict__ y)
{
    __shared__ float red[4];
    const uint4 *xr = x + (size_t)blockIdx.x * H8;
    uint4 v[NI];
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < NI; j++) {
        const int i = threadIdx.x + 256 * j;
        v[j] = make_uint4(0, 0, 0, 0);
        if (i < H8) {
            v[j] = xr[i];
            const float a0 = lo_of(v[j].x), a1 = hi_of(v[j].x), a2 = lo_of(v[j].y), a3 = hi_of(v[j].y);
            const float a4 = lo_of(v[j].z), a5 = hi_of(v[j].z), a6 = lo_of(v[j].w), a7 = hi_of(v[j].w);
            ss += ((a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3)) + ((a4 * a4 + a5 * a5) + (a6 * a6 + a7 * a7));
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float total = (red[0] + red[1]) + (red[2] + red[3]);
    const float r = 1.0f / sqrtf(total * inv_h + eps);
    uint4 *yr = y + (size_t)blockIdx.x * H8;
#pragma unroll
    for (int j = 0; j < NI; j++) {
        const int i = threadIdx.x + 256 * j;
        if (i < H8) {
            const uint4 g = gamma[i];
            uint4 o;
            o.x = pack2(lo_of(v[j].x) * r * lo_of(g.x), hi_of(v[j].x) * r * hi_of(g.x));
            o.y = pack2(lo_of(v[j].y) * r * lo_of(g.y), hi_of(v[j].y) * r * hi_of(g.y));
            o.z = pack2(lo_of(v[j].z) * r * lo_of(g.z), hi_of(v[j].z) * r * hi_of(g.z));
            o.w = pack2(lo_of(v[j].w) * r * lo_of(g.w), hi_of(v[j].w) * r * hi_of(g.w));
            yr[i] = o;
        }
    }
}

__global__ void __launch_bounds__(256) scale_columns_kernel(long total_oct, int NO, const uint4 *__restrict__ w,
                                                            const float4 *__restrict__ s, uint4 *__restrict__ out)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total_oct) return;
    const int c = (int)(i % NO);
    const float4 s0 = s[2 * c], s1 = s[2 * c + 1];
    const uint4 v = w[i];
    uint4 r;
    r.x = pack2(lo_of(v.x) / s0.x, hi_of(v.x) / s0.y);
    r.y = pack2(lo_of(v.y) / s0.z, hi_of(v.y) / s0.w);
    r.z = pack2(lo_of(v.z) / s1.x, hi_of(v.z) / s1.y);
    r.w = pack2(lo_of(v.w) / s1.z, hi_of(v.w) / s1.w);
    out[i] = r;
}

// One thread: 8 gate and 8 up columns of a row -> 16 interleaved columns.
__global__ void __launch_bounds__(256) interleave_kernel(long total_oct, int IO, const uint4 *__restrict__ wg,
                                                         const uint4 *__restrict__ wu, uint4 *__restrict__ out)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total_oct) return;
    const uint4 g = wg[i], u = wu[i];
    uint4 a, b;  // (g0,u0),(g1,u1),... : low halves of a gate/up dword pair, then the high halves
    a.x = __builtin_amdgcn_perm(u.x, g.x, 0x05040100u); a.y = __builtin_amdgcn_perm(u.x, g.x, 0x07060302u);
    a.z = __builtin_amdgcn_perm(u.y, g.y, 0x05040100u); a.w = __builtin_amdgcn_perm(u.y, g.y, 0x07060302u);
    b.x = __builtin_amdgcn_perm(u.z, g.z, 0x05040100u); b.y = __builtin_amdgcn_perm(u.z, g.z, 0x07060302u);
    b.z = __builtin_amdgcn_perm(u.w, g.w, 0x05040100u); b.w = __builtin_amdgcn_perm(u.w, g.w, 0x07060302u);
    const long row = i / IO, c = i % IO;
    uint4 *o = out + (row * IO + c) * 2;
    o[0] = a;
    o[1] = b;
}

}  // namespace

extern "C" int sqp_rmsnorm(int M, int H, const void *x, const void *gamma, float eps, void *y, void *stream)
{
    if (!x || !gamma || !y) return SQP_ERR_NULL;
    if (M <= 0 || H <= 0 || (H % 8) || sqp_too_big(M, H)) return SQP_ERR_SHAPE;
    if (!(eps >= 0.0f) || !(eps < 1.0f)) return SQP_ERR_ARG;
    if (sqp_misaligned(x) || sqp_misaligned(gamma) || sqp_misaligned(y)) return SQP_ERR_ALIGN;
    const int H8 = H / 8;
    const float inv_h = 1.0f / (float)H;
    hipStream_t st = (hipStream_t)stream;
    const uint4 *xp = (const uint4 *)x, *gp = (const uint4 *)gamma;
    uint4 *yp = (uint4 *)y;
    if (H8 <= 256) rmsnorm_reg_kernel<1><<<(unsigned)M, 256, 0, st>>>(H8, inv_h, eps, xp, gp, yp);
    else if (H8 <= 512) rmsnorm_reg_kernel<2><<<(unsigned)M, 256, 0, st>>>(H8, inv_h, eps, xp, gp, yp);
    else if (H8 <= 1024) rmsnorm_reg_kernel<4><<<(unsigned)M, 256, 0, st>>>(H8, inv_h, eps, xp, gp, yp);
    else if (H8 <= 2048) rmsnorm_reg_kernel<8><<<(unsigned)M, 256, 0, st>>>(H8, inv_h, eps, xp, gp, yp);
    else if (H8 <= 4096) rmsnorm_reg_kernel<16><<<(unsigned)M, 256, 0, st>>>(H8, inv_h, eps, xp, gp, yp);
    else rmsnorm_kernel<<<(unsigned)M, 256, 0, st>>>(H8, inv_h, eps, xp, gp, yp);
    return sqp_launch_status();
}

extern "C" int sqp_scale_columns(int K, int N, const void *w, const float *s, void *w_out, void *stream)
{
    if (!w || !s || !w_out) return SQP_ERR_NULL;
    if (K <= 0 || N <= 0 || (N % 8) || sqp_too_big(K, N)) return SQP_ERR_SHAPE;
    if (sqp_misaligned(w) || sqp_misaligned(s) || sqp_misaligned(w_out)) return SQP_ERR_ALIGN;
    const long total = (long)K * (N / 8);
    scale_columns_kernel<<<(unsigned)((total + 255) / 256), 256, 0, (hipStream_t)stream>>>(total, N / 8, (const uint4 *)w, (const float4 *)s, (uint4 *)w_out);
    return sqp_launch_status();
}

extern "C" int sqp_interleave_gate_up(int K, int I, const void *w_gate, const void *w_up, void *w_out, void *stream)
{
    if (!w_gate || !w_up || !w_out) return SQP_ERR_NULL;
    if (K <= 0 || I <= 0 || (I % 8) || sqp_too_big(K, 2L * I)) return SQP_ERR_SHAPE;
    if (sqp_misaligned(w_gate) || sqp_misaligned(w_up) || sqp_misaligned(w_out)) return SQP_ERR_ALIGN;
    const long total = (long)K * (I / 8);
    interleave_kernel<<<(unsigned)((total + 255) / 256), 256, 0, (hipStream_t)stream>>>(total, I / 8, (const uint4 *)w_gate, (const uint4 *)w_up, (uint4 *)w_out);
    return sqp_launch_status();
}

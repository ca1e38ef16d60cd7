// Entry point of the quantised linear layer (Eq. 3 of arXiv 2312.03788): argument checks
// and the choice between the weight-streaming path (small M) and the tiled matrix-core
// path (large M).
#include "sqp_common.h"

extern "C" const char *sqp_status_string(int status)
{
    switch (status) {
        case SQP_OK: return "ok";
        case SQP_ERR_NULL: return "null pointer";
        case SQP_ERR_SHAPE: return "shape rule violated";
        case SQP_ERR_ALIGN: return "pointer not 16-byte aligned";
        case SQP_ERR_ARG: return "argument out of range";
        case SQP_ERR_LAUNCH: return "HIP launch error";
        case SQP_ERR_WORKSPACE: return "device workspace unavailable";
        default: return "unknown status";
    }
}

// Plain device copy (16 bytes per lane, grid-stride): a kernel of known traffic that the
// benchmark can run to calibrate hardware byte counters.  Benchmark hook, not part of the ABI.
__global__ void __launch_bounds__(256) plain_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) dst[i] = src[i];
}
extern "C" int sqp_debug_plain_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst || (bytes & 15)) return SQP_ERR_SHAPE;
    plain_copy_kernel<<<8192, 256, 0, (hipStream_t)stream>>>((const uint4 *)src, (uint4 *)dst, bytes / 16);
    return sqp_launch_status();
}

// Plain streaming read (16 bytes per lane, eight loads in flight per lane, grid-stride), with or
// without the non-temporal hint: the read bandwidth the chip reaches with nothing else to do,
// the reference the weight-streaming GEMM is measured against beside the published peak.
// Benchmark hook, not part of the ABI.
typedef uint32_t probe_u32x4 __attribute__((ext_vector_type(4)));
template <bool NT>
__global__ void __launch_bounds__(256) read_probe_kernel(const probe_u32x4 *__restrict__ src, size_t n, uint32_t *__restrict__ sink)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    uint32_t acc = 0;
    for (; i + 7 * stride < n; i += 8 * stride) {
        probe_u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = NT ? __builtin_nontemporal_load(src + i + j * stride) : src[i + j * stride];
#pragma unroll
        for (int j = 0; j < 8; j++) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;  // keeps the loads alive; practically never taken
}
extern "C" int sqp_debug_read_probe(const void *src, size_t bytes, int nt, int blocks, void *sink, void *stream)
{
    if (!src || !sink || (bytes & 15) || blocks <= 0 || blocks > 65535) return SQP_ERR_SHAPE;
    const size_t n = bytes / 16;
    if (nt) read_probe_kernel<true><<<blocks, 256, 0, (hipStream_t)stream>>>((const probe_u32x4 *)src, n, (uint32_t *)sink);
    else read_probe_kernel<false><<<blocks, 256, 0, (hipStream_t)stream>>>((const probe_u32x4 *)src, n, (uint32_t *)sink);
    return sqp_launch_status();
}

// A loop of nothing but independent 32x32x16 fp16 MFMAs (16 accumulator tiles per wave, four
// waves per workgroup, operands taken from `data`): the rate the matrix cores sustain on this
// chip for the given operand values, i.e. the ceiling the tiled GEMM is measured against
// beside the published peak.  Benchmark hook, not part of the ABI.
__global__ void __launch_bounds__(256) mfma_ceiling_kernel(const h16x8 *__restrict__ data, float *__restrict__ out, int iters)
{
    h16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        a[i] = data[(threadIdx.x + 256 * i) & 4095];
        b[i] = data[(threadIdx.x + 256 * (i + 4)) & 4095];
    }
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) sum += acc[i][j][r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = sum;
}
// data: 64 KiB of fp16 values on the device; out: blocks * 256 floats.  Flops of the launch:
// blocks * 4 waves * iters * 16 MFMAs * 32768.
extern "C" int sqp_debug_mfma_ceiling(const void *data, float *out, int blocks, int iters, void *stream)
{
    if (!data || !out || blocks <= 0 || iters <= 0) return SQP_ERR_ARG;
    mfma_ceiling_kernel<<<blocks, 256, 0, (hipStream_t)stream>>>((const h16x8 *)data, out, iters);
    return sqp_launch_status();
}

static int g_decode_max_m = 64;
// Test/benchmark hook: rows up to which the weight-streaming path is used.
extern "C" void sqp_debug_set_decode_max_m(int m) { g_decode_max_m = m; }

// ---------------------------------------------------------------- caller-owned workspace
// One per device, set by sqp_set_workspace; the library only keeps the pointer.
static SqpWorkspace g_caller_ws[64] = {};

__global__ void __launch_bounds__(256) zero_tickets_kernel(unsigned *t, unsigned n)
{
    const unsigned i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) t[i] = 0u;
}

int sqp_zero_tickets(unsigned *tickets, hipStream_t stream)
{
    zero_tickets_kernel<<<(unsigned)(SQP_WS_TICKETS / 256), 256, 0, stream>>>(tickets, (unsigned)SQP_WS_TICKETS);
    return sqp_launch_status();
}

SqpWorkspace sqp_caller_workspace()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SqpWorkspace{nullptr, nullptr, 0};
    return g_caller_ws[dev];
}

extern "C" int sqp_set_workspace(void *dev_ptr, size_t bytes, void *stream)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SQP_ERR_WORKSPACE;
    if (dev_ptr == nullptr || bytes == 0) {
        g_caller_ws[dev] = SqpWorkspace{nullptr, nullptr, 0};
        return SQP_OK;
    }
    if (sqp_misaligned(dev_ptr)) return SQP_ERR_ALIGN;
    if (bytes <= SQP_WS_TICKET_BYTES) return SQP_ERR_WORKSPACE;
    int rc = sqp_zero_tickets((unsigned *)dev_ptr, (hipStream_t)stream);
    if (rc) return rc;
    SqpWorkspace ws;
    ws.tickets = (unsigned *)dev_ptr;
    ws.partial = (float *)((unsigned char *)dev_ptr + SQP_WS_TICKET_BYTES);
    ws.partial_bytes = (bytes - SQP_WS_TICKET_BYTES) & ~(size_t)15;
    g_caller_ws[dev] = ws;
    return SQP_OK;
}

static int check_gemm_args(int M, int N, int K, int group, const void *x, const uint32_t *packed, const void *scales,
                           const uint8_t *zeros, const void *y)
{
    if (!x || !packed || !scales || !zeros || !y) return SQP_ERR_NULL;
    if (M <= 0) return SQP_ERR_SHAPE;
    int rc = sqp_check_quant_shape(N, K, group);
    if (rc) return rc;
    if (sqp_too_big(M, K) || sqp_too_big(M, N)) return SQP_ERR_SHAPE;
    if (sqp_misaligned(x) || sqp_misaligned(packed) || sqp_misaligned(scales) || sqp_misaligned(zeros) || sqp_misaligned(y))
        return SQP_ERR_ALIGN;
    return SQP_OK;
}

static bool streaming_path(int M) { return M <= g_decode_max_m && M <= 64; }

extern "C" size_t sqp_w4a16_gemm_workspace_bytes(int M, int N, int K, int group)
{
    if (M <= 0 || sqp_check_quant_shape(N, K, group) != SQP_OK || sqp_too_big(M, K) || sqp_too_big(M, N)) return 0;
    const size_t partial = streaming_path(M) ? sqp_gemm_decode_partial_bytes(M, N, K, group)
                                             : sqp_gemm_prefill_partial_bytes(M, N, K, group);
    return partial ? SQP_WS_TICKET_BYTES + partial : 0;
}

// Shared by every GEMM entry point: argument checks, then the weight-streaming path (small M)
// or the tiled matrix-core path.
int sqp_gemm_entry(int M, int N, int K, int group, const void *x, const uint32_t *packed, const void *scales,
                   const uint8_t *zeros, void *y, int epi, const SqpWorkspace &ws, void *stream)
{
    int rc = check_gemm_args(M, N, K, group, x, packed, scales, zeros, y);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const h16 *xp = (const h16 *)x;
    const h16 *sp = (const h16 *)scales;
    h16 *yp = (h16 *)y;
    if (streaming_path(M)) return sqp_gemm_decode(M, N, K, group, xp, packed, sp, zeros, yp, epi, ws, st);
    return sqp_gemm_prefill(M, N, K, group, xp, packed, sp, zeros, yp, epi, ws, st);
}

extern "C" int sqp_w4a16_gemm(int M, int N, int K, int group, const void *x, const uint32_t *packed,
                              const void *scales, const uint8_t *zeros, void *y, void *stream)
{
    return sqp_gemm_entry(M, N, K, group, x, packed, scales, zeros, y, 0, sqp_caller_workspace(), stream);
}

extern "C" int sqp_w4a16_gemm_silu_mul(int M, int N, int K, int group, const void *x, const uint32_t *packed,
                                       const void *scales, const uint8_t *zeros, void *y, void *stream)
{
    if (N % 16) return SQP_ERR_SHAPE;          // the half-width output keeps 16-byte rows
    // the fused epilogue exists in the matrix-core kernels only
    if (!(group == 32 || group == 64 || group % 128 == 0)) return SQP_ERR_SHAPE;
    return sqp_gemm_entry(M, N, K, group, x, packed, scales, zeros, y, 1, sqp_caller_workspace(), stream);
}

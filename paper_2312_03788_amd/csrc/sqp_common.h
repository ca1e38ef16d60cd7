// Shared host-side helpers of the sqp library (argument checks, launch status).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sqp.h"

typedef _Float16 h16;
typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 h16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

static inline bool sqp_misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Size limit of every entry point: a tensor has fewer than 2^31 elements (the kernels keep
// per-lane offsets in 32 bits).
static inline bool sqp_too_big(long rows, long cols) { return rows * cols >= (1L << 31); }

static inline int sqp_check_quant_shape(int N, int K, int group)
{
    if (N <= 0 || K <= 0 || group < 8) return SQP_ERR_SHAPE;
    if (sqp_too_big(K, N)) return SQP_ERR_SHAPE;
    if ((N % 8) || (K % 8) || (group % 8) || (K % group)) return SQP_ERR_SHAPE;
    return SQP_OK;
}

static inline int sqp_launch_status()
{
    return hipGetLastError() == hipSuccess ? SQP_OK : SQP_ERR_LAUNCH;
}

// Decode (weight-streaming) and prefill (tiled matrix-core) back ends of sqp_w4a16_gemm.
// Arguments are already validated.
// epi: 0 = y [M][N] fp16; 1 = SiLU(gate) * up of interleaved (gate, up) column pairs, y [M][N/2].
int sqp_gemm_decode(int M, int N, int K, int group, const h16 *x, const uint32_t *packed,
                    const h16 *scales, const uint8_t *zeros, h16 *y, int epi, hipStream_t stream);
int sqp_gemm_prefill(int M, int N, int K, int group, const h16 *x, const uint32_t *packed,
                     const h16 *scales, const uint8_t *zeros, h16 *y, int epi, hipStream_t stream);

#ifdef __HIPCC__
// SiLU(g) = g / (1 + exp(-g)) in fp32 (the hardware exponential: about 1 ulp of fp32).
__device__ __forceinline__ float sqp_silu(float g) { return g / (1.0f + __expf(-g)); }
#endif
// Library-owned device buffer for fp32 partial sums (allocated on first use).
int sqp_partial_workspace(float **p, size_t *bytes, hipStream_t stream);

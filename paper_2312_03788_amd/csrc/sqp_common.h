// Shared host-side helpers of the sqp library (argument checks, launch status).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sqp.h"
#include "sqp_test_hooks.h"

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

// The device buffer the GEMM paths may use for fp32 partial sums when they split the inner
// dimension across workgroups: a ticket area (one counter per output tile, zero between
// launches: the last workgroup of a tile to arrive resets it) followed by the partial sums.
// It is never allocated here: it is the caller's buffer (sqp_set_workspace) or the library's
// static device array (sqp_w4a16_gemm_static).  partial == nullptr: none, plans do not split.
constexpr size_t SQP_WS_TICKETS = (size_t)1 << 17;                       // counters
constexpr size_t SQP_WS_TICKET_BYTES = SQP_WS_TICKETS * sizeof(unsigned);  // 512 KB
struct SqpWorkspace {
    unsigned *tickets;
    float *partial;
    size_t partial_bytes;
};
// The workspace the caller has set for the current device (partial == nullptr if none).
SqpWorkspace sqp_caller_workspace();
// Enqueue a kernel that zeroes the ticket area.
int sqp_zero_tickets(unsigned *tickets, hipStream_t stream);

// Decode (weight-streaming) and prefill (tiled matrix-core) back ends of sqp_w4a16_gemm.
// Arguments are already validated.
// epi: 0 = y [M][N] fp16; 1 = SiLU(gate) * up of interleaved (gate, up) column pairs, y [M][N/2].
// A plan that splits K needs ws; without one (partial == nullptr) the non-split plan runs;
// with one that is too small the call fails with SQP_ERR_WORKSPACE and enqueues nothing.
int sqp_gemm_decode(int M, int N, int K, int group, const h16 *x, const uint32_t *packed,
                    const h16 *scales, const uint8_t *zeros, h16 *y, int epi, const SqpWorkspace &ws, hipStream_t stream);
int sqp_gemm_prefill(int M, int N, int K, int group, const h16 *x, const uint32_t *packed,
                     const h16 *scales, const uint8_t *zeros, h16 *y, int epi, const SqpWorkspace &ws, hipStream_t stream);
// Column-slice variant of the decode path (up to 16 rows, groups of 128; needs no workspace).
bool sqp_gemm_slice_covers(int M, int N, int K, int group);
int sqp_gemm_slice(int variant, int M, int N, int K, const h16 *x, const uint32_t *packed, const h16 *scales,
                   const uint8_t *zeros, h16 *y, int epi, hipStream_t stream);
// Shared by every GEMM entry point: argument checks and the choice between the two paths.
int sqp_gemm_entry(int M, int N, int K, int group, const void *x, const uint32_t *packed, const void *scales,
                   const uint8_t *zeros, void *y, int epi, const SqpWorkspace &ws, void *stream);
// Bytes of partial sums the preferred plan of a shape needs (0: it does not split K).
size_t sqp_gemm_decode_partial_bytes(int M, int N, int K, int group);
size_t sqp_gemm_prefill_partial_bytes(int M, int N, int K, int group);

// Eq. 6 in two steps: per-channel maxima amax = [max_t|x_cal[t][j]| (K) | max_n|w[j][n]| (K)],
// then the factor for one alpha.  Arguments are already validated.
int sqp_channel_absmax(int T, int K, int N, const void *x_cal, const void *w, float *amax, hipStream_t stream);
int sqp_smooth_factor(int K, float alpha, const float *amax, float *s, hipStream_t stream);

#ifdef __HIPCC__
// SiLU(g) = g / (1 + exp(-g)) in fp32 (the hardware exponential: about 1 ulp of fp32).
__device__ __forceinline__ float sqp_silu(float g) { return g / (1.0f + __expf(-g)); }
#endif

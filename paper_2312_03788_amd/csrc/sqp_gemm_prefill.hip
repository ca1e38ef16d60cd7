// Tiled matrix-core W4A16 GEMM for large M (prefill).  Placeholder: runs the
// weight-streaming kernel over blocks of 64 rows until the tiled kernel lands.
#include "sqp_common.h"

int sqp_gemm_prefill(int M, int N, int K, int group, const h16 *x, const uint32_t *packed,
                     const h16 *scales, const uint8_t *zeros, h16 *y, hipStream_t stream)
{
    for (int m0 = 0; m0 < M; m0 += 64) {
        int mb = M - m0 < 64 ? M - m0 : 64;
        int rc = sqp_gemm_decode(mb, N, K, group, x + (size_t)m0 * K, packed, scales, zeros, y + (size_t)m0 * N, stream);
        if (rc) return rc;
    }
    return SQP_OK;
}

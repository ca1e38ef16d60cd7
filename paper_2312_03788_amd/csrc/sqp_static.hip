// sqp_w4a16_gemm for callers that cannot allocate device memory or own a workspace (code
// under HIP graph capture, tight serving loops): the same kernels and launch plans as
// sqp_w4a16_gemm, with the tickets and fp32 partial sums of split launches in a static device
// array of this library instead of a caller's buffer.
#include <mutex>

#include "sqp_common.h"

// Tickets (512 KB) followed by partial sums.  Every device the library runs on holds its own
// copy of this array, at its own address, until the process ends.  In host code the name is
// only a handle for hipGetSymbolAddress, never an address to pass on.
static __device__ __align__(256) unsigned char scratch[SQP_WS_TICKET_BYTES + SQP_STATIC_PARTIAL_BYTES];

static std::mutex g_setup_lock;
static unsigned char *g_scratch_ptr[64] = {};  // per device: the array's address there (set-up done)

extern "C" int sqp_w4a16_gemm_static(int M, int N, int K, int group, const void *x, const uint32_t *packed,
                                     const void *scales, const uint8_t *zeros, void *y, void *stream)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SQP_ERR_WORKSPACE;
    unsigned char *ptr;
    {
        std::lock_guard<std::mutex> hold(g_setup_lock);
        ptr = g_scratch_ptr[dev];
        if (ptr == nullptr) {
            // first call on this device (which is current): look the array up and zero its
            // tickets once with a fill kernel on the caller's stream; from then on every split
            // launch leaves them zero again
            void *p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return SQP_ERR_WORKSPACE;
            int rc = sqp_zero_tickets((unsigned *)p, (hipStream_t)stream);
            if (rc) return rc;
            ptr = g_scratch_ptr[dev] = (unsigned char *)p;
        }
    }
    SqpWorkspace ws;
    ws.tickets = (unsigned *)ptr;
    ws.partial = (float *)(ptr + SQP_WS_TICKET_BYTES);
    ws.partial_bytes = SQP_STATIC_PARTIAL_BYTES;
    return sqp_gemm_entry(M, N, K, group, x, packed, scales, zeros, y, 0, ws, stream);
}

// Calls the host-side logic of libsqp that needs no GPU -- launch-plan heuristics, workspace
// size queries and the argument checks of every entry point -- over a grid of shapes.  Built
// with the library's sources and AddressSanitizer / UndefinedBehaviorSanitizer on the host
// side by tests/test_host_sanitizers.py.
#include <cstdint>
#include <cstdio>

#include "sqp.h"
#include "sqp_test_hooks.h"

int main()
{
    long checks = 0, bad = 0;
    const int Ms[] = {1, 7, 16, 17, 32, 33, 64, 65, 130, 256, 2048, 4096, 100000};
    const int Ks[] = {8, 128, 1024, 4096, 8192, 22016, 65536};
    const int Ns[] = {8, 264, 4096, 10240, 44032, 1 << 20};
    const int Gs[] = {8, 24, 32, 64, 128, 256, 1024};
    for (int M : Ms)
        for (int K : Ks)
            for (int N : Ns)
                for (int g : Gs) {
                    if (K % g) continue;
                    int nw = 0, split = 0, kspg = -1, ks = 0;
                    long full = -1, half = -1;
                    sqp_debug_decode_plan(M < 64 ? M : 64, N, K, g, &nw, &split, &kspg);
                    sqp_debug_prefill_plan(M, N, K, 256, &full, &half, &ks);
                    const size_t ws = sqp_w4a16_gemm_workspace_bytes(M, N, K, g);
                    bad += nw < 1 || nw > 8 || split < 1 || kspg < 0 || full < 0 || half < 0 || ks < 1;
                    bad += ws != 0 && ws <= ((size_t)512 << 10);
                    checks++;
                }
    // forced plans go through the same size arithmetic
    sqp_debug_set_decode_plan(8, 64);
    bad += sqp_w4a16_gemm_workspace_bytes(16, 44032, 8192, 128) == 0;
    sqp_debug_set_decode_plan(0, 0);
    sqp_debug_set_prefill_ksplit(16);
    bad += sqp_w4a16_gemm_workspace_bytes(300, 1000, 2048, 128) == 0;
    sqp_debug_set_prefill_ksplit(-1);
    // argument checks return before anything touches a device
    void *good = (void *)0x1000, *odd = (void *)0x1008;
    bad += sqp_w4a16_gemm(4, 1024, 1024, 128, nullptr, (const uint32_t *)good, good, (const uint8_t *)good, good, nullptr) != SQP_ERR_NULL;
    bad += sqp_w4a16_gemm(4, 1020, 1024, 128, good, (const uint32_t *)good, good, (const uint8_t *)good, good, nullptr) != SQP_ERR_SHAPE;
    bad += sqp_w4a16_gemm(4, 1024, 1024, 128, good, (const uint32_t *)odd, good, (const uint8_t *)good, good, nullptr) != SQP_ERR_ALIGN;
    bad += sqp_w4a16_gemm_static(0, 1024, 1024, 128, good, (const uint32_t *)good, good, (const uint8_t *)good, good, nullptr) == SQP_OK;
    bad += sqp_quantize_pack(1024, 1024, 100, good, (uint32_t *)good, good, (uint8_t *)good, nullptr) != SQP_ERR_SHAPE;
    bad += sqp_smooth_scales(8, 1024, 1024, 1.5f, good, good, (float *)good, nullptr) != SQP_ERR_ARG;
    bad += sqp_quant_loss(4, 1024, 1024, 128, good, good, good, (const uint32_t *)good, good, (const uint8_t *)good, (double *)0x1004,
                          (double *)good, nullptr) != SQP_ERR_ALIGN;
    float alphas[2] = {0.5f, 2.0f};
    bad += sqp_alpha_search(8, 1024, 1024, 128, 2, alphas, good, good, (float *)good, (float *)good, good, good, (uint32_t *)good, good,
                            (uint8_t *)good, (double *)good, (double *)good, (int *)good, nullptr) != SQP_ERR_ARG;
    bad += sqp_quant_loss_scratch_doubles(129, 130) != 4;
    for (int code = 0; code >= -7; code--) bad += sqp_status_string(code) == nullptr;
    std::printf("host plan sanitizer run: %ld shapes, %ld inconsistencies\n", checks, bad);
    return bad != 0;
}

// Quantisation loss of one linear layer, Eq. 4 of arXiv 2312.03788:
//   E = || X W - X_hat W_hat ||_F^2,   W_hat = dequantised 4-bit weights (Eq. 1),
// with X_hat = X diag(s)^-1 and the quantised W_hat of diag(s) W (Eq. 5), as the search over the
// smoothing strength alpha needs it (Sec 2.2: alpha is chosen to minimise the loss).
//
// The two products are never formed separately: rounding either of them to fp16 would
// swamp their difference.  One fp32 accumulator per output element takes both, as a single
// contraction over the concatenated inner dimension [X, X_hat] * [W; -W_hat]: per k-step one
// MFMA with the fp16 weights and one with the negated dequantised codes.  A workgroup of 8
// waves owns a 128 x 128 tile (wave tile 64 x 32 = 2 tiles of v_mfma_f32_32x32x16_f16),
// squares and sums its accumulators in fp64 and writes one partial; a second kernel adds the
// partials in a fixed order, so the result does not depend on scheduling.
//   - X and X_hat tiles (128 rows x 64 k) go through LDS as they are (k is contiguous).
//   - W is row-major [K][N], so a column's 8 consecutive k (one lane's B operand) are N apart:
//     the tile is transposed on its way into LDS (8 rows x 2 columns per thread, v_perm_b32).
//   - Packed words are loaded straight into registers (a word is one lane's B operand) and
//     unpacked with the step negated.
// This is an offline calibration kernel: plain loads and barriers; the global loads of the next
// k-step are issued before the current one is multiplied, and the eight waves (two per SIMD)
// cover each other's waits: one wave per SIMD issued an instruction only every ten cycles.
#include "sqp_common.h"
#include "sqp_w4_unpack.h"

namespace {

constexpr int LBM = 128, LBN = 128, LBK = 64, LPAD = 8;  // row stride 144 bytes: 16-byte reads of 32 rows spread over the banks

// FULL: M and N are multiples of the tile and K of the k-step, so no access needs a bounds check.
template <bool FULL>
__global__ void __launch_bounds__(512)
quant_loss_kernel(int M, int N, int K, int group, const h16 *__restrict__ x, const h16 *__restrict__ w,
                  const h16 *__restrict__ xh, const uint32_t *__restrict__ packed, const h16 *__restrict__ scales,
                  const uint8_t *__restrict__ zeros, double *__restrict__ partials)
{
    __shared__ __attribute__((aligned(16))) h16 sx[LBM][LBK + LPAD];
    __shared__ __attribute__((aligned(16))) h16 sxh[LBM][LBK + LPAD];
    __shared__ __attribute__((aligned(16))) h16 sw[LBN][LBK + LPAD];  // transposed: [column][k]
    __shared__ double red[8];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;                   // wave tile: rows wm*64 .. +64, columns wn*32 .. +32
    const int l32 = lane & 31, kb = lane >> 5;
    const int m0 = blockIdx.y * LBM, n0 = blockIdx.x * LBN;
    const UnpackConsts uc = SQP_UNPACK_CONSTS;

    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[i][r] = 0.f;

    // loader roles
    const int arow = tid >> 2, apart = tid & 3;               // X, X_hat: row, 16-half part of the 64 k
    int agrow = m0 + arow;
    if (!FULL && agrow >= M) agrow = M - 1;                    // rows past M: duplicates, masked at the end
    const int wkb = tid >> 6, wcp = tid & 63;                  // W: k-block of 8 rows, column pair
    const int wcol = n0 + 2 * wcp;
    const int qcol = n0 + wn * 32 + l32;                       // packed words: this lane's column
    const bool wcol_ok = FULL || wcol < N, qcol_ok = FULL || qcol < N;
    // per-thread pointers at this thread's piece of k-step 0, advanced by one step per iteration
    const h16 *px = x + (size_t)agrow * K + apart * 16;
    const h16 *ph = xh + (size_t)agrow * K + apart * 16;
    const h16 *pw = w + (size_t)(wkb * 8) * N + (wcol_ok ? wcol : 0);
    const uint32_t *pq = packed + (size_t)kb * N + (qcol_ok ? qcol : 0);
    const bool one_group = group % LBK == 0;                   // a k-step lies within one quantisation group

    // Software pipeline over the k-steps: the global loads of step k0 + LBK are in flight (into
    // registers) while step k0 is multiplied out of LDS; two waves per SIMD cover each other's waits.
    uint4 rx[2], rh[2];     // X and X_hat: this thread's 2 x 8 halves of its row
    uint32_t rw[8];         // W: 8 rows x one column pair
    uint32_t rword[4], rz[4], rd[4];  // packed word, zero point, negated step per k sub-step
    auto fetch = [&](int k0) {
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const bool ok = FULL || k0 + apart * 16 + j * 8 < K;
            rx[j] = ok ? *reinterpret_cast<const uint4 *>(px + j * 8) : make_uint4(0, 0, 0, 0);
            rh[j] = ok ? *reinterpret_cast<const uint4 *>(ph + j * 8) : make_uint4(0, 0, 0, 0);
        }
        const bool wok = FULL || (wcol_ok && k0 + wkb * 8 < K);          // K is a multiple of 8: a block of 8 rows is in or out as a whole
#pragma unroll
        for (int i = 0; i < 8; i++) rw[i] = wok ? *reinterpret_cast<const uint32_t *>(pw + (size_t)i * N) : 0u;
        const int gstep = k0 / group;
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            const int kk = k0 + ks * 16 + kb * 8;
            rword[ks] = 0; rz[ks] = 0; rd[ks] = 0;
            if (FULL || (qcol_ok && kk < K)) {
                const size_t gi = (size_t)(one_group ? gstep : kk / group) * N + qcol;
                rword[ks] = pq[(size_t)(ks * 2) * N];
                rz[ks] = zeros[gi];
                rd[ks] = __builtin_bit_cast(uint16_t, scales[gi]) ^ 0x8000u;  // -Delta
            }
        }
        px += LBK; ph += LBK; pw += (size_t)LBK * N; pq += (size_t)(LBK / 8) * N;
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += LBK) {
        // ---- registers -> LDS
#pragma unroll
        for (int j = 0; j < 2; j++) {
            *reinterpret_cast<uint4 *>(&sx[arow][apart * 16 + j * 8]) = rx[j];
            *reinterpret_cast<uint4 *>(&sxh[arow][apart * 16 + j * 8]) = rh[j];
        }
        {
            uint4 c0, c1;  // column wcol: the low halves of the 8 rows; column wcol + 1: the high halves
            c0.x = __builtin_amdgcn_perm(rw[1], rw[0], 0x05040100u); c1.x = __builtin_amdgcn_perm(rw[1], rw[0], 0x07060302u);
            c0.y = __builtin_amdgcn_perm(rw[3], rw[2], 0x05040100u); c1.y = __builtin_amdgcn_perm(rw[3], rw[2], 0x07060302u);
            c0.z = __builtin_amdgcn_perm(rw[5], rw[4], 0x05040100u); c1.z = __builtin_amdgcn_perm(rw[5], rw[4], 0x07060302u);
            c0.w = __builtin_amdgcn_perm(rw[7], rw[6], 0x05040100u); c1.w = __builtin_amdgcn_perm(rw[7], rw[6], 0x07060302u);
            *reinterpret_cast<uint4 *>(&sw[2 * wcp][wkb * 8]) = c0;
            *reinterpret_cast<uint4 *>(&sw[2 * wcp + 1][wkb * 8]) = c1;
        }
        // ---- packed words of this wave's 32 columns: registers only
        h16x8 bq[4];
#pragma unroll
        for (int ks = 0; ks < 4; ks++)
            bq[ks] = dequant_word_scaled(rword[ks], neg_hi_of(rz[ks]), neg_lo_of(rz[ks]),
                                         __builtin_bit_cast(h16x2, rd[ks] * 0x00010001u), uc);
        __syncthreads();
        if (k0 + LBK < K) fetch(k0 + LBK);
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            h16x8 ax[2], ah[2];
#pragma unroll
            for (int mt = 0; mt < 2; mt++) {
                const int row = wm * 64 + mt * 32 + l32;
                ax[mt] = *reinterpret_cast<const h16x8 *>(&sx[row][ks * 16 + kb * 8]);
                ah[mt] = permute_x(*reinterpret_cast<const u32x4 *>(&sxh[row][ks * 16 + kb * 8]));
            }
            const h16x8 bw = *reinterpret_cast<const h16x8 *>(&sw[wn * 32 + l32][ks * 16 + kb * 8]);
#pragma unroll
            for (int mt = 0; mt < 2; mt++) {
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ax[mt], bw, acc[mt], 0, 0, 0);
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[mt], bq[ks], acc[mt], 0, 0, 0);
            }
        }
        __syncthreads();
    }

    // ---- sum of squares of the tile.  Accumulator register r of tile mt: row
    // 8*(r/4) + 4*(lane/32) + r%4 of the 32-row tile, column lane%32.
    double ss = 0.0;
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int row = m0 + wm * 64 + mt * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
            if (FULL || (row < M && qcol_ok)) ss += (double)acc[mt][r] * (double)acc[mt][r];
        }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    if (tid == 0)
        partials[(size_t)blockIdx.y * gridDim.x + blockIdx.x] = ((red[0] + red[1]) + (red[2] + red[3])) + ((red[4] + red[5]) + (red[6] + red[7]));
}

// Adds n partials in a fixed order: thread t takes t, t + 256, ..., then a tree over the block.
__global__ void __launch_bounds__(256) sum_partials_kernel(const double *__restrict__ partials, long n, double *__restrict__ out)
{
    __shared__ double s[256];
    double a = 0.0;
    for (long i = threadIdx.x; i < n; i += 256) a += partials[i];
    s[threadIdx.x] = a;
    __syncthreads();
    for (int half = 128; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) s[threadIdx.x] += s[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = s[0];
}

// Index of the smallest of n values, the lowest index on ties (n is a grid of alphas: tiny).
__global__ void argmin_kernel(const double *__restrict__ v, int n, int *__restrict__ best)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    int b = 0;
    for (int i = 1; i < n; i++)
        if (v[i] < v[b]) b = i;
    *best = b;
}

}  // namespace

extern "C" long sqp_quant_loss_scratch_doubles(int M, int N)
{
    if (M <= 0 || N <= 0) return 0;
    return (long)((M + LBM - 1) / LBM) * (long)((N + LBN - 1) / LBN);
}

extern "C" int sqp_quant_loss(int M, int N, int K, int group, const void *x, const void *w, const void *x_hat,
                              const uint32_t *packed, const void *scales, const uint8_t *zeros, double *scratch,
                              double *loss, void *stream)
{
    if (!x || !w || !x_hat || !packed || !scales || !zeros || !scratch || !loss) return SQP_ERR_NULL;
    if (M <= 0) return SQP_ERR_SHAPE;
    int rc = sqp_check_quant_shape(N, K, group);
    if (rc) return rc;
    if (sqp_too_big(M, K) || sqp_too_big(M, N)) return SQP_ERR_SHAPE;
    if (sqp_misaligned(x) || sqp_misaligned(w) || sqp_misaligned(x_hat) || sqp_misaligned(packed) ||
        sqp_misaligned(scales) || sqp_misaligned(zeros))
        return SQP_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(scratch) & 7u) || (reinterpret_cast<uintptr_t>(loss) & 7u)) return SQP_ERR_ALIGN;
    const int gy = (M + LBM - 1) / LBM, gx = (N + LBN - 1) / LBN;
    if (gy > 65535) return SQP_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    if (M % LBM == 0 && N % LBN == 0 && K % LBK == 0)
        quant_loss_kernel<true><<<dim3(gx, gy), 512, 0, st>>>(M, N, K, group, (const h16 *)x, (const h16 *)w, (const h16 *)x_hat,
                                                             packed, (const h16 *)scales, zeros, scratch);
    else
        quant_loss_kernel<false><<<dim3(gx, gy), 512, 0, st>>>(M, N, K, group, (const h16 *)x, (const h16 *)w, (const h16 *)x_hat,
                                                              packed, (const h16 *)scales, zeros, scratch);
    sum_partials_kernel<<<1, 256, 0, st>>>(scratch, (long)gx * gy, loss);
    return sqp_launch_status();
}

extern "C" int sqp_alpha_search(int T, int N, int K, int group, int n_alpha, const float *alphas, const void *x_cal,
                                const void *w, float *amax, float *s, void *x_hat, void *w_s, uint32_t *packed,
                                void *scales, uint8_t *zeros, double *scratch, double *loss, int *best, void *stream)
{
    if (!alphas || !x_cal || !w || !amax || !s || !x_hat || !w_s || !packed || !scales || !zeros || !scratch || !loss || !best)
        return SQP_ERR_NULL;
    if (T <= 0 || n_alpha <= 0 || n_alpha > 4096) return SQP_ERR_SHAPE;
    int rc = sqp_check_quant_shape(N, K, group);
    if (rc) return rc;
    if (sqp_too_big(T, K) || sqp_too_big(T, N)) return SQP_ERR_SHAPE;
    if ((T + LBM - 1) / LBM > 65535 || K / group > 65535) return SQP_ERR_SHAPE;
    for (int i = 0; i < n_alpha; i++)
        if (!(alphas[i] >= 0.0f && alphas[i] <= 1.0f)) return SQP_ERR_ARG;
    if (sqp_misaligned(x_cal) || sqp_misaligned(w) || sqp_misaligned(amax) || sqp_misaligned(s) || sqp_misaligned(x_hat) ||
        sqp_misaligned(w_s) || sqp_misaligned(packed) || sqp_misaligned(scales) || sqp_misaligned(zeros))
        return SQP_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(scratch) & 7u) || (reinterpret_cast<uintptr_t>(loss) & 7u) ||
        (reinterpret_cast<uintptr_t>(best) & 3u))
        return SQP_ERR_ALIGN;
    // every check any step below would make has passed: from here on only launch errors can occur
    hipStream_t st = (hipStream_t)stream;
    rc = sqp_channel_absmax(T, K, N, x_cal, w, amax, st);
    for (int i = 0; i < n_alpha && rc == SQP_OK; i++) {
        rc = sqp_smooth_factor(K, alphas[i], amax, s, st);
        if (rc == SQP_OK) rc = sqp_smooth_apply_x(T, K, x_cal, s, x_hat, stream);
        if (rc == SQP_OK) rc = sqp_smooth_apply_w(K, N, w, s, w_s, stream);
        if (rc == SQP_OK) rc = sqp_quantize_pack(N, K, group, w_s, packed, scales, zeros, stream);
        if (rc == SQP_OK) rc = sqp_quant_loss(T, N, K, group, x_cal, w, x_hat, packed, scales, zeros, scratch, loss + i, stream);
    }
    if (rc != SQP_OK) return rc;
    argmin_kernel<<<1, 64, 0, st>>>(loss, n_alpha, best);
    return sqp_launch_status();
}

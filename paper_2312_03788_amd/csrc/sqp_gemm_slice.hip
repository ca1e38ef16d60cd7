// Weight-streaming W4A16 GEMM for a few rows (decode with a small batch): y = x * w_hat, Eq. 3 of
// arXiv 2312.03788 with w_hat = (code - Z) * Delta of Eq. 1, groups of 128 along K (Sec 2.2).
//
// The strip kernel splits K across workgroups to fill the chip, and the hand-over of partial
// sums between workgroups (through memory, with a ticket) costs a fixed few microseconds per
// launch - as much as streaming the whole layer on the narrowest ones.  Here a workgroup owns a
// slice of 16 TB output columns (32 or 64) over ALL of K and K is split between its waves
// instead: wave w takes the chunks (128 k each) w, w + WV, w + 2 WV, ...; the waves never meet
// in the main loop (each fetches the activations of its own chunks into a ring of LDS slots of
// its own, so there is no barrier) and add their fp32 sums through LDS at the end, in wave
// order: no workspace, no tickets, and the result does not depend on scheduling.
// The price: every workgroup fetches all of x (from L2), workgroups x rows x K x 2 bytes per
// launch, which at 16 rows costs as much as the hand-over saved; the kernel is used up to 8 or
// 12 rows, where only the blocks of four rows that hold real rows are fetched.
//
// Column mapping: lane (lc = lane % 16, lk = lane / 16) holds the TB adjacent columns
// n0 + TB lc ... (one 8- or 16-byte load per k-step: their packed words, k-block lk), which are
// the B operands of TB v_mfma_f32_16x16x32_f16 (column block b = every TB-th column of the
// slice, starting at b); their steps Delta are one load, their zero points another.  With the
// fused SiLU(gate)*up output a lane's columns are whole (gate, up) pairs.
#include <type_traits>

#include "sqp_common.h"
#include "sqp_w4_unpack.h"

namespace {

// WV: waves per workgroup.  D: stages (registers for the weight side, LDS slots for the
// activations) per wave; D - 1 chunks are in flight per wave while one is consumed.
// XB: blocks of four activation rows that are fetched (M <= 4 XB); the other rows of the
// 16-row matrix operand are whatever the LDS holds, and only feed output rows that are never stored.
template <int TB, int WV, int D, int XB>
__global__ void __launch_bounds__(WV * 64)
w4a16_decode_slice_kernel(int M, int N, int K, const h16 *__restrict__ x, const uint32_t *__restrict__ packed,
                          const h16 *__restrict__ scales, const uint8_t *__restrict__ zeros, h16 *__restrict__ y, int epi)
{
    constexpr int P = D - 1;
    constexpr int XSTAGE = XB * 1024;  // one chunk of x: 4 XB rows of 256 bytes, as 1 KB blocks of four rows
    constexpr int LOADS = XB + 4 + 2;  // per chunk and wave: activations, weights, steps and zero points
    static_assert((P - 1) * LOADS < 64, "vmcnt field");
    static_assert(TB == 2 || TB == 4, "column blocks of 16 per workgroup");
    constexpr int RING = WV * D * XSTAGE, EXCH = WV * TB * 1024;  // the exchange of sums at the end reuses the rings
    __shared__ __attribute__((aligned(1024))) unsigned char xring[RING > EXCH ? RING : EXCH];

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lc = lane & 15, lk = lane >> 4;
    const int n0 = blockIdx.x * (16 * TB);
    const int chunks = K / 128;
    // lanes past the last column read column 0 instead; their results are never stored
    const int nout = n0 + TB * lc;
    const int ncol = nout < N ? nout : 0;
    // this wave's chunks: wv, wv + WV, ...  (none when the layer has fewer chunks than waves)
    const int nmine = wv < chunks ? (chunks - wv + WV - 1) / WV : 0;
    const int c0 = wv < chunks ? wv : 0;

    f32x4 acc[TB];
#pragma unroll
    for (int b = 0; b < TB; b++) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    const UnpackConsts uc = SQP_UNPACK_CONSTS;

    typedef uint32_t wvec __attribute__((ext_vector_type(TB)));       // the packed words of the lane's TB columns
    typedef typename std::conditional<TB == 2, uint32_t, u32x2>::type svec;  // their TB fp16 steps
    struct Stage {
        wvec w[4];    // per k-step
        svec sc;
        uint32_t zr;  // TB zero points, one byte each
    };

    // Addresses: a wave-uniform byte pointer per stream (stepped on the scalar unit) plus a
    // per-lane 32-bit offset that never changes.
    const uint32_t voff_w = (uint32_t)(lk * N + ncol) * 4u;
    const uint32_t voff_s = (uint32_t)ncol * 2u, voff_z = (uint32_t)ncol;
    const long wstep1 = (long)N * 16;  // one k-step: four packed rows, in bytes
    const unsigned char *wq = reinterpret_cast<const unsigned char *>(packed) + (long)c0 * 4 * wstep1;
    const unsigned char *sq = reinterpret_cast<const unsigned char *>(scales) + (long)c0 * N * 2;
    const unsigned char *zq = zeros + (long)c0 * N;
    const unsigned char *xq = reinterpret_cast<const unsigned char *>(x) + (long)c0 * 256;
    int issued = 0;  // issue calls so far; the pointers are at own chunk min(issued, nmine - 1)

    // Weight-side loads, in assembly so that this kernel decides when to wait for them (a stage
    // must not be read before `landed`).  They carry the non-temporal hint (every weight byte
    // is read once per launch).  `live` (wave-uniform) is false for the look-ahead past the
    // wave's last chunk: those loads are issued under an empty execution mask, fetch nothing and
    // write no register, but keep their place in the in-order load queue, so the wait counts
    // are the same in every iteration.  Mask change, loads and restore are one statement.
    auto issue_w = [&](Stage &s, bool live) {
        const unsigned char *b0 = wq, *b1 = wq + wstep1, *b2 = wq + 2 * wstep1, *b3 = wq + 3 * wstep1;
        const uint32_t m = __builtin_amdgcn_readfirstlane(live ? 0xffffffffu : 0u);
        uint64_t saved;
        if constexpr (TB == 2) {
            asm volatile("s_mov_b64 %[sv], exec\n\t"
                         "s_and_b32 exec_lo, exec_lo, %[m]\n\t"
                         "s_and_b32 exec_hi, exec_hi, %[m]\n\t"
                         "global_load_dwordx2 %[w0], %[vw], %[b0] nt\n\t"
                         "global_load_dwordx2 %[w1], %[vw], %[b1] nt\n\t"
                         "global_load_dwordx2 %[w2], %[vw], %[b2] nt\n\t"
                         "global_load_dwordx2 %[w3], %[vw], %[b3] nt\n\t"
                         "global_load_dword %[sc], %[vs], %[sq] nt\n\t"
                         "global_load_ushort %[zr], %[vz], %[zq] nt\n\t"
                         "s_mov_b64 exec, %[sv]"
                         : [w0] "=&v"(s.w[0]), [w1] "=&v"(s.w[1]), [w2] "=&v"(s.w[2]), [w3] "=&v"(s.w[3]), [sc] "=&v"(s.sc),
                           [zr] "=&v"(s.zr), [sv] "=&s"(saved)
                         : [m] "s"(m), [vw] "v"(voff_w), [vs] "v"(voff_s), [vz] "v"(voff_z), [b0] "s"(b0), [b1] "s"(b1),
                           [b2] "s"(b2), [b3] "s"(b3), [sq] "s"(sq), [zq] "s"(zq)
                         : "memory", "scc");  // s_and_b32 writes SCC
        } else {
            asm volatile("s_mov_b64 %[sv], exec\n\t"
                         "s_and_b32 exec_lo, exec_lo, %[m]\n\t"
                         "s_and_b32 exec_hi, exec_hi, %[m]\n\t"
                         "global_load_dwordx4 %[w0], %[vw], %[b0] nt\n\t"
                         "global_load_dwordx4 %[w1], %[vw], %[b1] nt\n\t"
                         "global_load_dwordx4 %[w2], %[vw], %[b2] nt\n\t"
                         "global_load_dwordx4 %[w3], %[vw], %[b3] nt\n\t"
                         "global_load_dwordx2 %[sc], %[vs], %[sq] nt\n\t"
                         "global_load_dword %[zr], %[vz], %[zq] nt\n\t"
                         "s_mov_b64 exec, %[sv]"
                         : [w0] "=&v"(s.w[0]), [w1] "=&v"(s.w[1]), [w2] "=&v"(s.w[2]), [w3] "=&v"(s.w[3]), [sc] "=&v"(s.sc),
                           [zr] "=&v"(s.zr), [sv] "=&s"(saved)
                         : [m] "s"(m), [vw] "v"(voff_w), [vs] "v"(voff_s), [vz] "v"(voff_z), [b0] "s"(b0), [b1] "s"(b1),
                           [b2] "s"(b2), [b3] "s"(b3), [sq] "s"(sq), [zq] "s"(zq)
                         : "memory", "scc");  // s_and_b32 writes SCC
        }
    };
    auto landed = [&](Stage &s) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((P - 1) * LOADS) : "memory");
#pragma unroll
        for (int ks = 0; ks < 4; ks++) asm volatile("" : "+v"(s.w[ks]));
        asm volatile("" : "+v"(s.sc));
        asm volatile("" : "+v"(s.zr));
    };

    // Activations of a chunk: XB direct global->LDS loads of 1 KB (four rows of 256 bytes
    // each).  Lane i of a block handles row i / 16 of the block and fetches piece
    // (i % 16) ^ (row % 16) of that row, so that a row's pieces (whole 128-byte lines) come from
    // adjacent lanes, while in LDS (where the hardware puts lane i at byte 16 i of the block)
    // the pieces the 16 rows need for one k-step fall into 16 different bank groups.  Rows past
    // M re-read row M - 1.  Past the wave's last chunk the loads re-read that chunk (cache hits).
    unsigned char *const ring = xring + wv * (D * XSTAGE);
    uint32_t xoff[XB];
#pragma unroll
    for (int j = 0; j < XB; j++) {
        const int row = j * 4 + (lane >> 4);
        const int rowc = row < M ? row : M - 1;
        xoff[j] = (uint32_t)rowc * (uint32_t)K * 2u + (uint32_t)(((lane & 15) ^ row) * 16);
    }
    auto issue_x = [&](int slot) {
#pragma unroll
        for (int j = 0; j < XB; j++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(xq + xoff[j]),
                                             (__attribute__((address_space(3))) void *)(ring + slot * XSTAGE + j * 1024), 16, 0, 0);
    };
    // LDS byte address of this lane's A fragment (row lc) in slot 0, piece 0
    // (rows that are not fetched take the fragment of a fetched row instead: defined data, unused results)
    const int lr = lc % (4 * XB);
    const uint32_t xrd = (uint32_t)(size_t)ring + (uint32_t)((lr >> 2) * 1024 + (lr & 3) * 256);

    auto advance = [&]() {
        issued++;
        const bool more = issued < nmine;
        wq += more ? (long)WV * 4 * wstep1 : 0;
        sq += more ? (long)WV * N * 2 : 0;
        zq += more ? (long)WV * N : 0;
        xq += more ? WV * 256 : 0;
    };

    auto compute = [&](const Stage &s, int slot) {
        h16x2 neg_hi[TB], neg_lo[TB];
        float delta[TB];
#pragma unroll
        for (int b = 0; b < TB; b++) {
            const uint32_t z = (s.zr >> (8 * b)) & 0xffu;
            neg_hi[b] = neg_hi_of(z);
            neg_lo[b] = neg_lo_of(z);
            uint32_t pair;
            if constexpr (TB == 2) pair = s.sc;
            else pair = s.sc[b >> 1];
            const h16x2 sv = __builtin_bit_cast(h16x2, pair);
            delta[b] = (float)((b & 1) ? sv.y : sv.x);
        }
        // The A fragments are read with instructions written in assembly: the compiler cannot
        // tell which ring slot a direct load filled and would wait for every outstanding load.
        u32x4 xa[4];
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            const uint32_t a = xrd + (uint32_t)(slot * XSTAGE) + (uint32_t)(((ks * 4 + lk) ^ lr) * 16);
            asm volatile("ds_read_b128 %0, %1" : "=&v"(xa[ks]) : "v"(a) : "memory");
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int ks = 0; ks < 4; ks++) asm volatile("" : "+v"(xa[ks]));  // no use ahead of the wait
        f32x4 accg[TB];
#pragma unroll
        for (int b = 0; b < TB; b++) accg[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            const h16x8 a = permute_x(xa[ks]);
#pragma unroll
            for (int b = 0; b < TB; b++) {
                const h16x8 bw = dequant_word(s.w[ks][b], neg_hi[b], neg_lo[b], uc);
                accg[b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bw, accg[b], 0, 0, 0);
            }
        }
#pragma unroll
        for (int b = 0; b < TB; b++)
#pragma unroll
            for (int r = 0; r < 4; r++) acc[b][r] = fmaf(delta[b], accg[b][r], acc[b][r]);
    };

    // Software pipeline over the wave's own chunks, P ahead; the chunk count is padded to a
    // multiple of D (stage and slot indices are static), padded iterations only keep the load
    // counts in step.  Slot (i + P) % D, filled in iteration i, was consumed in iteration i - 1
    // by this same wave (its LDS reads have been waited for), so no barrier is needed.
    Stage st[D];
#pragma unroll
    for (int j = 0; j < P; j++) {
        issue_x(j);
        issue_w(st[j], j < nmine);
        advance();
    }
    const int nblk = (nmine + D - 1) / D;
    for (int blk = 0; blk < nblk; blk++) {
#pragma unroll
        for (int d = 0; d < D; d++) {
            const int i = blk * D + d;
            landed(st[d]);
            issue_x((d + P) % D);
            issue_w(st[(d + P) % D], i + P < nmine);
            advance();
            if (i < nmine) compute(st[d], d);
        }
    }
    // Look-ahead loads may still be in flight: wait for them with every stage still allocated,
    // so that nothing else lives in those registers (or is read from LDS) while they land.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int j = 0; j < D; j++) {
#pragma unroll
        for (int ks = 0; ks < 4; ks++) asm volatile("" ::"v"(st[j].w[ks]));
        asm volatile("" ::"v"(st[j].sc));
        asm volatile("" ::"v"(st[j].zr));
    }

    // ---- the waves add their sums through LDS (the rings are idle once every wave is here), in
    // wave order.  Accumulator block b, register r of a lane: row 4 lk + r, column n0 + TB lc + b.
    __syncthreads();
    f32x4 *ex = reinterpret_cast<f32x4 *>(xring);
#pragma unroll
    for (int b = 0; b < TB; b++) ex[(wv * TB + b) * 64 + lane] = acc[b];
    __syncthreads();
    if (wv != 0 || nout >= N) return;
    f32x4 sum[TB];
#pragma unroll
    for (int b = 0; b < TB; b++) sum[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < WV; w++)
#pragma unroll
        for (int b = 0; b < TB; b++) sum[b] += ex[(w * TB + b) * 64 + lane];
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const int m = 4 * lk + r;
        if (m >= M) continue;
        // epi == 0: the fp16 values themselves, y [M][N].  epi == 1: the lane's columns are
        // (gate, up) pairs of a merged, interleaved gate/up projection and the output is
        // SiLU(gate) * up, y [M][N/2] (the LlamaMLP activation of Fig. 5, from the fp32 sums).
        if constexpr (TB == 2) {
            if (epi == 0) {
                h16x2 o;
                o.x = (h16)sum[0][r];
                o.y = (h16)sum[1][r];
                *reinterpret_cast<h16x2 *>(y + (size_t)m * N + nout) = o;
            } else {
                y[(size_t)m * (N >> 1) + (nout >> 1)] = (h16)(sqp_silu(sum[0][r]) * sum[1][r]);
            }
        } else {
            if (epi == 0) {
                h16x4 o;
                o.x = (h16)sum[0][r]; o.y = (h16)sum[1][r]; o.z = (h16)sum[2][r]; o.w = (h16)sum[3][r];
                *reinterpret_cast<h16x4 *>(y + (size_t)m * N + nout) = o;
            } else {
                h16x2 o;
                o.x = (h16)(sqp_silu(sum[0][r]) * sum[1][r]);
                o.y = (h16)(sqp_silu(sum[2][r]) * sum[3][r]);
                *reinterpret_cast<h16x2 *>(y + (size_t)m * (N >> 1) + (nout >> 1)) = o;
            }
        }
    }
}

}  // namespace

// Whether the column-slice kernel covers a call (the caller decides whether it is the better plan).
bool sqp_gemm_slice_covers(int M, int N, int K, int group)
{
    return M >= 1 && M <= 16 && group == 128 && K % 128 == 0 && N % 8 == 0;
}

// variant: 0 = 32-column slices, 1 = 64-column slices.
int sqp_gemm_slice(int variant, int M, int N, int K, const h16 *x, const uint32_t *packed, const h16 *scales,
                   const uint8_t *zeros, h16 *y, int epi, hipStream_t stream)
{
#define SQP_SLICE_LAUNCH(TB, XB) \
    w4a16_decode_slice_kernel<TB, 8, 2, XB><<<(N + 16 * TB - 1) / (16 * TB), 8 * 64, 0, stream>>>(M, N, K, x, packed, scales, zeros, y, epi)
    const int xb = (M + 3) / 4;  // blocks of four rows that hold real rows
    if (variant == 0) {
        if (xb == 1) SQP_SLICE_LAUNCH(2, 1);
        else if (xb == 2) SQP_SLICE_LAUNCH(2, 2);
        else if (xb == 3) SQP_SLICE_LAUNCH(2, 3);
        else SQP_SLICE_LAUNCH(2, 4);
    } else {
        if (xb == 1) SQP_SLICE_LAUNCH(4, 1);
        else if (xb == 2) SQP_SLICE_LAUNCH(4, 2);
        else if (xb == 3) SQP_SLICE_LAUNCH(4, 3);
        else SQP_SLICE_LAUNCH(4, 4);
    }
#undef SQP_SLICE_LAUNCH
    return sqp_launch_status();
}

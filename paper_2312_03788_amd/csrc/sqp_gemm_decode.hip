// Weight-streaming W4A16 GEMM for small M (decode): y = x * w_hat, Eq. 3 of
// arXiv 2312.03788 with w_hat = (code - Z) * Delta of Eq. 1, group-wise along K (Sec 2.2).
//
// The kernel is bound by the HBM stream of packed weights, and on this chip that stream is
// limited by how many cache-line requests a compute unit's vector L1 keeps in flight: the
// L1 handles requests in order, so every request that is not a weight line (activations,
// steps, zero points) takes a place a weight line could have had.  The design follows:
//   - A workgroup of NW waves covers 64*NW output columns; each wave owns a 64-column strip
//     and every wave walks the same range of K.  One dwordx4 load per lane fetches, for
//     k-block (lane / 16), the packed words of 4 adjacent columns: a word is 8 consecutive k
//     of one column, which is exactly one lane's B operand of v_mfma_f32_16x16x32_f16
//     (column = lane % 16, k-block = lane / 16).
//   - The activations of a K chunk are fetched ONCE per workgroup, as whole 128-byte lines,
//     by direct global->LDS loads into a ring of D slots, and every wave takes its A operands
//     from there (row = lane % 16, permuted to the nibble order of the unpack).
//   - The codes become exact fp16 integers (code - Z) with 9 VALU ops per word: the nibbles
//     are OR-ed into the mantissa of 1024.0 (bits 3:0) or 64.0 (bits 7:4) and the offset
//     (1024 + Z or 64 + Z) is subtracted with a packed fp16 add, which is exact.
//   - The MFMA accumulates one chunk in fp32, then the step Delta (a per-lane scalar in the
//     16x16 accumulator layout: column = lane % 16) scales it into the running sum:
//     sum_k x (q - Z) Delta = Delta * sum_k x (q - Z).  (The 64-row variant multiplies the
//     unpacked weights by Delta instead, which is less vector work there.)
//   - Weight loads and all waits are written in assembly: D - 1 chunks of weights stay in
//     flight per wave while one is consumed, and the compiler's conservative waits (it cannot
//     tell ring slots apart) would serialise that.
// With SPLIT > 1 workgroups along K, fp32 partial tiles go to a workspace and the workgroup
// that arrives last (atomic ticket) adds them in split order, so the result does not depend
// on scheduling.
#include <type_traits>

#include "sqp_common.h"
#include "sqp_w4_unpack.h"

// Pipeline depth (stages of weights per wave, slots of activations): three, i.e. two chunks in
// flight per wave while one is consumed; the 32-row variant runs best with four (three with two
// chunks per iteration, whose activation slots are twice as large).  (With the
// streaming hint, masked look-ahead loads and up to eight waves per workgroup three beats four by
// 1-10 % on most shapes; deeper pipelines were slower.)  SQP_DECODE_DEPTH overrides it for experiments.
#ifdef SQP_DECODE_DEPTH
#define SQP_DEPTH_OF(MT, KP) SQP_DECODE_DEPTH
#else
#define SQP_DEPTH_OF(MT, KP) ((MT) == 2 && (KP) == 1 ? 4 : 3)
#endif

namespace {

struct Workspace {
    float *partial;      // [tiles][SPLIT][NW][REGS][64]
    unsigned *tickets;   // [tiles], zero between launches
};

// Final store of 4 adjacent columns n .. n+3 of row m.  epi == 0: the fp16 values themselves,
// y [M][N].  epi == 1: the columns are (gate j, up j, gate j+1, up j+1) of a merged,
// interleaved gate/up projection and the output is SiLU(gate) * up, y [M][N/2] (the LlamaMLP
// activation of Fig. 5, formed from the fp32 sums before any rounding).
__device__ __forceinline__ void store_row4(h16 *y, int m, int N, int n, int epi, float a0, float a1, float a2, float a3)
{
    if (epi == 0) {
        h16x4 o;
        o.x = (h16)a0; o.y = (h16)a1; o.z = (h16)a2; o.w = (h16)a3;
        *reinterpret_cast<h16x4 *>(y + (size_t)m * N + n) = o;
    } else {
        h16x2 o;
        o.x = (h16)(sqp_silu(a0) * a1);
        o.y = (h16)(sqp_silu(a2) * a3);
        *reinterpret_cast<h16x2 *>(y + (size_t)m * (N >> 1) + (n >> 1)) = o;
    }
}

// Split-K tickets: one per 128-byte line (atomics on one line are served one after the other).
constexpr int TICKET_STRIDE = 32;

// MT: 16-row tiles of x (M <= 16*MT).  NW: 64-column strips per workgroup.
// KSPG: k-steps (of 32) per chunk; a quantisation group is cpg chunks (cpg = 1 unless the
// group is a multiple of 128 above 128).
// KW: waves per strip and chunk.  With KW = 2 a strip's two waves share every chunk, each taking
// half of its k-steps, and add their sums through LDS at the end: two waves per SIMD, whose
// instructions the hardware interleaves, where a launch has only one workgroup per compute
// unit and a single wave's dependent vector instructions would leave issue slots empty.
// KP: chunks per iteration.  With KP = 2 the workgroup has twice the waves and takes two
// consecutive chunks per iteration, one per half of its waves (same purpose as KW = 2, without
// making a wave's share of a chunk smaller); the halves add up through LDS like KW's.
template <int MT, int NW, int KSPG, int KW, int KP>
__global__ void __launch_bounds__(NW * KW * KP * 64) __attribute__((amdgpu_waves_per_eu(KW * KP >= 2 ? 2 : (MT == 1 && NW >= 4 ? 3 : 1))))
w4a16_decode_kernel(int M, int N, int K, int cpg, const h16 *__restrict__ x, const uint32_t *__restrict__ packed,
                    const h16 *__restrict__ scales, const uint8_t *__restrict__ zeros, h16 *__restrict__ y,
                    Workspace ws, int epi)
{
    constexpr int D = SQP_DEPTH_OF(MT, KP);  // register stages of packed weights
    constexpr int XD = D;                  // LDS slots of activations
    constexpr int P = D - 1;               // chunks in flight ahead of the one being consumed
    constexpr int REGS = MT * 4 * 4;       // fp32 accumulator registers per lane
    constexpr int BN = 64 * NW;
    // One chunk of x in LDS: MT*16 rows of KSPG*64 bytes, stored as 1 KB blocks, one per
    // direct load instruction: a block holds 16/KSPG rows, PP = 4*KSPG 16-byte pieces each.
    constexpr int PP = 4 * KSPG;
    constexpr int RPB = 16 / KSPG;         // rows per block
    constexpr int CBLOCKS = MT * KSPG;     // blocks per chunk
    constexpr int XBLOCKS = CBLOCKS * KP;  // blocks per iteration (KP consecutive chunks)
    constexpr int XSTAGE = XBLOCKS * 1024;
    constexpr int WAVES = NW * KW * KP;
    constexpr int KS = KSPG / KW;                // k-steps of a chunk this wave takes
    static_assert(KS * KW == KSPG, "k-steps divide among a strip's waves");
    constexpr int OX = (XBLOCKS + WAVES - 1) / WAVES;  // direct loads per wave per chunk (at most)
    // When the blocks do not divide evenly among the waves, waves XREM and above copy one block
    // fewer (none, where a chunk has fewer blocks than the workgroup has waves): every block is
    // fetched exactly once per workgroup, and such a wave waits on a count of its own.
    constexpr int XREM = XBLOCKS % WAVES;
    constexpr int OW = KS + 2;                   // weight-side loads per wave per chunk
    // With four row tiles the per-chunk scaling of 64 accumulator registers costs more vector
    // work than multiplying the unpacked weights by the step (4 packed multiplies per word, as
    // in the tiled kernel), so that variant accumulates fp16(w_hat) products directly.
    constexpr bool SCALED_B = MT == 4;
    static_assert((P - 1) * (OX + OW) < 64, "vmcnt field");
    constexpr int EXCHANGE = (KW * KP - 1) * NW * REGS * 256;  // bytes of the sums a strip's waves exchange at the end
    __shared__ __attribute__((aligned(1024))) unsigned char xring[XD * XSTAGE > EXCHANGE ? XD * XSTAGE : EXCHANGE];
    static_assert(sizeof(xring) + 16 <= 65536, "static LDS of a workgroup");
    __shared__ unsigned ticket_s;

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);    // wave-uniform, kept scalar
    const int wave = wv % NW, kh = (wv / NW) % KW, ph = wv / (NW * KW);   // strip, which k-steps of a chunk, which chunk of an iteration
    const int lc = lane & 15, lk = lane >> 4;
    const int tile = blockIdx.x;
    const int n0 = tile * BN + wave * 64;
    const int split = gridDim.y, sidx = blockIdx.y;
    const int chunks = K / (32 * KSPG);
    // this workgroup's chunk range (all waves walk it together)
    const int g0 = (int)((long)chunks * sidx / split), g1 = (int)((long)chunks * (sidx + 1) / split);

    // lanes past the last column read column 0 instead; their results are never stored
    int ncol = n0 + 4 * lc;
    if (ncol >= N) ncol = 0;

    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int t = 0; t < 4; t++) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    const UnpackConsts uc = SQP_UNPACK_CONSTS;

    struct Stage {
        u32x4 w[KS];
        u32x2 sc;     // 4 fp16 steps
        uint32_t zr;  // 4 zero points, one byte each
    };

    // Weight-side addresses are a scalar base (advanced on the scalar unit) plus a per-lane
    // 32-bit offset that never changes, so the loads cost no vector arithmetic.  The loads are
    // written in assembly so that this kernel, not the compiler, decides when to wait for
    // them: a stage must not be read before `landed` below.  They carry the non-temporal hint:
    // every weight byte is read once per launch, and a plain streaming probe reads 12-15 % faster
    // with it on this chip (the kernel gains about 2 %).
    const uint32_t voff_w = (uint32_t)(lk * N + ncol) * 4u;
    const int wrow_stride = N;
    const uint32_t voff_s = (uint32_t)ncol * 2u, voff_z = (uint32_t)ncol;
    // The loading side walks the chunks with wave-uniform byte pointers stepped by constant
    // strides (scalar adds, no multiplies or divisions in the loop).
    const long wstep1 = (long)wrow_stride * 16;                 // one k-step: 4 packed rows, in bytes
    // An iteration covers KP consecutive chunks; this wave's are g0 + ph, g0 + ph + KP, ...  (with
    // KP = 2 and an odd range the second half of the waves has one chunk fewer; a wave without
    // any chunk points at g0 and never computes).  The activations are fetched per iteration
    // for all KP chunks by all waves together.
    const int nsup = (g1 - g0 + KP - 1) / KP;                    // iterations of this workgroup
    const bool own_any = g0 + ph < g1;
    const int cs = own_any ? g0 + ph : g0;                       // this wave's first chunk
    const int wlast = own_any ? cs + ((g1 - 1 - cs) / KP) * KP : cs;  // and its last
    const unsigned char *wq = reinterpret_cast<const unsigned char *>(packed) + (long)cs * KSPG * wstep1;
    const unsigned char *sq = reinterpret_cast<const unsigned char *>(scales) + (long)(cs / cpg) * N * 2;
    const unsigned char *zq = zeros + (long)(cs / cpg) * N;
    const unsigned char *xq = reinterpret_cast<const unsigned char *>(x) + (long)g0 * (64 * KSPG);
    int gi = cs, kin = cs % cpg;                                 // own chunk being issued, its position in its group
    int xg = g0;                                                 // first chunk of the iteration whose activations are being issued
    // `live` (wave-uniform) is false for the look-ahead loads past the end of the workgroup's range:
    // those are issued with an empty execution mask, so they fetch nothing (with the streaming
    // hint their lines would not be cache hits) and write no register, but still take their
    // place in the in-order load queue, which keeps the wait counts below the same for every
    // iteration.  Mask change, loads and mask restore are one asm statement, so the compiler can
    // place nothing of its own under the changed mask.
    auto issue_w = [&](Stage &s, bool live) {
        const unsigned char *b0 = wq + (kh * KS) * wstep1;  // wave-uniform
        const uint32_t m = __builtin_amdgcn_readfirstlane(live ? 0xffffffffu : 0u);  // both halves of the mask
        uint64_t saved;
        if constexpr (KS == 4) {
            const unsigned char *b1 = b0 + wstep1, *b2 = b0 + 2 * wstep1, *b3 = b0 + 3 * wstep1;
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
        } else if constexpr (KS == 2) {
            const unsigned char *b1 = b0 + wstep1;
            asm volatile("s_mov_b64 %[sv], exec\n\t"
                         "s_and_b32 exec_lo, exec_lo, %[m]\n\t"
                         "s_and_b32 exec_hi, exec_hi, %[m]\n\t"
                         "global_load_dwordx4 %[w0], %[vw], %[b0] nt\n\t"
                         "global_load_dwordx4 %[w1], %[vw], %[b1] nt\n\t"
                         "global_load_dwordx2 %[sc], %[vs], %[sq] nt\n\t"
                         "global_load_dword %[zr], %[vz], %[zq] nt\n\t"
                         "s_mov_b64 exec, %[sv]"
                         : [w0] "=&v"(s.w[0]), [w1] "=&v"(s.w[1]), [sc] "=&v"(s.sc), [zr] "=&v"(s.zr), [sv] "=&s"(saved)
                         : [m] "s"(m), [vw] "v"(voff_w), [vs] "v"(voff_s), [vz] "v"(voff_z), [b0] "s"(b0), [b1] "s"(b1),
                           [sq] "s"(sq), [zq] "s"(zq)
                         : "memory", "scc");  // s_and_b32 writes SCC
        } else {
            static_assert(KS == 1, "k-steps per wave and chunk");
            asm volatile("s_mov_b64 %[sv], exec\n\t"
                         "s_and_b32 exec_lo, exec_lo, %[m]\n\t"
                         "s_and_b32 exec_hi, exec_hi, %[m]\n\t"
                         "global_load_dwordx4 %[w0], %[vw], %[b0] nt\n\t"
                         "global_load_dwordx2 %[sc], %[vs], %[sq] nt\n\t"
                         "global_load_dword %[zr], %[vz], %[zq] nt\n\t"
                         "s_mov_b64 exec, %[sv]"
                         : [w0] "=&v"(s.w[0]), [sc] "=&v"(s.sc), [zr] "=&v"(s.zr), [sv] "=&s"(saved)
                         : [m] "s"(m), [vw] "v"(voff_w), [vs] "v"(voff_s), [vz] "v"(voff_z), [b0] "s"(b0), [sq] "s"(sq), [zq] "s"(zq)
                         : "memory", "scc");  // s_and_b32 writes SCC
        }
    };
    // wait until at most `after` loads are outstanding, then tie the stage's registers to the
    // wait so that no use of them is scheduled ahead of it
    const bool x_full = XREM == 0 || wv < XREM;  // wave-uniform: this wave issues all OX direct loads per chunk
    auto landed = [&](Stage &s) {
        if (x_full) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((P - 1) * (OX + OW)) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"((P - 1) * (OX - 1 + OW)) : "memory");
#pragma unroll
        for (int ks = 0; ks < KS; ks++) asm volatile("" : "+v"(s.w[ks]));
        asm volatile("" : "+v"(s.sc));
        asm volatile("" : "+v"(s.zr));
    };

    // Activations: wave w copies blocks w, w+NW, ... of the chunk straight into LDS.  Lane i
    // of a block handles row i / PP of the block and fetches piece (i % PP) ^ (row % PP) of
    // that row, so that a row's pieces (whole 128-byte lines) come from adjacent lanes, while
    // in LDS (where the hardware puts lane i at byte 16*i of the block) the pieces the 16
    // rows need for one k-step fall into 16 different bank groups.
    const int xrr = lane / PP, xpp = lane % PP;
    uint32_t xoff[OX];  // per-lane byte offset into x of each block this wave copies
#pragma unroll
    for (int i = 0; i < OX; i++) {
        const int b = ((wv + i * WAVES) % XBLOCKS) % CBLOCKS;   // block within its chunk
        const int row = b * RPB + xrr;
        const int rowc = row < M ? row : M - 1;
        xoff[i] = (uint32_t)rowc * (uint32_t)K * 2u + (uint32_t)((xpp ^ (row % PP)) * 16);
    }
    auto issue_x = [&](int slot) {
#pragma unroll
        for (int i = 0; i < OX; i++) {
            if (i + 1 == OX && !x_full) break;
            const int b = (wv + i * WAVES) % XBLOCKS;
            // block b belongs to chunk xg + b / CBLOCKS of the iteration; past the range (the
            // second chunk of an odd range's last iteration) the first chunk is fetched again
            const int sub = b / CBLOCKS;
            const unsigned char *src = xq + (KP > 1 && xg + sub < g1 ? sub * (64 * KSPG) : 0) + xoff[i];
            unsigned char *dst = xring + slot * XSTAGE + b * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
        }
    };
    // LDS byte address of this lane's A fragment (row lc of m-tile mt) in slot 0, piece 0
    uint32_t xrd[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        const int row = mt * 16 + lc;
        xrd[mt] = (uint32_t)(size_t)xring + (uint32_t)(ph * CBLOCKS * 1024 + (row / RPB) * 1024 + (row % RPB) * PP * 16);
    }
    const int xsw = lc % PP;  // the row's swizzle (16 % PP == 0, so mt does not matter)

    auto compute = [&](const Stage &s, int slot) {
        f32x4 accg[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int t = 0; t < 4; t++) accg[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        h16x2 neg_hi[4], neg_lo[4], delta2[4];
        float delta[4];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const uint32_t z = (s.zr >> (8 * c)) & 0xffu;
            neg_hi[c] = neg_hi_of(z);
            neg_lo[c] = neg_lo_of(z);
            const h16x2 sv = __builtin_bit_cast(h16x2, (uint32_t)s.sc[c >> 1]);
            const h16 d16 = (c & 1) ? sv.y : sv.x;
            delta[c] = (float)d16;
            delta2[c] = h16x2{d16, d16};
        }
        // The A fragments come out of the LDS ring with reads written in assembly: the
        // compiler cannot tell which ring slot a direct global->LDS load filled and would wait
        // for every outstanding load; the caller has already waited for this slot.
        auto read_x = [&](u32x4 *dst, int ks) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const uint32_t a = xrd[mt] + (uint32_t)(slot * XSTAGE) + (uint32_t)((((kh * KS + ks) * 4 + lk) ^ xsw) * 16);
                asm volatile("ds_read_b128 %0, %1" : "=&v"(dst[mt]) : "v"(a) : "memory");
            }
        };
        auto wait_x = [&](u32x4 *dst, int n) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < n; i++) asm volatile("" : "+v"(dst[i]));  // no use ahead of the wait
        };
        if constexpr (MT == 1) {
            // one row tile: all of the wave's fragments of the chunk in one batch (other waves of
            // the SIMD, where there are any, cover the wait)
            u32x4 xa[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ks++) read_x(&xa[ks], ks);
            wait_x(xa, KS);
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                const h16x8 a = permute_x(xa[ks]);
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    const h16x8 b = dequant_word(s.w[ks][c], neg_hi[c], neg_lo[c], uc);
                    accg[0][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, accg[0][c], 0, 0, 0);
                }
            }
        } else {
            // several row tiles, one or two waves per SIMD: the fragments of the next k-step are
            // on their way from LDS while this one's MFMAs issue, and the scheduler is told to
            // put the unpack and permute instructions between the MFMAs (they hide behind them)
            // instead of in front of them.
            u32x4 xa[2][MT];
            read_x(xa[0], 0);
            wait_x(xa[0], MT);
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                const int cur = ks & 1, nxt = cur ^ 1;
                if (ks + 1 < KS) read_x(xa[nxt], ks + 1);
                __builtin_amdgcn_sched_barrier(0);
                h16x8 a[MT];
#pragma unroll
                for (int mt = 0; mt < MT; mt++) a[mt] = permute_x(xa[cur][mt]);
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    if constexpr (SCALED_B) {
                        const h16x8 b = dequant_word_scaled(s.w[ks][c], neg_hi[c], neg_lo[c], delta2[c], uc);
#pragma unroll
                        for (int mt = 0; mt < MT; mt++)
                            acc[mt][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], b, acc[mt][c], 0, 0, 0);
                    } else {
                        const h16x8 b = dequant_word(s.w[ks][c], neg_hi[c], neg_lo[c], uc);
#pragma unroll
                        for (int mt = 0; mt < MT; mt++)
                            accg[mt][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], b, accg[mt][c], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int i = 0; i < 4 * MT; i++) {
                    __builtin_amdgcn_sched_group_barrier(0x002, MT == 2 ? 6 : (SCALED_B ? 4 : 3), 0);  // VALU
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                // 1 MFMA
                }
                __builtin_amdgcn_sched_barrier(0);
                if (ks + 1 < KS) wait_x(xa[nxt], MT);
            }
        }
        if constexpr (!SCALED_B) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int t = 0; t < 4; t++)
#pragma unroll
                    for (int r = 0; r < 4; r++) acc[mt][t][r] = fmaf(delta[t], accg[mt][t][r], acc[mt][t][r]);
        }
    };

    // Software pipeline over the chunk range, P = D - 1 chunks ahead.  Iteration g: wait for
    // everything issued up to iteration g-P (weights and this wave's part of x of chunk g),
    // meet the other waves (now all of x(g) is in LDS and nobody reads the slot of chunk g-1 any
    // more), issue x(g+P) and the weights of chunk g+P into that slot and the stage just freed
    // (stage index static: the loop is unrolled by D), consume chunk g.  The pipeline is primed
    // by issuing chunks g0 .. g0+P-1.
    // The loading side of the loop body is free of branches: the chunk count is rounded up to a
    // multiple of D; loads past the range point at the range's last chunk (the activations: cache
    // hits) or are issued with an empty execution mask (the weight side); the arithmetic of such
    // padded iterations is skipped.  Every iteration of a wave thus issues the same number of
    // loads (OX + OW, or one fewer on the waves that copy one block less), and since loads
    // complete in issue order "at most P-1 iterations' worth of loads outstanding" means all but
    // the last P-1 iterations' have landed.  Past the range the pointers stop.
    const int xlast = g0 + (nsup > 0 ? nsup - 1 : 0) * KP;  // first chunk of the last iteration
    auto advance = [&]() {
        const bool more = gi < wlast;
        gi += more ? KP : 0;
        wq += more ? KP * KSPG * wstep1 : 0;
        if constexpr (KP == 1) {
            kin += more ? 1 : 0;
            const bool wrap = kin == cpg;
            kin = wrap ? 0 : kin;
            sq += wrap ? (long)N * 2 : 0;
            zq += wrap ? (long)N : 0;
        } else {  // launched only with one chunk per group (cpg == 1)
            sq += more ? (long)KP * N * 2 : 0;
            zq += more ? (long)KP * N : 0;
        }
        const bool xmore = xg < xlast;
        xg += xmore ? KP : 0;
        xq += xmore ? KP * 64 * KSPG : 0;
    };
    Stage st[D];
#pragma unroll
    for (int j = 0; j < P; j++) {
        issue_x(j);
        issue_w(st[j], cs + j * KP < g1 && own_any);
        advance();
    }
    int slot = 0;  // ring slot of iteration it
    const int nblk = (nsup + D - 1) / D;
    for (int b = 0; b < nblk; b++) {
#pragma unroll
        for (int d = 0; d < D; d++) {
            const int it = b * D + d;             // iteration; this wave's chunk in it: cs + it * KP
            landed(st[d]);
            asm volatile("s_barrier" ::: "memory");
            const int fill = slot >= 1 ? slot - 1 : XD - 1;  // (slot + P) % XD
            issue_x(fill);
            issue_w(st[(d + P) % D], own_any && cs + (it + P) * KP < g1);
            advance();
            if (own_any && cs + it * KP < g1) compute(st[d], slot);  // padded iterations only keep the load counts in step
            slot = slot + 1 == XD ? 0 : slot + 1;
        }
    }
    // Look-ahead loads may still be in flight here (a range shorter than the pipeline issues
    // real loads it never consumes).  Their destination registers are dead by now as far as the
    // compiler can tell, but the hardware still writes them when the data arrives: `drain` waits
    // for everything outstanding and its empty uses keep every stage allocated until then, so
    // that nothing else is placed in those registers while a load is in flight.  It runs after the epilogue's stores have been issued (they only read the
    // accumulators), so that one wait covers both.
    auto drain = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < D; j++) {
#pragma unroll
            for (int ks = 0; ks < KS; ks++) asm volatile("" ::"v"(st[j].w[ks]));
            asm volatile("" ::"v"(st[j].sc));
            asm volatile("" ::"v"(st[j].zr));
        }
    };

    // ---- epilogue.  Accumulator tile t, register r of a lane: row mt*16 + 4*(lane/16) + r,
    // column n0 + 4*(lane%16) + t.
    const int nout = n0 + 4 * lc;
    drain();
    constexpr int SENDERS = KW * KP - 1;   // waves per strip beside the one that stores its results
    const int sid = kh + KW * ph;          // 0: the wave that stores the strip's results
    if constexpr (SENDERS > 0) {
        // A strip's waves add their sums: the others' go through LDS (the activation ring is idle
        // once every wave has passed the barrier) and the first adds them in a fixed order, then
        // only the first carries on.
        static_assert(SENDERS * NW * REGS * 256 == EXCHANGE, "the exchange fits the LDS array");
        f32x4 *ex = reinterpret_cast<f32x4 *>(xring) + (size_t)wave * (REGS / 4) * 64 + lane;
        constexpr int SSTRIDE = NW * (REGS / 4) * 64;  // one sender's strips
        __syncthreads();
        if (sid != 0) {
#pragma unroll
            for (int q = 0; q < REGS / 4; q++) ex[(sid - 1) * SSTRIDE + q * 64] = acc[q / 4][q % 4];
        }
        __syncthreads();
        if (sid == 0) {
#pragma unroll
            for (int sd = 0; sd < SENDERS; sd++)
#pragma unroll
                for (int q = 0; q < REGS / 4; q++) acc[q / 4][q % 4] += ex[sd * SSTRIDE + q * 64];
        }
    }
    const bool lead = sid == 0;
    if (split == 1) {
        if (lead && nout < N) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const int m = mt * 16 + 4 * lk + r;
                    if (m < M) store_row4(y, m, N, nout, epi, acc[mt][0][r], acc[mt][1][r], acc[mt][2][r], acc[mt][3][r]);
                }
        }
        return;
    }

    // ---- cross-workgroup: the last arrival adds the SPLIT partial tiles in split order.
    // Partials travel as device-scope (sc1) 16-byte stores and loads, written through and read
    // past the per-XCD L2, so no cache-wide write-back or invalidate is needed: each thread
    // waits for its own stores to complete, the barrier collects the workgroup, and only then
    // is the ticket taken.  Layout: [tile][split][wave][Q][lane][4] floats (each instruction
    // moves 1 KB contiguous per wave).
    constexpr int Q = REGS / 4;                         // 16-byte pieces per lane
    // partials fetched per round trip: what fits the register budget without spilling (the
    // variants with two waves per SIMD have 256 registers, so a split of 8 takes one round trip)
    constexpr int SB = MT == 1 ? (KW * KP >= 2 ? 8 : 6) : 32 / Q;
    {
        float *mine = ws.partial + (((size_t)tile * split + sidx) * NW + wave) * (64 * REGS) + lane * 4;
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
            if (lead && mt * 16 + 4 * lk < M) {  // lanes whose four rows are all past M have nothing to hand over
#pragma unroll
                for (int t = 0; t < 4; t++)
                    // (the s_nop: a store of more than 8 bytes reads its data registers up to two wait
                    // states after issue, and the compiler, which does not look inside asm statements,
                    // may reuse them for the next copy out of the accumulator registers right away)
                    asm volatile("global_store_dwordx4 %0, %1, off offset:%2 sc1\n\ts_nop 1" ::"v"(mine + mt * 1024), "v"(acc[mt][t]), "n"(t * 1024) : "memory");
            }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    if (threadIdx.x == 0) ticket_s = __hip_atomic_fetch_add(&ws.tickets[tile * TICKET_STRIDE], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (ticket_s != (unsigned)(split - 1)) return;
    if (lead) {
        const float *base = ws.partial + (((size_t)tile * split) * NW + wave) * (64 * REGS) + lane * 4;
        const size_t sstride = (size_t)NW * 64 * REGS;
        // Lanes whose four rows are all past M stored nothing and their sums are never written:
        // they re-read the first 16 lanes' pieces (the same cache lines) instead of lines of
        // their own, which for M <= 4 cuts the bytes the last arrival pulls in to a quarter.
        // (The loads stay unconditional: every lane's destination registers must be written by
        // exactly these instructions for the wait below to cover them.)
        int dead[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) dead[mt] = mt * 16 + 4 * lk < M ? 0 : -64 * lk;
        f32x4 sum[Q];
#pragma unroll
        for (int q = 0; q < Q; q++) sum[q] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int s0 = 0; s0 < split; s0 += SB) {
            f32x4 tmp[SB][Q];
#pragma unroll
            for (int j = 0; j < SB; j++)
                if (s0 + j < split) {
#pragma unroll
                    for (int q = 0; q < Q; q++)
                        asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(tmp[j][q]) : "v"(base + (size_t)(s0 + j) * sstride + q * 256 + dead[q / 4]) : "memory");
                }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int j = 0; j < SB; j++)
#pragma unroll
                for (int q = 0; q < Q; q++) asm volatile("" : "+v"(tmp[j][q]));
#pragma unroll
            for (int j = 0; j < SB; j++)
                if (s0 + j < split) {
#pragma unroll
                    for (int q = 0; q < Q; q++) sum[q] += tmp[j][q];
                }
        }
        if (nout < N) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const int m = mt * 16 + 4 * lk + r;
                    if (m < M) store_row4(y, m, N, nout, epi, sum[mt * 4 + 0][r], sum[mt * 4 + 1][r], sum[mt * 4 + 2][r], sum[mt * 4 + 3][r]);
                }
        }
    }
    if (threadIdx.x == 0)  // ready for the next launch on this stream
        __hip_atomic_store(&ws.tickets[tile * TICKET_STRIDE], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Any group size that is a multiple of 8 and any M: one thread per output element.
// Correctness path for group sizes the matrix-core kernels do not cover.
__global__ void __launch_bounds__(256)
w4a16_generic_kernel(int M, int N, int K, int group, const h16 *__restrict__ x, const uint32_t *__restrict__ packed,
                     const h16 *__restrict__ scales, const uint8_t *__restrict__ zeros, h16 *__restrict__ y)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int m = blockIdx.y;
    if (n >= N) return;
    const h16 *xr = x + (size_t)m * K;
    float acc = 0.f;
    for (int g = 0; g < K / group; g++) {
        const float d = (float)scales[(size_t)g * N + n];
        const int z = zeros[(size_t)g * N + n];
        float accg = 0.f;
        for (int j = 0; j < group / 8; j++) {
            const int row = g * (group / 8) + j;
            const uint32_t w = packed[(size_t)row * N + n];
#pragma unroll
            for (int i = 0; i < 8; i++)
                accg = fmaf((float)xr[row * 8 + i], (float)((int)((w >> (4 * i)) & 15u) - z), accg);
        }
        acc = fmaf(d, accg, acc);
    }
    y[(size_t)m * N + n] = (h16)acc;
}

// ---------------------------------------------------------------- launch

// Test/benchmark hooks: 1 = never two waves per strip; two chunks per iteration: 0 = automatic,
// 1 = never, 2 = wherever built.
int g_decode_kw = 0;
int g_decode_kp = 0;

// Two chunks per iteration (the kernel's KP = 2, twice the waves: two per SIMD where the launch
// has one workgroup per compute unit) pays once a workgroup walks at least 10 chunks: 5-10 %
// on the narrow 34B layers and on 11008->4096 / 13824->5120, a loss on ranges of 4 to 7 chunks
// (4096->4096, 5120->5120), where the pipeline is mostly ramp.
static bool two_chunks(int chunks, int split)
{
    if (g_decode_kp == 1) return false;
    if (g_decode_kp == 2) return true;
    return chunks / split >= 10;
}

// The split a launch really runs with (at most one part per chunk; none when the layer has
// more tiles than the workspace has tickets: such a layer fills the chip anyway) and the
// bytes of fp32 partial tiles it then leaves in the workspace.
int effective_split(int mt, int nw, int kspg, int N, int K, int split, size_t *partial_bytes)
{
    const int tiles = (N + 64 * nw - 1) / (64 * nw);
    const int chunks = K / (32 * kspg);
    if (split > chunks) split = chunks;
    if (split < 1) split = 1;
    if ((size_t)tiles * TICKET_STRIDE > SQP_WS_TICKETS) split = 1;
    *partial_bytes = split > 1 ? (size_t)tiles * split * nw * mt * 16 * 64 * sizeof(float) : 0;
    return split;
}

template <int MT, int NW, int KSPG>
int launch(int M, int N, int K, int cpg, int split, const h16 *x, const uint32_t *packed, const h16 *scales,
           const uint8_t *zeros, h16 *y, int epi, const SqpWorkspace &cws, hipStream_t st)
{
    constexpr int BN = 64 * NW;
    const int tiles = (N + BN - 1) / BN;
    size_t need = 0;
    split = effective_split(MT, NW, KSPG, N, K, split, &need);
    Workspace ws = {nullptr, nullptr};
    if (split > 1) {
        if (!cws.partial || !cws.tickets || need > cws.partial_bytes) return SQP_ERR_WORKSPACE;
        ws.partial = cws.partial;
        ws.tickets = cws.tickets;
    }
    // Up to 32 rows, chunks of four k-steps, two-strip workgroups, at most one workgroup per
    // compute unit: two waves per strip (see the kernel's KW)
    if constexpr (MT <= 2 && KSPG == 4 && NW == 2) {
        if (g_decode_kw != 1 && tiles * split <= 256) {
            {
                if (cpg == 1 && two_chunks(K / 128, split)) {  // and two chunks per iteration: eight waves
                    w4a16_decode_kernel<MT, NW, KSPG, 2, 2><<<dim3(tiles, split), NW * 4 * 64, 0, st>>>(M, N, K, cpg, x, packed, scales, zeros, y, ws, epi);
                    return sqp_launch_status();
                }
            }
            w4a16_decode_kernel<MT, NW, KSPG, 2, 1><<<dim3(tiles, split), NW * 2 * 64, 0, st>>>(M, N, K, cpg, x, packed, scales, zeros, y, ws, epi);
            return sqp_launch_status();
        }
    }
    if constexpr (MT <= 2 && KSPG == 4 && NW == 4) {
        if (cpg == 1 && tiles * split <= 256 && two_chunks(K / 128, split)) {
            w4a16_decode_kernel<MT, NW, KSPG, 1, 2><<<dim3(tiles, split), NW * 2 * 64, 0, st>>>(M, N, K, cpg, x, packed, scales, zeros, y, ws, epi);
            return sqp_launch_status();
        }
    }
    w4a16_decode_kernel<MT, NW, KSPG, 1, 1><<<dim3(tiles, split), NW * 64, 0, st>>>(M, N, K, cpg, x, packed, scales, zeros, y, ws, epi);
    return sqp_launch_status();
}

struct Plan {
    int nw, split;
};

// Strips per workgroup and K split, from sweeps on Code Llama shapes.  Four strips per
// workgroup share one copy of the activations.  Narrow layers (up to 128 column tiles) run
// best with at most one workgroup per compute unit (256 in all; one more than that and a
// second round of workgroups starts, which costs 20 % and more), each walking a long K
// range; wider ones with two to three workgroups per unit.  More splits than that cost
// more in fp32 partial tiles than the extra parallelism brings.
// Two strips per workgroup with half the split: the same number of waves when each strip
// has two (KW = 2: up to 32 rows, chunks of four k-steps), with half as many partial tiles to
// hand over but the activations fetched by twice as many workgroups.  That wins on the
// narrowest layers (up to 32 four-strip tiles) unless K is long (more than 24 chunks per
// workgroup), where the streaming phase outweighs the hand-over; with 17 to 32 rows the
// partial tiles are twice as large and it wins up to 40 tiles whatever K.  Without the two-wave
// variant, two strips only pay where 256 four-strip workgroups would get fewer than eight
// chunks each.
// kp_ok: the launch can take two chunks per iteration (up to 16 rows, groups of 128); then a
// layer of up to 40 four-strip tiles runs best in two-strip workgroups with half the split
// whatever K (8192->10240: 80 tiles x 3 instead of 40 x 6; 22016->8192: 64 x 4 instead of
// 32 x 8: half the partial tiles), if that leaves each workgroup at least 16 chunks.
Plan make_plan(int M, int N, int K, int chunk, bool kp_ok)
{
    const int chunks = K / chunk;
    int max_split = chunks / 4;  // at least four chunks per workgroup
    if (max_split < 1) max_split = 1;
    auto split_for = [&](int tiles) {
        int want = tiles <= 128 ? 256 / tiles : (704 + tiles / 2) / tiles;
        if (want > max_split) want = max_split;
        return want < 1 ? 1 : want;
    };
    Plan p;
    p.nw = 4;
    const int tiles4 = (N + 255) / 256;
    p.split = split_for(tiles4);
    const int split2 = split_for((N + 127) / 128);
    const bool two_waves = M <= 32 && chunk == 128;  // the launch will give each strip two waves
    bool two_strips;
    if (two_waves && M <= 16)
        two_strips = (tiles4 <= 32 && chunks <= 24 * split2) || (kp_ok && g_decode_kp != 1 && tiles4 <= 40 && chunks / split2 >= 16);
    else if (two_waves) two_strips = tiles4 <= 40;  // 17..32 rows: partial tiles twice as large, so also with a long K
    else two_strips = tiles4 <= 24 && chunks < 8 * (256 / tiles4);
    if (two_strips) {
        p.nw = 2;
        p.split = split2;
    }
    // More than 32 rows: the fp32 partial tiles are four times as large and the last arrival's
    // fetch of them is bound by its one compute unit, so the same waves are grouped into twice as
    // many workgroups of two strips (half the bytes per fetching unit; 1-6 % faster at M = 64).
    if (M > 32 && p.nw == 4 && p.split > 1) p.nw = 2;
    return p;
}

template <int MT, int KSPG>
int dispatch_mt(const Plan &p, int M, int N, int K, int cpg, const h16 *x, const uint32_t *packed, const h16 *scales,
                const uint8_t *zeros, h16 *y, int epi, const SqpWorkspace &ws, hipStream_t st)
{
    if (p.nw == 1) return launch<MT, 1, KSPG>(M, N, K, cpg, p.split, x, packed, scales, zeros, y, epi, ws, st);
    if (p.nw == 2) return launch<MT, 2, KSPG>(M, N, K, cpg, p.split, x, packed, scales, zeros, y, epi, ws, st);
    if constexpr (MT < 4)  // eight waves of the 64-row variant would not fit the register file
        if (p.nw == 8) return launch<MT, 8, KSPG>(M, N, K, cpg, p.split, x, packed, scales, zeros, y, epi, ws, st);
    return launch<MT, 4, KSPG>(M, N, K, cpg, p.split, x, packed, scales, zeros, y, epi, ws, st);
}

template <int KSPG>
int dispatch_kspg(const Plan &p, int M, int N, int K, int cpg, const h16 *x, const uint32_t *packed, const h16 *scales,
                  const uint8_t *zeros, h16 *y, int epi, const SqpWorkspace &ws, hipStream_t st)
{
    if (M <= 16) return dispatch_mt<1, KSPG>(p, M, N, K, cpg, x, packed, scales, zeros, y, epi, ws, st);
    if (M <= 32) return dispatch_mt<2, KSPG>(p, M, N, K, cpg, x, packed, scales, zeros, y, epi, ws, st);
    return dispatch_mt<4, KSPG>(p, M, N, K, cpg, x, packed, scales, zeros, y, epi, ws, st);
}

}  // namespace

// Test/benchmark hooks: force the K split, or the whole launch plan (0 = automatic).
static int g_force_split = 0;
static Plan g_force_plan = {0, 0};
extern "C" void sqp_debug_set_decode_split(int split) { g_force_split = split; }
extern "C" void sqp_debug_set_decode_plan(int nw, int split) { g_force_plan = Plan{nw, split}; }
extern "C" void sqp_debug_set_decode_kw(int kw) { g_decode_kw = kw; }
extern "C" void sqp_debug_set_decode_kp(int kp) { g_decode_kp = kp; }
static int g_slice_mode = 0;
extern "C" void sqp_debug_set_decode_slice(int mode) { g_slice_mode = mode; }

// Whether a call takes the column-slice kernel (-1: no), and which variant (0: 32-column
// slices, 1: 64-column slices).  From sweeps on Code Llama shapes: the slice kernel has no
// hand-over between workgroups, but every workgroup fetches all of x from L2, and that traffic
// (workgroups x fetched rows x K) is what it costs.  It wins up to 8 rows (a third to a half of
// the activation traffic of 16 rows at K = 8192) and beyond that where x is small (short K) and
// the strip kernel is furthest from its roofline (narrow layers): 64-column slices from 150
// slices on (more than 8 rows: up to 128 KB of x per workgroup, or up to 192 KB and at most 400
// slices); below that 32-column slices, unless K is long and the slices are few (then the
// activations dominate again; 5 to 12 rows: only with K up to 8192, 13 to 16: up to 4096).
static int slice_variant(int M, int N, int K, int group)
{
    if (g_slice_mode < 0 || !sqp_gemm_slice_covers(M, N, K, group)) return -1;
    if (g_slice_mode > 0) return g_slice_mode - 1;
    const long xbytes = 4L * ((M + 3) / 4) * K * 2;  // activations a workgroup fetches
    const int slices64 = (N + 63) / 64, slices32 = (N + 31) / 32;
    if (slices64 >= 150) return (M <= 8 || xbytes <= (128L << 10) || (xbytes <= (192L << 10) && slices64 <= 400)) ? 1 : -1;
    if (slices32 >= 96 && (slices32 >= 200 || K <= 8192)) return (M <= 4 || (M <= 12 && K <= 8192) || K <= 4096) ? 0 : -1;
    return -1;
}
extern "C" int sqp_debug_decode_slice_choice(int M, int N, int K, int group) { return slice_variant(M, N, K, group); }

int sqp_gemm_generic(int M, int N, int K, int group, const h16 *x, const uint32_t *packed, const h16 *scales,
                     const uint8_t *zeros, h16 *y, hipStream_t stream)
{
    if (M > 65535) return SQP_ERR_SHAPE;
    w4a16_generic_kernel<<<dim3((N + 255) / 256, M), 256, 0, stream>>>(M, N, K, group, x, packed, scales, zeros, y);
    return sqp_launch_status();
}

// Test hook: the launch plan the library would pick for a shape (no launch, no GPU needed):
// strips per workgroup, K split as requested by the heuristic, and the kernel family
// (0 = generic, else k-steps per chunk).
extern "C" void sqp_debug_decode_plan(int M, int N, int K, int group, int *nw, int *split, int *kspg)
{
    const int chunk = group % 128 == 0 ? 128 : group;
    const Plan p = make_plan(M, N, K, chunk, M <= 16 && group == 128);
    *nw = p.nw;
    *split = p.split;
    *kspg = group == 32 ? 1 : (group == 64 ? 2 : (group % 128 == 0 ? 4 : 0));
}

// The plan a call runs with: the heuristic's, overridden by the test hooks, without a split
// when there is no workspace to put partial sums in.
static Plan plan_for(int M, int N, int K, int group, bool have_workspace)
{
    const int chunk = group % 128 == 0 ? 128 : group;
    Plan p = make_plan(M, N, K, chunk, M <= 16 && group == 128);
    if (g_force_plan.nw > 0) p = g_force_plan;
    if (g_force_split > 0) p.split = g_force_split;
    if (!have_workspace) p.split = 1;
    return p;
}

size_t sqp_gemm_decode_partial_bytes(int M, int N, int K, int group)
{
    const int kspg = group == 32 ? 1 : (group == 64 ? 2 : (group % 128 == 0 ? 4 : 0));
    if (kspg == 0) return 0;  // generic kernel
    if (slice_variant(M, N, K, group) >= 0) return 0;
    const Plan p = plan_for(M, N, K, group, true);
    const int mt = M <= 16 ? 1 : (M <= 32 ? 2 : 4);
    int nw = p.nw;
    if (nw != 1 && nw != 2 && !(nw == 8 && mt < 4)) nw = 4;
    size_t bytes = 0;
    effective_split(mt, nw, kspg, N, K, p.split, &bytes);
    return bytes;
}

int sqp_gemm_decode(int M, int N, int K, int group, const h16 *x, const uint32_t *packed, const h16 *scales,
                    const uint8_t *zeros, h16 *y, int epi, const SqpWorkspace &ws, hipStream_t stream)
{
    const int sv = slice_variant(M, N, K, group);
    if (sv >= 0) return sqp_gemm_slice(sv, M, N, K, x, packed, scales, zeros, y, epi, stream);
    const Plan p = plan_for(M, N, K, group, ws.partial != nullptr);
    if (group == 32) return dispatch_kspg<1>(p, M, N, K, 1, x, packed, scales, zeros, y, epi, ws, stream);
    if (group == 64) return dispatch_kspg<2>(p, M, N, K, 1, x, packed, scales, zeros, y, epi, ws, stream);
    if (group % 128 == 0) return dispatch_kspg<4>(p, M, N, K, group / 128, x, packed, scales, zeros, y, epi, ws, stream);
    if (epi != 0) return SQP_ERR_SHAPE;  // the fused activation needs a group size the matrix-core kernels cover
    return sqp_gemm_generic(M, N, K, group, x, packed, scales, zeros, y, stream);
}

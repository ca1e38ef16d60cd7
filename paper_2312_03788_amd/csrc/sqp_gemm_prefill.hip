// Tiled matrix-core W4A16 GEMM for large M (prefill): y = x * w_hat, Eq. 3 of
// arXiv 2312.03788 with w_hat = fp16((code - Z) * Delta) of Eq. 1, group-wise along K.
//
// A workgroup of 4 waves (one per SIMD, the whole register file each) computes a 128 x 512
// tile of y, the waves side by side on the same 128 rows (or a 256 x 256 tile, waves 2 x 2);
// a wave owns 128 rows x 128 columns as 4 x 4 accumulator tiles of v_mfma_f32_32x32x16_f16
// (256 fp32 registers per lane).
//   - Weights never pass through LDS: one dwordx4 load per lane fetches, for k-block
//     (lane / 32), the packed words of 4 adjacent columns; a word is 8 consecutive k of one
//     column, i.e. one lane's B operand of the 32x32x16 MFMA (column = lane % 32).  The word
//     is unpacked in registers to the fp16 dequantised weights (13 VALU ops) and each B
//     operand feeds 4 MFMAs (the 4 row tiles); each activation fragment feeds 4 as well
//     (4.25 VALU ops per MFMA).
//   - Activations are the shared operand: a 128 x 64 (256 x 64) slice of x per stage is copied
//     once per workgroup straight into a four-slot LDS ring (direct global->LDS loads of whole
//     128-byte lines, pieces XOR-swizzled so that the 16-byte reads of one k-step spread over
//     all banks) and every wave reads its A operands from there.
//   - With a single wave per SIMD the order of issue is the schedule, so the MFMAs and the
//     vector instructions of a k-step are written out in issue order (see the stream below):
//     while the 16 MFMAs of one k-step run, the activation fragments of the next arrive from
//     LDS and the next weight words are unpacked; the hand-over to the next stage (wait for
//     its loads, barrier) sits inside the last k-step, so the pipeline never drains.
//   - Loads, waits and the per-stage barrier are explicit (assembly), as in the decode
//     kernel: two stages stay in flight while one is consumed.
// Eight waves of 128 x 64 (two per SIMD) needed fewer cycles per MFMA, but the chip then
// clocked lower under its power limit and the result was a little slower, so one wave per SIMD
// it is.
#include <type_traits>

#include "sqp_common.h"
#include "sqp_w4_unpack.h"

namespace {

constexpr int BK = 64;

// NT: 32-column MFMA tiles per wave (wave tile 128 rows x 32 NT columns); WM: waves along the
// rows, the other 4 / WM along the columns.
//   <4, 1>: 128 x 512 tile, the four waves side by side on the same 128 rows.  Every packed word
//           is then loaded and unpacked by exactly one wave, and a workgroup stages half as
//           many activation bytes per matrix instruction as with the square tile.
//   <4, 2>: 256 x 256 tile, waves 2 x 2 (the two waves of a column pair unpack the same words).
//   <2, *>: the same with half the columns (128 x 256 / 256 x 128), used for the tiles left over
//           after the last full round so that the tail of a launch costs half a round, and for
//           the K-split launches.
// Workgroup b of the launch handles tile tile0 + b / (full columns / columns) of the tn x tm grid
// of full tiles (column index fastest), column half b % 2 of it when it covers half.
// G32: quantisation groups of 32 rows, i.e. two groups per 64-row stage (the steps and zero
// points of both are loaded per stage and the unpack switches sets after the second k-step);
// otherwise the group is a multiple of 64 rows.
template <int NT, int WM, bool G32>
__global__ void __launch_bounds__(256)
w4a16_prefill_kernel(int M, int N, int K, int group, int tile0, int tn, const h16 *__restrict__ x,
                     const uint32_t *__restrict__ packed, const h16 *__restrict__ scales,
                     const uint8_t *__restrict__ zeros, h16 *__restrict__ y, float *__restrict__ part, int epi)
{
    constexpr int W = 4;                   // waves: one per SIMD
    constexpr int WNW = W / WM;            // waves along the columns
    constexpr int BM = 128 * WM;           // rows per workgroup
    constexpr int FULLN = WNW * 128;       // columns of a full tile of this arrangement
    constexpr int WN = 32 * NT;            // columns per wave
    typedef uint32_t wvec __attribute__((ext_vector_type(NT)));
    typedef std::conditional_t<NT == 4, u32x2, uint32_t> scvec;
    constexpr int D = 3;                   // register stages of packed weights (two in flight)
    constexpr int XD = 4;                  // LDS slots of activations
    constexpr int XSTAGE = BM * BK * 2;   // 16 or 32 KB: blocks of 8 rows x 128 bytes
    constexpr int OX = (BM / 8) / W;       // direct loads per wave per stage (one per 1 KB block)
    constexpr int WGN = WNW * WN;          // columns per workgroup: a full tile's or half of them
    static_assert(OX % 4 == 0, "the loads of a stage are spread evenly over its four k-steps");
    constexpr int NQ = G32 ? 2 : 1;        // quantisation groups per stage
    constexpr int OW = 4 + 2 * NQ;
    __shared__ __attribute__((aligned(1024))) unsigned char xring[XD * XSTAGE];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WNW, wn = wave % WNW;
    const int l32 = lane & 31, kb = lane >> 5;
    const int tile = tile0 + (int)blockIdx.x / (FULLN / WGN);
    const int nbase = (tile % tn) * FULLN + (WGN == FULLN ? 0 : ((int)blockIdx.x & 1) * WGN);
    const int m0 = (tile / tn) * BM;
    const int n0 = nbase + wn * WN;
    // K split across gridDim.y workgroups (part != nullptr): this one takes stages
    // [stage0, stage0 + stages) and leaves its fp32 sums in part[blockIdx.y][M][N].
    const int stages_all = K / BK;
    const int stage0 = (int)((long)stages_all * blockIdx.y / gridDim.y);
    const int stages = (int)((long)stages_all * (blockIdx.y + 1) / gridDim.y) - stage0;
    const int spg = G32 ? 1 : group / BK;  // stages per quantisation group (G32: two groups per stage)

    int ncol = n0 + NT * l32;
    if (ncol >= N) ncol = 0;

    f32x16 acc[4][NT];
#pragma unroll
    for (int mt = 0; mt < 4; mt++)
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[mt][t][r] = 0.f;
    const UnpackConsts uc = SQP_UNPACK_CONSTS;

    struct Stage {
        wvec w[4];    // per k-step: packed words of the lane's NT columns
        scvec sc[NQ];     // NT fp16 steps (per group of the stage)
        uint32_t zr[NQ];  // NT zero points, one byte each
    };

    // The loading side walks the stages with wave-uniform byte pointers that are advanced by
    // constant strides (scalar adds only); past the last stage they stop, so that the padded
    // stages of the branch-free loop re-read the last one (cache hits).
    const long wrow2 = (long)N * 8;        // two packed rows (one k-step) in bytes
    const unsigned char *wq = reinterpret_cast<const unsigned char *>(packed) + (long)stage0 * 4 * wrow2;
    const long prow = G32 ? (long)stage0 * 2 : (long)(stage0 / spg);  // first parameter row of this workgroup
    const unsigned char *sq = reinterpret_cast<const unsigned char *>(scales) + prow * N * 2;
    const unsigned char *zq = zeros + prow * N;
    const unsigned char *xq = reinterpret_cast<const unsigned char *>(x) + (long)stage0 * (BK * 2);
    int ist = 0, kin = stage0 % spg;        // stage being issued (relative), its position inside its group
    const uint32_t voff_w = (uint32_t)(kb * N + ncol) * 4u;
    const uint32_t voff_s = (uint32_t)ncol * 2u, voff_z = (uint32_t)ncol;
    auto issue_w = [&](Stage &s) {
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            const unsigned char *base = wq + ks * wrow2;  // wave-uniform
            if constexpr (NT == 4)
                asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(s.w[ks]) : "v"(voff_w), "s"(base) : "memory");
            else
                asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(s.w[ks]) : "v"(voff_w), "s"(base) : "memory");
        }
#pragma unroll
        for (int g = 0; g < NQ; g++) {
            const unsigned char *sg = sq + (long)g * N * 2, *zg = zq + (long)g * N;  // wave-uniform
            if constexpr (NT == 4) {
                asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(s.sc[g]) : "v"(voff_s), "s"(sg) : "memory");
                asm volatile("global_load_dword %0, %1, %2" : "=v"(s.zr[g]) : "v"(voff_z), "s"(zg) : "memory");
            } else {
                asm volatile("global_load_dword %0, %1, %2" : "=v"(s.sc[g]) : "v"(voff_s), "s"(sg) : "memory");
                asm volatile("global_load_ushort %0, %1, %2" : "=v"(s.zr[g]) : "v"(voff_z), "s"(zg) : "memory");
            }
        }
    };
    auto landed = [&](Stage &s, auto after) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(decltype(after)::value) : "memory");
#pragma unroll
        for (int ks = 0; ks < 4; ks++) asm volatile("" : "+v"(s.w[ks]));
#pragma unroll
        for (int g = 0; g < NQ; g++) {
            asm volatile("" : "+v"(s.sc[g]));
            asm volatile("" : "+v"(s.zr[g]));
        }
    };

    // Activations: wave w copies blocks w, w+4, ..., w+28 of the stage (a block = 8 rows x 128
    // bytes).  Lane i of a block handles row i / 8 of the block and fetches piece
    // (i % 8) ^ key(row) of that row's 128 bytes, key(row) = (row / 2) % 8; the hardware puts
    // lane i at byte 16*i of the block.
    uint32_t xoff[OX];
#pragma unroll
    for (int j = 0; j < OX; j++) {
        const int b = wave + W * j;
        const int row = b * 8 + (lane >> 3);
        int grow = m0 + row;
        if (grow >= M) grow = M - 1;
        const int piece = (lane & 7) ^ ((row >> 1) & 7);
        xoff[j] = (uint32_t)grow * (uint32_t)K * 2u + (uint32_t)(piece * 16);
    }
    auto issue_x = [&](int slot, int j) {
        unsigned char *dst = xring + slot * XSTAGE + (wave + W * j) * 1024;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(xq + xoff[j]),
                                         (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    };
    // all loads of the stage have been issued: step the pointers unless it was the last stage
    auto advance = [&]() {
        const bool more = ist + 1 < stages;
        ist += more ? 1 : 0;
        wq += more ? 4 * wrow2 : 0;
        xq += more ? BK * 2 : 0;
        kin += more ? 1 : 0;
        const bool wrap = kin == spg;
        kin = wrap ? 0 : kin;
        sq += wrap ? (long)N * 2 * NQ : 0;
        zq += wrap ? (long)N * NQ : 0;
    };
    const uint32_t xrd0 = (uint32_t)(size_t)xring +
                          (uint32_t)(((wm * 128 + l32) >> 3) * 1024 + ((wm * 128 + l32) & 7) * 128);
    const int xkey = (l32 >> 1) & 7;

    auto read_a = [&](u32x4 (&xa)[4], int slot, int ks) {
        const uint32_t poff = xrd0 + (uint32_t)(slot * XSTAGE) + (uint32_t)((((ks * 2 + kb) ^ xkey)) * 16);
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(xa[mt]) : "v"(poff), "n"(mt * 4096) : "memory");
    };
    auto wait_a = [&](u32x4 (&xa)[4]) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int mt = 0; mt < 4; mt++) asm volatile("" : "+v"(xa[mt]));
    };

    // per-stage constants of the unpack: -(1024 + Z), -(64 + Z) and the step, each in both
    // halves of a register; a stage past the end gets a step of 0 and adds nothing
    // (one set per quantisation group of the stage)
    h16x2 neg_hi[NQ][NT], neg_lo[NQ][NT], delta[NQ][NT];
    auto stage_consts = [&](const Stage &s, bool live) {
        const uint32_t sel_even = live ? 0x01000100u : 0x0c0c0c0cu;  // byte selectors of v_perm_b32
        const uint32_t sel_odd = live ? 0x03020302u : 0x0c0c0c0cu;   // (0x0c selects a zero byte)
#pragma unroll
        for (int g = 0; g < NQ; g++)
#pragma unroll
            for (int t = 0; t < NT; t++) {
                const uint32_t z = (s.zr[g] >> (8 * t)) & 0xffu;
                neg_hi[g][t] = neg_hi_of(z);
                neg_lo[g][t] = neg_lo_of(z);
                uint32_t sw;
                if constexpr (NT == 4) sw = s.sc[g][t >> 1]; else sw = s.sc[g];
                delta[g][t] = __builtin_bit_cast(h16x2, __builtin_amdgcn_perm(sw, sw, (t & 1) ? sel_odd : sel_even));
            }
    };

    // One continuous software pipeline over all k-steps.  While the 16 MFMAs of a k-step
    // issue, the A fragments of the next k-step come from LDS and the next weight word is
    // unpacked.  The hand-over to the next stage happens inside the last k-step of a stage
    // (wait for the next stage's loads, barrier, new constants), so the first LDS reads and
    // the first unpack of a stage are hidden like any other.  Ring discipline: the barrier in
    // the last k-step of stage s-1 proves every wave has finished stage s-2, whose LDS slot
    // (four slots) and weight registers (three stages) are refilled during stage s with the
    // loads of stage s+2.
    Stage stg[D];
    u32x4 xa[2][4];          // raw A fragments from LDS: [k-step parity][row tile]
    uint32_t aq[2][4];       // permuted A operand of row tile m in aq[m % 2]
    uint32_t bq[2][NT][4];   // B operands (dequantised weights): [k-step parity][column tile]
    uint32_t w8[NT];
    const uint32_t sel_a = 0x05040100u, sel_b = 0x07060302u;  // v_perm_b32 selectors of permute_x

    // ---- The instruction stream of one k-step, in issue order, written out by hand.
    // With one wave per SIMD the order of issue is the schedule: measured on this chip, an
    // independent vector instruction costs 4 cycles and up to 4 of them hide behind a
    // 32x32x16 MFMA, but one that depends on the instruction just before it costs about 8, and
    // the compiler's own order left many such pairs.  So every MFMA and every vector
    // instruction of the k-step is a volatile asm statement (these keep their order), grouped
    // so that a result is used no sooner than 4 instructions later:
    //   MFMA i (row tile i / NT, column tile i % NT), then the next 4-5 entries of the list
    //     P1, S, AO.., P2, AO.., ADD.., P3, ADD.., MUL.., P0', MUL
    //   P<m>: 4 perms giving row tile m's A operand (P0': row tile 0 of the NEXT k-step, after
    //   the wait for its LDS reads); S: word >> 8; AO/ADD/MUL<t>: the and-or, add and multiply
    //   of the 4 registers of the next k-step's B operand t.
    // The compiler does not look inside asm statements, so the wait states it would insert
    // are guaranteed by the order itself: vector write -> MFMA read needs 2 (every operand is
    // written >= 4 instructions ahead), vector write -> packed-math read needs 1.
    auto mfma = [&](f32x16 &c, const uint32_t (&av)[4], const uint32_t (&bv)[4]) {
        const u32x4 a4 = {av[0], av[1], av[2], av[3]};
        const u32x4 b4 = {bv[0], bv[1], bv[2], bv[3]};
        asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a4), "v"(b4));
    };
    auto perm4 = [&](uint32_t (&dst)[4], const u32x4 &v, int j) {
        if (j == 0) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(dst[0]) : "v"(v.z), "v"(v.x), "s"(sel_a));
        if (j == 1) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(dst[1]) : "v"(v.z), "v"(v.x), "s"(sel_b));
        if (j == 2) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(dst[2]) : "v"(v.w), "v"(v.y), "s"(sel_a));
        if (j == 3) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(dst[3]) : "v"(v.w), "v"(v.y), "s"(sel_b));
    };
    enum { G_P1, G_P2, G_P3, G_P0N, G_S, G_AO, G_ADD = G_AO + 4, G_MUL = G_ADD + 4 };
    constexpr int NG = NT == 4 ? 17 : 11;
    constexpr int order4[17] = {G_P1, G_S, G_AO + 0, G_AO + 1, G_P2, G_AO + 2, G_AO + 3, G_ADD + 0, G_P3,
                                G_ADD + 1, G_ADD + 2, G_ADD + 3, G_MUL + 0, G_MUL + 1, G_MUL + 2, G_P0N, G_MUL + 3};
    constexpr int order2[17] = {G_P1, G_S, G_P2, G_AO + 0, G_AO + 1, G_P3, G_ADD + 0, G_ADD + 1, G_MUL + 0, G_P0N, G_MUL + 1,
                                0, 0, 0, 0, 0, 0};
    constexpr int NMF = 4 * NT;                 // MFMAs per k-step
    constexpr int WAIT_AT = NT == 4 ? 13 : 5;   // the LDS wait goes in front of this MFMA

    // one entry j of group g; wn = the packed words of the next k-step, kn = that k-step's
    // position in its stage (it selects the quantisation group's constants)
    auto valu = [&](int g, int j, int cur, const wvec &wn, int kn) {
        const int nxt = cur ^ 1;
        const int qs = G32 ? (kn >> 1) : 0;
        if (g == G_P1) perm4(aq[1], xa[cur][1], j);
        else if (g == G_P2) perm4(aq[0], xa[cur][2], j);
        else if (g == G_P3) perm4(aq[1], xa[cur][3], j);
        else if (g == G_P0N) perm4(aq[0], xa[nxt][0], j);
        else if (g == G_S) {
            if (j < NT) asm volatile("v_lshrrev_b32 %0, 8, %1" : "=v"(w8[j]) : "v"(wn[j]));
        } else if (g < G_ADD) {
            const int t = g - G_AO;
            if (j & 1) asm volatile("v_and_or_b32 %0, %1, %2, %3" : "=v"(bq[nxt][t][j]) : "v"(j < 2 ? wn[t] : w8[t]), "v"(uc.mask_hi), "v"(uc.magic_hi));
            else       asm volatile("v_and_or_b32 %0, %1, %2, %3" : "=v"(bq[nxt][t][j]) : "v"(j < 2 ? wn[t] : w8[t]), "v"(uc.mask_lo), "v"(uc.magic_lo));
        } else if (g < G_MUL) {
            const int t = g - G_ADD;
            if (j & 1) asm volatile("v_pk_add_f16 %0, %0, %1" : "+v"(bq[nxt][t][j]) : "v"(neg_lo[qs][t]));
            else       asm volatile("v_pk_add_f16 %0, %0, %1" : "+v"(bq[nxt][t][j]) : "v"(neg_hi[qs][t]));
        } else {
            const int t = g - G_MUL;
            asm volatile("v_pk_mul_f16 %0, %0, %1" : "+v"(bq[nxt][t][j]) : "v"(delta[qs][t]));
        }
    };

    issue_w(stg[0]);
#pragma unroll
    for (int j = 0; j < OX; j++) issue_x(0, j);
    advance();
    issue_w(stg[1]);
#pragma unroll
    for (int j = 0; j < OX; j++) issue_x(1, j);
    advance();
    landed(stg[0], std::integral_constant<int, OX + OW>());
    asm volatile("s_barrier" ::: "memory");
    stage_consts(stg[0], true);
    read_a(xa[0], 0, 0);
    // first operands of the pipeline, by the ordinary helpers
#pragma unroll
    for (int t = 0; t < NT; t++) {
        const u32x4 bw = __builtin_bit_cast(u32x4, dequant_word_scaled(stg[0].w[0][t], neg_hi[0][t], neg_lo[0][t], delta[0][t], uc));
        bq[0][t][0] = bw.x; bq[0][t][1] = bw.y; bq[0][t][2] = bw.z; bq[0][t][3] = bw.w;
    }
    wait_a(xa[0]);
    {
        const u32x4 a0 = __builtin_bit_cast(u32x4, permute_x(xa[0][0]));
        aq[0][0] = a0.x; aq[0][1] = a0.y; aq[0][2] = a0.z; aq[0][3] = a0.w;
    }
    asm volatile("s_nop 3" ::: "memory");  // compiler-issued vector writes above -> asm MFMA reads below

    int slot = 0;  // ring slot of the stage being consumed
    const int nblk = (stages + D - 1) / D;
    for (int blk = 0; blk < nblk; blk++) {
#pragma unroll
        for (int d = 0; d < D; d++) {
            const int st = blk * D + d;
            Stage &cur_s = stg[d];
            Stage &next_s = stg[(d + 1) % D];
            Stage &fill_s = stg[(d + 2) % D];
            const int slot_next = (slot + 1) & (XD - 1), slot_fill = (slot + 2) & (XD - 1);
            issue_w(fill_s);
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                const int cur = ks & 1, nxt = cur ^ 1;
#pragma unroll
                for (int j = 0; j < OX / 4; j++) issue_x(slot_fill, (OX / 4) * ks + j);
                if (ks < 3) {
                    read_a(xa[nxt], slot, ks + 1);
                } else {
                    advance();
                    landed(next_s, std::integral_constant<int, OX + OW>());
                    asm volatile("s_barrier" ::: "memory");
                    stage_consts(next_s, st + 1 < stages);
                    read_a(xa[nxt], slot_next, 0);
                }
                const wvec wn = ks < 3 ? cur_s.w[ks + 1] : next_s.w[0];
#pragma unroll
                for (int i = 0; i < NMF; i++) {
                    if (i == WAIT_AT) wait_a(xa[nxt]);
                    mfma(acc[i / NT][i % NT], aq[(i / NT) & 1], bq[cur][i % NT]);
#pragma unroll
                    for (int e = i * (4 * NG) / NMF; e < (i + 1) * (4 * NG) / NMF; e++)
                        valu(NT == 4 ? order4[e / 4] : order2[e / 4], e % 4, cur, wn, (ks + 1) & 3);
                }
            }
            // End of the last iteration.  (1) Drain the clamped look-ahead loads: their
            // destination registers are dead as far as the compiler can tell, but the hardware
            // still writes them when the data arrives, so the empty uses keep every stage
            // allocated until the wait has completed.  (2) The compiler does not know that the
            // asm statements above wrote the accumulators with MFMAs, so it will not insert the
            // wait states a matrix result needs before another instruction may read it (up to
            // 18); the epilogue's reads follow the loop directly, so they are spent here.
            if (d == D - 1 && blk == nblk - 1) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
                for (int j = 0; j < D; j++) {
#pragma unroll
                    for (int ks = 0; ks < 4; ks++) asm volatile("" ::"v"(stg[j].w[ks]));
#pragma unroll
                    for (int g = 0; g < NQ; g++) {
                        asm volatile("" ::"v"(stg[j].sc[g]));
                        asm volatile("" ::"v"(stg[j].zr[g]));
                    }
                }
                asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
            }
            slot = slot_next;
        }
    }

    // epilogue: accumulator register r of tile (mt, t): row 8*(r/4) + 4*(lane/32) + r%4 of the
    // 32-row tile, column NT*(lane%32) + t of the wave's 32*NT
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int e_l32 = tid & 31, e_kb = (tid >> 5) & 1, e_wave = tid >> 6;
    const int nout = nbase + (e_wave % WNW) * WN + NT * e_l32;
    const int mrow0 = m0 + (e_wave / WNW) * 128 + 4 * e_kb;
    if (part != nullptr) {
        if (nout < N) {
            float *pcol = part + (size_t)blockIdx.y * M * N + nout;
#pragma unroll
            for (int mt = 0; mt < 4; mt++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int m = mrow0 + mt * 32 + 8 * (r >> 2) + (r & 3);
                    if (m < M) {
                        if constexpr (NT == 4)
                            *reinterpret_cast<f32x4 *>(pcol + (size_t)m * N) = f32x4{acc[mt][0][r], acc[mt][1][r], acc[mt][2][r], acc[mt][3][r]};
                        else
                            *reinterpret_cast<float2 *>(pcol + (size_t)m * N) = make_float2(acc[mt][0][r], acc[mt][1][r]);
                    }
                }
        }
        return;
    }
    if (nout < N) {
        h16 *ycol = y + nout;
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int m = mrow0 + mt * 32 + 8 * (r >> 2) + (r & 3);
                if (m < M) {
                    if (epi != 0) {
                        // adjacent columns are (gate j, up j): y [M][N/2] = SiLU(gate) * up
                        h16 *yh = y + (size_t)m * (N >> 1) + (nout >> 1);
                        if constexpr (NT == 4) {
                            h16x2 o;
                            o.x = (h16)(sqp_silu(acc[mt][0][r]) * acc[mt][1][r]);
                            o.y = (h16)(sqp_silu(acc[mt][2][r]) * acc[mt][3][r]);
                            *reinterpret_cast<h16x2 *>(yh) = o;
                        } else {
                            *yh = (h16)(sqp_silu(acc[mt][0][r]) * acc[mt][1][r]);
                        }
                    } else if constexpr (NT == 4) {
                        h16x4 o;
                        o.x = (h16)acc[mt][0][r]; o.y = (h16)acc[mt][1][r];
                        o.z = (h16)acc[mt][2][r]; o.w = (h16)acc[mt][3][r];
                        *reinterpret_cast<h16x4 *>(ycol + (size_t)m * N) = o;
                    } else {
                        h16x2 o;
                        o.x = (h16)acc[mt][0][r]; o.y = (h16)acc[mt][1][r];
                        *reinterpret_cast<h16x2 *>(ycol + (size_t)m * N) = o;
                    }
                }
            }
    }
}

// y = fp16(sum over the K parts, in part order) of the fp32 partial matrices: 8 elements
// per thread.
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const float *__restrict__ part, long total8, long stride, int parts,
                                                            h16 *__restrict__ y, int epi)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total8) return;
    const f32x4 *p = reinterpret_cast<const f32x4 *>(part) + 2 * i;
    f32x4 a = p[0], b = p[1];
    for (int s = 1; s < parts; s++) {
        const f32x4 *q = reinterpret_cast<const f32x4 *>(part + (size_t)s * stride) + 2 * i;
        a += q[0];
        b += q[1];
    }
    if (epi != 0) {  // (gate, up) pairs -> SiLU(gate) * up; 8 adjacent columns of [M][N] are 4 of [M][N/2]
        h16x4 o;
        o.x = (h16)(sqp_silu(a.x) * a.y); o.y = (h16)(sqp_silu(a.z) * a.w);
        o.z = (h16)(sqp_silu(b.x) * b.y); o.w = (h16)(sqp_silu(b.z) * b.w);
        reinterpret_cast<h16x4 *>(y)[i] = o;
        return;
    }
    h16x8 o;
    o.s0 = (h16)a.x; o.s1 = (h16)a.y; o.s2 = (h16)a.z; o.s3 = (h16)a.w;
    o.s4 = (h16)b.x; o.s5 = (h16)b.y; o.s6 = (h16)b.z; o.s7 = (h16)b.w;
    reinterpret_cast<h16x8 *>(y)[i] = o;
}

int compute_units()
{
    static int cus = 0;  // same on every device of a node
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cus = n;
    }
    return cus;
}

}  // namespace

// Test/benchmark hooks.  Tiles: 0 = automatic tile choice, 1 = full tiles only, 2 = half tiles
// only.  K split: -1 = automatic, 0 or 1 = never, k >= 2 = k parts.  Shape: 0 = automatic,
// 1 = 128 x 512 full tiles (waves 1 x 4), 2 = 256 x 256 (waves 2 x 2).
static int g_tile_mode = 0, g_ksplit = -1, g_tile_shape = 0;
extern "C" void sqp_debug_set_prefill_tiles(int mode) { g_tile_mode = mode; }
extern "C" void sqp_debug_set_prefill_ksplit(int k) { g_ksplit = k; }
extern "C" void sqp_debug_set_prefill_shape(int shape) { g_tile_shape = shape; }

// The weight-streaming kernel, 64 rows at a time.
static int decode_in_row_blocks(int M, int N, int K, int group, const h16 *x, const uint32_t *packed,
                                const h16 *scales, const uint8_t *zeros, h16 *y, int epi, const SqpWorkspace &ws, hipStream_t stream)
{
    const size_t ystride = epi != 0 ? (size_t)(N >> 1) : (size_t)N;
    for (int mb = 0; mb < M; mb += 64) {
        int rows = M - mb < 64 ? M - mb : 64;
        int rc = sqp_gemm_decode(rows, N, K, group, x + (size_t)mb * K, packed, scales, zeros, y + (size_t)mb * ystride, epi, ws, stream);
        if (rc) return rc;
    }
    return SQP_OK;
}

// Launch plan of the tiled path: `full` full tiles (128 x 512 with wm == 1, 256 x 256 with
// wm == 2) in a first launch, then `half` half-width tiles (starting at full tile `full`), the
// latter times `ksplit` K parts.
struct TilePlan {
    long full, half;
    int ksplit, wm;
};

static TilePlan plan_tiles(int M, int N, int K, int group, int cus, bool have_workspace)
{
    const int wm = (g_tile_shape == 2 && group != 32) ? 2 : 1;  // groups of 32: the 128 x 512 shape only
    const int bm = 128 * wm, fulln = (4 / wm) * 128;
    const int tn = (N + fulln - 1) / fulln, tm = (M + bm - 1) / bm;
    const long tiles = (long)tn * tm;
    const int stages = K / BK;
    TilePlan p = {tiles, 0, 1, wm};
    // (1) Too few tiles to occupy the chip even as half-width tiles: split K as well.  Half
    // tiles times K parts fill the compute units; every part leaves an fp32 [M][N] matrix in
    // the workspace and a second kernel adds the parts in order (deterministic).
    int ksplit = 1;
    if (g_tile_mode == 0 && 4 * tiles <= cus) {
        ksplit = (int)(cus / (2 * tiles));
        if (ksplit > stages / 8) ksplit = stages / 8;   // at least 8 stages per part
        if (ksplit > 16) ksplit = 16;
    }
    if (g_ksplit >= 0) ksplit = g_ksplit;
    if (ksplit > stages) ksplit = stages;
    if (!have_workspace) ksplit = 1;
    if (ksplit >= 2) {
        p.full = 0;
        p.half = 2 * tiles;
        p.ksplit = ksplit;
        return p;
    }
    // (2) One workgroup per compute unit is resident, so a launch proceeds in rounds of `cus`
    // tiles.  When the last round would be at most half full, its tiles are done as twice
    // as many half-width tiles by a second launch, which then costs about half a round.
    const long rounds = tiles / cus, left = tiles - rounds * cus;
    long full = (left > 0 && 2 * left <= cus) ? rounds * cus : tiles;
    if (g_tile_mode == 1) full = tiles;
    if (g_tile_mode == 2) full = 0;
    p.full = full;
    p.half = 2 * (tiles - full);
    return p;
}

// Test hook: the plan for a shape on a chip of `cus` compute units (no launch, no GPU needed).
extern "C" void sqp_debug_prefill_plan(int M, int N, int K, int cus, long *full, long *half, int *ksplit)
{
    const TilePlan p = plan_tiles(M, N, K, 128, cus, true);
    *full = p.full;
    *half = p.half;
    *ksplit = p.ksplit;
}

size_t sqp_gemm_prefill_partial_bytes(int M, int N, int K, int group)
{
    if (group % BK != 0 && !(group == 32 && K % BK == 0)) return sqp_gemm_decode_partial_bytes(M < 64 ? M : 64, N, K, group);  // row-block fallback
    const TilePlan p = plan_tiles(M, N, K, group, compute_units(), true);
    return p.ksplit >= 2 ? (size_t)p.ksplit * M * N * sizeof(float) : 0;
}

template <int WM, bool G32>
static int launch_tiles(const TilePlan &p, int M, int N, int K, int group, const h16 *x, const uint32_t *packed, const h16 *scales,
                        const uint8_t *zeros, h16 *y, int epi, const SqpWorkspace &ws, hipStream_t stream)
{
    constexpr int FULLN = (4 / WM) * 128;
    const int tn = (N + FULLN - 1) / FULLN;
    if (p.ksplit >= 2) {
        if ((size_t)p.ksplit * M * N * sizeof(float) > ws.partial_bytes) return SQP_ERR_WORKSPACE;
        float *part = ws.partial;
        w4a16_prefill_kernel<2, WM, G32><<<dim3((unsigned)p.half, p.ksplit), 256, 0, stream>>>(M, N, K, group, 0, tn, x, packed, scales, zeros, y, part, epi);
        const long total8 = (long)M * N / 8;
        splitk_reduce_kernel<<<(unsigned)((total8 + 255) / 256), 256, 0, stream>>>(part, total8, (long)M * N, p.ksplit, y, epi);
        return sqp_launch_status();
    }
    if (p.full > 0)
        w4a16_prefill_kernel<4, WM, G32><<<dim3((unsigned)p.full), 256, 0, stream>>>(M, N, K, group, 0, tn, x, packed, scales, zeros, y, nullptr, epi);
    if (p.half > 0)
        w4a16_prefill_kernel<2, WM, G32><<<dim3((unsigned)p.half), 256, 0, stream>>>(M, N, K, group, (int)p.full, tn, x, packed, scales, zeros, y, nullptr, epi);
    return sqp_launch_status();
}

int sqp_gemm_prefill(int M, int N, int K, int group, const h16 *x, const uint32_t *packed,
                     const h16 *scales, const uint8_t *zeros, h16 *y, int epi, const SqpWorkspace &ws, hipStream_t stream)
{
    if (group % BK == 0 || (group == 32 && K % BK == 0)) {
        const TilePlan p = plan_tiles(M, N, K, group, compute_units(), ws.partial != nullptr);
        if (group == 32) return launch_tiles<1, true>(p, M, N, K, group, x, packed, scales, zeros, y, epi, ws, stream);  // one tile shape only
        if (p.wm == 1) return launch_tiles<1, false>(p, M, N, K, group, x, packed, scales, zeros, y, epi, ws, stream);
        return launch_tiles<2, false>(p, M, N, K, group, x, packed, scales, zeros, y, epi, ws, stream);
    }
    // group sizes the tiled kernel does not cover (neither a multiple of 64, nor 32 with K a multiple of 64)
    return decode_in_row_blocks(M, N, K, group, x, packed, scales, zeros, y, epi, ws, stream);
}

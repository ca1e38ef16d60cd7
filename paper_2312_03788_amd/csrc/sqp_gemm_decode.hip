// Weight-streaming W4A16 GEMM for small M (decode): y = x * w_hat, Eq. 3 of
// arXiv 2312.03788 with w_hat = (code - Z) * Delta of Eq. 1, group-wise along K (Sec 2.2).
//
// The kernel is bound by the HBM stream of packed weights.  Each wave owns a strip of
// 16*VW*NT output columns and a contiguous range of quantisation groups along K:
//   - one dwordx{VW} load per lane fetches, for k-block (lane / 16), the packed words of
//     VW adjacent columns: a word is 8 consecutive k of one column, which is exactly one
//     lane's B operand of v_mfma_f32_16x16x32_f16 (column = lane % 16, k-block = lane / 16);
//   - the codes become exact fp16 integers (code - Z) with 9 VALU ops per word: the
//     nibbles are OR-ed into the mantissa of 1024.0 (bits 3:0) or 64.0 (bits 7:4) and the
//     offset (1024 + Z or 64 + Z) is subtracted with a packed fp16 add, which is exact;
//   - x supplies the A operand (row = lane % 16), permuted to the same nibble order;
//   - the MFMA accumulates one group in fp32, then the group's step Delta (a per-lane
//     scalar in the 16x16 accumulator layout: column = lane % 16) scales it into the
//     running sum: sum_k x (q - Z) Delta = Delta * sum_k x (q - Z).
// The K ranges of the NW waves of a workgroup are summed through LDS in wave order; with
// SPLIT > 1 workgroups along K, fp32 partial tiles go to a workspace and the workgroup
// that arrives last (atomic ticket) adds them in split order, so the result does not
// depend on scheduling.
#include <type_traits>

#include "sqp_common.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int VW> struct WVec;
template <> struct WVec<1> { typedef uint32_t T; };
template <> struct WVec<2> { typedef uint2 T; };
template <> struct WVec<4> { typedef uint4 T; };

template <int VW> __device__ __forceinline__ uint32_t wword(const typename WVec<VW>::T &v, int c);
template <> __device__ __forceinline__ uint32_t wword<1>(const uint32_t &v, int) { return v; }
template <> __device__ __forceinline__ uint32_t wword<2>(const uint2 &v, int c) { return c ? v.y : v.x; }
template <> __device__ __forceinline__ uint32_t wword<4>(const uint4 &v, int c)
{
    return c == 0 ? v.x : (c == 1 ? v.y : (c == 2 ? v.z : v.w));
}

template <int VW> __device__ __forceinline__ typename WVec<VW>::T wzero();
template <> __device__ __forceinline__ uint32_t wzero<1>() { return 0u; }
template <> __device__ __forceinline__ uint2 wzero<2>() { return make_uint2(0u, 0u); }
template <> __device__ __forceinline__ uint4 wzero<4>() { return make_uint4(0u, 0u, 0u, 0u); }

// Constants of the nibble unpack, held in registers: v_and_or_b32 cannot take literals.
struct UnpackConsts {
    uint32_t mask_lo, mask_hi, magic_lo, magic_hi;
};

// packed word (8 codes of one column) -> 8 exact fp16 values (code - Z), in the order
// (k0,k4),(k1,k5),(k2,k6),(k3,k7).  neg_hi = -(1024 + Z), neg_lo = -(64 + Z), both halves.
// 1 shift + 4 and-or + 4 packed adds.
__device__ __forceinline__ h16x8 dequant_word(uint32_t w, h16x2 neg_hi, h16x2 neg_lo, const UnpackConsts &uc)
{
    const uint32_t w8 = w >> 8;
    uint32_t t0, t1, t2, t3;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t0) : "v"(w), "v"(uc.mask_lo), "v"(uc.magic_lo));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t1) : "v"(w), "v"(uc.mask_hi), "v"(uc.magic_hi));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t2) : "v"(w8), "v"(uc.mask_lo), "v"(uc.magic_lo));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t3) : "v"(w8), "v"(uc.mask_hi), "v"(uc.magic_hi));
    h16x2 b0 = __builtin_bit_cast(h16x2, t0) + neg_hi;
    h16x2 b1 = __builtin_bit_cast(h16x2, t1) + neg_lo;
    h16x2 b2 = __builtin_bit_cast(h16x2, t2) + neg_hi;
    h16x2 b3 = __builtin_bit_cast(h16x2, t3) + neg_lo;
    h16x8 r;
    r.s0 = b0.x; r.s1 = b0.y; r.s2 = b1.x; r.s3 = b1.y;
    r.s4 = b2.x; r.s5 = b2.y; r.s6 = b3.x; r.s7 = b3.y;
    return r;
}

// 8 consecutive-k activations (x0..x7 as four dwords) -> the nibble order above.
__device__ __forceinline__ h16x8 permute_x(const u32x4 &v)
{
    u32x4 p;
    p.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);  // (x0, x4)
    p.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);  // (x1, x5)
    p.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);  // (x2, x6)
    p.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);  // (x3, x7)
    return __builtin_bit_cast(h16x8, p);
}

struct Workspace {
    float *partial;      // [tiles][SPLIT][tile floats]
    unsigned *tickets;   // [tiles], zero between launches
};

// MT: 16-row tiles of x (M <= 16*MT).  VW: packed words per lane per load.  NT: loads per
// k-step (strip width 16*VW*NT).  NW: waves per workgroup.  KSPG: k-steps (of 32) per
// chunk; a quantisation group is cpg chunks (cpg = 1 unless the group is a multiple of
// 128 above 128).  D: register stages of packed weights (groups in flight + 1).
// XD: LDS stages of activations per wave.
template <int MT, int VW, int NT, int NW, int KSPG, int D, int XD>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(MT * NT == 1 ? 3 : 1)))
w4a16_decode_kernel(int M, int N, int K, int cpg, const h16 *__restrict__ x, const uint32_t *__restrict__ packed,
                    const h16 *__restrict__ scales, const uint8_t *__restrict__ zeros, h16 *__restrict__ y,
                    Workspace ws)
{
    typedef typename WVec<VW>::T wvec;
    constexpr int NTILE = NT * VW;        // 16x16 accumulator tiles per m-tile
    constexpr int REGS = MT * NTILE * 4;  // fp32 accumulator registers per lane
    constexpr int BN = 16 * VW * NT;      // strip width
    // Activations reach the matrix cores through a per-wave LDS ring filled by direct
    // global->LDS loads (no registers held while they are in flight); the same LDS is
    // reused for the cross-wave sum at the end.
    constexpr int XSTAGE = KSPG * MT * 1024;  // bytes: one group of x for this wave
    constexpr int XRING = XD * XSTAGE;
    constexpr int RED_BYTES = NW * REGS * 64 * 4;
    constexpr int SMEM = NW * XRING > RED_BYTES ? NW * XRING : RED_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
    __shared__ unsigned ticket_s;
    float(*red)[REGS][64] = reinterpret_cast<float(*)[REGS][64]>(smem);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform, kept scalar
    const int lc = lane & 15, lk = lane >> 4;
    const int n0 = blockIdx.x * BN;
    const int split = gridDim.y, sidx = blockIdx.y;
    const int groups = K / (32 * KSPG);
    // this workgroup's group range, then this wave's share of it
    const int gb0 = (int)((long)groups * sidx / split), gb1 = (int)((long)groups * (sidx + 1) / split);
    const int g0 = gb0 + (gb1 - gb0) * wave / NW, g1 = gb0 + (gb1 - gb0) * (wave + 1) / NW;
    unsigned char *xring = smem + wave * XRING;

    // lanes past the last column read column 0 instead; their results are never stored
    int ncol[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        ncol[nt] = n0 + nt * 16 * VW + VW * lc;
        if (ncol[nt] >= N) ncol[nt] = 0;
    }
    const h16 *xsrc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        int m = mt * 16 + lc;
        m = m < M ? m : M - 1;
        xsrc[mt] = x + (size_t)m * K + lk * 8;
    }

    f32x4 acc[MT][NTILE];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int t = 0; t < NTILE; t++) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    const UnpackConsts uc = {0x000f000fu, 0x00f000f0u, 0x64006400u, 0x54005400u};

    static_assert(VW == 4, "one dwordx4 of packed words per lane");
    struct Stage {
        u32x4 w[KSPG][NT];
        u32x2 sc[NT];     // 4 fp16 steps
        uint32_t zr[NT];  // 4 zero points, one byte each
    };

    // The weight, step and zero-point loads are written in assembly so that this kernel, not
    // the compiler, decides when to wait for them: the registers of a stage must not be read
    // before the s_waitcnt issued by `landed` below.
    // Addresses are a scalar base (advanced on the scalar unit) plus a per-lane 32-bit offset
    // that never changes, so the loads cost no vector arithmetic.
    const uint32_t voff_w = (uint32_t)(lk * N + 0) * 4u;  // + column, below
    uint32_t voff_wn[NT], voff_sn[NT], voff_zn[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        voff_wn[nt] = voff_w + (uint32_t)ncol[nt] * 4u;
        voff_sn[nt] = (uint32_t)ncol[nt] * 2u;
        voff_zn[nt] = (uint32_t)ncol[nt];
    }
    auto issue_w = [&](Stage &s, int g) {
#pragma unroll
        for (int ks = 0; ks < KSPG; ks++) {
            const uint32_t *base = packed + (size_t)(g * KSPG + ks) * 4 * N;  // wave-uniform
#pragma unroll
            for (int nt = 0; nt < NT; nt++)
                asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(s.w[ks][nt]) : "v"(voff_wn[nt]), "s"(base) : "memory");
        }
        const int gs = g / cpg;  // quantisation group of this chunk
        const h16 *sbase = scales + (size_t)gs * N;
        const uint8_t *zbase = zeros + (size_t)gs * N;
#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
            asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(s.sc[nt]) : "v"(voff_sn[nt]), "s"(sbase) : "memory");
            asm volatile("global_load_dword %0, %1, %2" : "=v"(s.zr[nt]) : "v"(voff_zn[nt]), "s"(zbase) : "memory");
        }
    };
    // wait until at most `AFTER` loads are outstanding, then tie the stage's registers to the
    // wait so that no use of them is scheduled ahead of it
    auto landed = [&](Stage &s, auto after) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(decltype(after)::value) : "memory");
#pragma unroll
        for (int ks = 0; ks < KSPG; ks++)
#pragma unroll
            for (int nt = 0; nt < NT; nt++) asm volatile("" : "+v"(s.w[ks][nt]));
#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
            asm volatile("" : "+v"(s.sc[nt]));
            asm volatile("" : "+v"(s.zr[nt]));
        }
    };

    // lane (row lc, k-block lk) copies its 16 bytes of x straight into LDS; the hardware
    // places lane i at byte 16*i of the destination block, which is where it reads them back.
    auto issue_x = [&](int slot, int g) {
#pragma unroll
        for (int ks = 0; ks < KSPG; ks++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const h16 *src = xsrc[mt] + (size_t)(g * KSPG + ks) * 32;
                unsigned char *dst = xring + slot * XSTAGE + (ks * MT + mt) * 1024;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                 (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
            }
    };

    auto compute = [&](const Stage &s, int slot, bool live) {
        f32x4 accg[MT][NTILE];
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int t = 0; t < NTILE; t++) accg[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        h16x2 neg_hi[NTILE], neg_lo[NTILE];
        float delta[NTILE];
#pragma unroll
        for (int nt = 0; nt < NT; nt++)
#pragma unroll
            for (int c = 0; c < VW; c++) {
                // fp16 bit patterns: 1024 + Z is 0x6400 + Z and 64 + Z is 0x5400 + 16 Z (Z <= 15);
                // with the sign bit, replicated into both halves
                const uint32_t z = (s.zr[nt] >> (8 * c)) & 0xffu;
                neg_hi[nt * VW + c] = __builtin_bit_cast(h16x2, z * 0x00010001u + 0xe400e400u);
                neg_lo[nt * VW + c] = __builtin_bit_cast(h16x2, z * 0x00100010u + 0xd400d400u);
                const uint32_t sw = s.sc[nt][c >> 1];
                const h16x2 sv = __builtin_bit_cast(h16x2, sw);
                delta[nt * VW + c] = live ? (float)((c & 1) ? sv.y : sv.x) : 0.f;
            }
        // The x fragments of the whole group come out of the LDS ring in one go.  The reads
        // are written in assembly because the compiler cannot tell which ring slot a direct
        // global->LDS load filled and would otherwise wait for every outstanding load; the
        // caller has already waited for exactly the loads that filled this slot.
        const unsigned xs = (unsigned)(size_t)(xring + slot * XSTAGE + lane * 16);
        constexpr int XB = MT == 1 ? KSPG : 1;  // k-steps fetched from LDS per batch
#pragma unroll
        for (int kb = 0; kb < KSPG; kb += XB) {
            u32x4 xa[XB * MT];
#pragma unroll
            for (int i = 0; i < XB * MT; i++)
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(xa[i]) : "v"(xs), "n"((kb * MT + i) * 1024) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < XB * MT; i++) asm volatile("" : "+v"(xa[i]));  // no use ahead of the wait
#pragma unroll
            for (int kk = 0; kk < XB; kk++) {
                const int ks = kb + kk;
                h16x8 a[MT];
#pragma unroll
                for (int mt = 0; mt < MT; mt++) a[mt] = permute_x(xa[kk * MT + mt]);
#pragma unroll
                for (int nt = 0; nt < NT; nt++)
#pragma unroll
                    for (int c = 0; c < VW; c++) {
                        const int t = nt * VW + c;
                        const h16x8 b = dequant_word(s.w[ks][nt][c], neg_hi[t], neg_lo[t], uc);
#pragma unroll
                        for (int mt = 0; mt < MT; mt++)
                            accg[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], b, accg[mt][t], 0, 0, 0);
                    }
            }
        }
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int t = 0; t < NTILE; t++)
#pragma unroll
                for (int r = 0; r < 4; r++) acc[mt][t][r] = fmaf(delta[t], accg[mt][t][r], acc[mt][t][r]);
    };

    // Software pipeline over this wave's groups.  Iteration g issues x(g+1) into the other
    // LDS slot, then the packed weights of group g+D-1 into the register stage that has just
    // been freed (stage index static: the loop is unrolled by D), then consumes group g.  The
    // pipeline is primed by running the issue part of iterations g0-(D-1) .. g0-1.
    // The loop body is free of branches: the group count is rounded up to a multiple of D,
    // loads past the wave's range are clamped to a valid group (they hit data a neighbour
    // streams anyway) and such groups enter the sum with a step of 0.  Every iteration thus
    // issues the same number of loads, and since loads complete in issue order "x(g) has
    // landed" is "at most 2*OW + OX loads are still outstanding" (those issued behind it).
    constexpr int OW = KSPG * NT + 2 * NT, OX = KSPG * MT;
    static_assert(XD == 2, "the x ring is double buffered");
    static_assert(2 * OW + OX < 64, "vmcnt field");
    static_assert(D >= 3, "x(g) must be issued behind w(g)");
    auto gc = [&](int g) { return g < groups ? g : groups - 1; };
    Stage st[D];
#pragma unroll
    for (int j = 0; j < D - 1; j++) {
        if (j == D - 2) issue_x(0, gc(g0));
        issue_w(st[j], gc(g0 + j));
    }
    int xslot = 0;
    const int nblk = (g1 - g0 + D - 1) / D;
    for (int b = 0; b < nblk; b++) {
        const int g = g0 + b * D;
#pragma unroll
        for (int d = 0; d < D; d++) {
            const int gg = g + d;
            issue_x(xslot ^ 1, gc(gg + 1));
            issue_w(st[(d + D - 1) % D], gc(gg + D - 1));
            landed(st[d], std::integral_constant<int, 2 * OW + OX>());
            compute(st[d], xslot, gg < g1);
            xslot ^= 1;
        }
    }
    // Drain the clamped look-ahead loads.  Their destination registers are dead by now as far
    // as the compiler can tell, but the hardware still writes them when the data arrives: the
    // empty uses below keep every stage allocated until the wait has completed, so that
    // nothing else is placed in those registers while a load is in flight.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int j = 0; j < D; j++) {
#pragma unroll
        for (int ks = 0; ks < KSPG; ks++)
#pragma unroll
            for (int nt = 0; nt < NT; nt++) asm volatile("" ::"v"(st[j].w[ks][nt]));
#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
            asm volatile("" ::"v"(st[j].sc[nt]));
            asm volatile("" ::"v"(st[j].zr[nt]));
        }
    }
    __syncthreads();  // every wave is done with its x ring before the LDS is reused

    // ---- sum the NW waves' K ranges through LDS, in wave order
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int t = 0; t < NTILE; t++)
#pragma unroll
            for (int r = 0; r < 4; r++) red[wave][(mt * NTILE + t) * 4 + r][lane] = acc[mt][t][r];
    __syncthreads();

    // output item e = (mt, nt, r, lane): VW adjacent columns of one row
    constexpr int ITEMS = MT * NT * 4 * 64;
    constexpr int TILE_FLOATS = ITEMS * VW;
    const int tile = blockIdx.x;
    float *mypart = ws.partial ? ws.partial + ((size_t)tile * split + sidx) * TILE_FLOATS : nullptr;

    for (int e = threadIdx.x; e < ITEMS; e += NW * 64) {
        const int l = e & 63, r = (e >> 6) & 3, nt = (e >> 8) % NT, mt = (e >> 8) / NT;
        float v[VW];
#pragma unroll
        for (int c = 0; c < VW; c++) {
            const int reg = (mt * NTILE + nt * VW + c) * 4 + r;
            float sum = red[0][reg][l];
#pragma unroll
            for (int w = 1; w < NW; w++) sum += red[w][reg][l];
            v[c] = sum;
        }
        if (split == 1) {
            const int m = mt * 16 + 4 * (l >> 4) + r;
            const int n = n0 + nt * 16 * VW + VW * (l & 15);
            if (m < M && n < N) {
                h16 *dst = y + (size_t)m * N + n;
#pragma unroll
                for (int c = 0; c < VW; c++) dst[c] = (h16)v[c];
            }
        } else {
#pragma unroll
            for (int c = 0; c < VW; c++)
                __hip_atomic_store(mypart + (size_t)e * VW + c, v[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (split == 1) return;

    // ---- cross-workgroup: the last arrival adds the SPLIT partial tiles in split order.
    // Partials travel as device-scope relaxed atomic stores/loads (written through and read
    // past the per-XCD L2), so no cache-wide write-back or invalidate is needed: each thread
    // waits for its own stores to complete, the barrier collects the workgroup, and only then
    // is the ticket taken.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (threadIdx.x == 0) ticket_s = __hip_atomic_fetch_add(&ws.tickets[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (ticket_s != (unsigned)(split - 1)) return;
    const float *base = ws.partial + (size_t)tile * split * TILE_FLOATS;
    for (int e = threadIdx.x; e < ITEMS; e += NW * 64) {
        const int l = e & 63, r = (e >> 6) & 3, nt = (e >> 8) % NT, mt = (e >> 8) / NT;
        float v[VW];
#pragma unroll
        for (int c = 0; c < VW; c++) v[c] = 0.f;
        for (int s = 0; s < split; s++)
#pragma unroll
            for (int c = 0; c < VW; c++)
                v[c] += __hip_atomic_load(base + (size_t)s * TILE_FLOATS + (size_t)e * VW + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int m = mt * 16 + 4 * (l >> 4) + r;
        const int n = n0 + nt * 16 * VW + VW * (l & 15);
        if (m < M && n < N) {
            h16 *dst = y + (size_t)m * N + n;
#pragma unroll
            for (int c = 0; c < VW; c++) dst[c] = (h16)v[c];
        }
    }
    if (threadIdx.x == 0)  // ready for the next launch on this stream
        __hip_atomic_store(&ws.tickets[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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

// ---------------------------------------------------------------- workspace

constexpr size_t WS_PARTIAL_BYTES = 64u << 20;
constexpr int WS_TICKETS = 1 << 16;
Workspace g_ws[16] = {};

__global__ void zero_tickets_kernel(unsigned *t, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) t[i] = 0u;
}

int get_workspace(Workspace *out, hipStream_t st)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return SQP_ERR_WORKSPACE;
    if (!g_ws[dev].partial) {
        void *p = nullptr, *t = nullptr;
        if (hipMalloc(&p, WS_PARTIAL_BYTES) != hipSuccess) return SQP_ERR_WORKSPACE;
        if (hipMalloc(&t, WS_TICKETS * sizeof(unsigned)) != hipSuccess) {
            (void)hipFree(p);
            return SQP_ERR_WORKSPACE;
        }
        zero_tickets_kernel<<<WS_TICKETS / 256, 256, 0, st>>>((unsigned *)t, WS_TICKETS);
        g_ws[dev].partial = (float *)p;
        g_ws[dev].tickets = (unsigned *)t;
    }
    *out = g_ws[dev];
    return SQP_OK;
}

template <int MT, int VW, int NT, int NW, int KSPG, int D = 3, int XD = 2>
int launch(int M, int N, int K, int cpg, int split, const h16 *x, const uint32_t *packed, const h16 *scales,
           const uint8_t *zeros, h16 *y, hipStream_t st)
{
    constexpr int BN = 16 * VW * NT;
    const int tiles = (N + BN - 1) / BN;
    Workspace ws = {nullptr, nullptr};
    if (split > 1) {
        const size_t tile_bytes = (size_t)MT * NT * 4 * 64 * VW * sizeof(float);
        if (tiles > WS_TICKETS || (size_t)tiles * split * tile_bytes > WS_PARTIAL_BYTES) split = 1;
    }
    if (split > 1) {
        int rc = get_workspace(&ws, st);
        if (rc) return rc;
    }
    w4a16_decode_kernel<MT, VW, NT, NW, KSPG, D, XD><<<dim3(tiles, split), NW * 64, 0, st>>>(M, N, K, cpg, x, packed, scales, zeros, y, ws);
    return sqp_launch_status();
}

struct Plan {
    int vw, nt, nw, split;
};

// Pick strip width, waves per workgroup and K split so that the grid fills 256 compute
// units several times over while every wave still streams a few groups.
Plan make_plan(int M, int N, int K, int group)
{
    const int groups = K / group;
    Plan p;
    p.vw = 4;
    p.nt = 1;
    p.nw = 4;
    p.split = 1;
    const int tiles = (N + 63) / 64;
    // target about 8 waves per compute unit in flight
    int want = (2048 + tiles * p.nw - 1) / (tiles * p.nw);
    int max_split = groups / (p.nw * 2);
    if (max_split < 1) max_split = 1;
    if (want > max_split) want = max_split;
    if (want > 16) want = 16;
    if (want < 1) want = 1;
    p.split = want;
    (void)M;
    return p;
}

#define SQP_TRY(VW_, NT_, NW_)                                   \
    if (p.vw == VW_ && p.nt == NT_ && p.nw == NW_)               \
        return launch<MT, VW_, NT_, NW_, KSPG>(M, N, K, cpg, p.split, x, packed, scales, zeros, y, st);

template <int MT, int KSPG>
int dispatch_mt(const Plan &p, int M, int N, int K, int cpg, const h16 *x, const uint32_t *packed, const h16 *scales,
                const uint8_t *zeros, h16 *y, hipStream_t st)
{
    if constexpr (KSPG == 4 && MT == 1) {
        SQP_TRY(4, 1, 2)
        SQP_TRY(4, 1, 8)
        SQP_TRY(4, 2, 4)
    }
    return launch<MT, 4, 1, 4, KSPG>(M, N, K, cpg, p.split, x, packed, scales, zeros, y, st);
}
#undef SQP_TRY

template <int KSPG>
int dispatch_kspg(const Plan &p, int M, int N, int K, int cpg, const h16 *x, const uint32_t *packed, const h16 *scales,
                  const uint8_t *zeros, h16 *y, hipStream_t st)
{
    if (M <= 16) return dispatch_mt<1, KSPG>(p, M, N, K, cpg, x, packed, scales, zeros, y, st);
    if (M <= 32) return dispatch_mt<2, KSPG>(p, M, N, K, cpg, x, packed, scales, zeros, y, st);
    return dispatch_mt<4, KSPG>(p, M, N, K, cpg, x, packed, scales, zeros, y, st);
}

}  // namespace

// Test/benchmark hooks: force the K split, or the whole launch plan (0 = automatic).
static int g_force_split = 0;
static Plan g_force_plan = {0, 0, 0, 0};
extern "C" void sqp_debug_set_decode_split(int split) { g_force_split = split; }
extern "C" void sqp_debug_set_decode_plan(int vw, int nt, int nw, int split)
{
    g_force_plan = Plan{vw, nt, nw, split};
}

int sqp_gemm_generic(int M, int N, int K, int group, const h16 *x, const uint32_t *packed, const h16 *scales,
                     const uint8_t *zeros, h16 *y, hipStream_t stream)
{
    if (M > 65535) return SQP_ERR_SHAPE;
    w4a16_generic_kernel<<<dim3((N + 255) / 256, M), 256, 0, stream>>>(M, N, K, group, x, packed, scales, zeros, y);
    return sqp_launch_status();
}

int sqp_gemm_decode(int M, int N, int K, int group, const h16 *x, const uint32_t *packed, const h16 *scales,
                    const uint8_t *zeros, h16 *y, hipStream_t stream)
{
    Plan p = make_plan(M, N, K, group);
    if (g_force_plan.vw > 0) p = g_force_plan;
    if (p.split > K / group) p.split = K / group;
    if (g_force_split > 0) {
        p.split = g_force_split;
        if (p.split > K / group) p.split = K / group;
    }
    if (group == 32) return dispatch_kspg<1>(p, M, N, K, 1, x, packed, scales, zeros, y, stream);
    if (group == 64) return dispatch_kspg<2>(p, M, N, K, 1, x, packed, scales, zeros, y, stream);
    if (group % 128 == 0) return dispatch_kspg<4>(p, M, N, K, group / 128, x, packed, scales, zeros, y, stream);
    return sqp_gemm_generic(M, N, K, group, x, packed, scales, zeros, y, stream);
}

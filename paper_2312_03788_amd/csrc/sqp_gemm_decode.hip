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
#include "sqp_common.h"

namespace {

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

// packed word (8 codes of one column) -> 8 exact fp16 values (code - Z), in the order
// (k0,k4),(k1,k5),(k2,k6),(k3,k7).  neg_hi = -(1024 + Z), neg_lo = -(64 + Z), both halves.
__device__ __forceinline__ h16x8 dequant_word(uint32_t w, h16x2 neg_hi, h16x2 neg_lo)
{
    const uint32_t w8 = w >> 8;
    uint32_t t0 = (w & 0x000f000fu) | 0x64006400u;
    uint32_t t1 = (w & 0x00f000f0u) | 0x54005400u;
    uint32_t t2 = (w8 & 0x000f000fu) | 0x64006400u;
    uint32_t t3 = (w8 & 0x00f000f0u) | 0x54005400u;
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
__device__ __forceinline__ h16x8 permute_x(const uint4 &v)
{
    uint4 p;
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
// quantisation group.
template <int MT, int VW, int NT, int NW, int KSPG>
__global__ void __launch_bounds__(NW * 64)
w4a16_decode_kernel(int M, int N, int K, const h16 *__restrict__ x, const uint32_t *__restrict__ packed,
                    const h16 *__restrict__ scales, const uint8_t *__restrict__ zeros, h16 *__restrict__ y,
                    Workspace ws)
{
    typedef typename WVec<VW>::T wvec;
    constexpr int NTILE = NT * VW;        // 16x16 accumulator tiles per m-tile
    constexpr int REGS = MT * NTILE * 4;  // fp32 accumulator registers per lane
    constexpr int BN = 16 * VW * NT;      // strip width
    __shared__ float red[NW][REGS][64];
    __shared__ unsigned ticket_s;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lc = lane & 15, lk = lane >> 4;
    const int n0 = blockIdx.x * BN;
    const int split = gridDim.y, sidx = blockIdx.y;
    const int groups = K / (32 * KSPG);
    // this workgroup's group range, then this wave's share of it
    const int gb0 = (int)((long)groups * sidx / split), gb1 = (int)((long)groups * (sidx + 1) / split);
    const int g0 = gb0 + (gb1 - gb0) * wave / NW, g1 = gb0 + (gb1 - gb0) * (wave + 1) / NW;

    int ncol[NT];
    bool nok[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        ncol[nt] = n0 + nt * 16 * VW + VW * lc;
        nok[nt] = ncol[nt] < N;
        if (!nok[nt]) ncol[nt] = 0;
    }
    int xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        int m = mt * 16 + lc;
        xrow[mt] = m < M ? m : M - 1;
    }

    f32x4 acc[MT][NTILE];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int t = 0; t < NTILE; t++) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    struct Stage {
        wvec w[KSPG][NT];
        uint4 xa[KSPG][MT];
        uint32_t sc[NT][(VW + 1) / 2];  // VW fp16 steps
        uint32_t zr[NT];                // VW zero points, one byte each
    };

    auto issue = [&](Stage &s, int g) {
#pragma unroll
        for (int ks = 0; ks < KSPG; ks++) {
            const int row = (g * KSPG + ks) * 4 + lk;  // packed row = k / 8
#pragma unroll
            for (int nt = 0; nt < NT; nt++)
                s.w[ks][nt] = nok[nt] ? *reinterpret_cast<const wvec *>(packed + (size_t)row * N + ncol[nt]) : wzero<VW>();
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
                s.xa[ks][mt] = *reinterpret_cast<const uint4 *>(x + (size_t)xrow[mt] * K + (size_t)row * 8);
        }
#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
            const h16 *sp = scales + (size_t)g * N + ncol[nt];
            const uint8_t *zp = zeros + (size_t)g * N + ncol[nt];
            if (VW == 4) {
                uint2 v = *reinterpret_cast<const uint2 *>(sp);
                s.sc[nt][0] = v.x;
                s.sc[nt][(VW + 1) / 2 - 1] = v.y;
                s.zr[nt] = *reinterpret_cast<const uint32_t *>(zp);
            } else if (VW == 2) {
                s.sc[nt][0] = *reinterpret_cast<const uint32_t *>(sp);
                s.zr[nt] = *reinterpret_cast<const uint16_t *>(zp);
            } else {
                s.sc[nt][0] = *reinterpret_cast<const uint16_t *>(sp);
                s.zr[nt] = *zp;
            }
        }
    };

    auto compute = [&](const Stage &s) {
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
                const int z = (int)((s.zr[nt] >> (8 * c)) & 0xffu);
                const h16 zh = (h16)(float)z;  // exact
                const h16 a = (h16)(-1024.0f) - zh, b = (h16)(-64.0f) - zh;
                neg_hi[nt * VW + c] = h16x2{a, a};
                neg_lo[nt * VW + c] = h16x2{b, b};
                const uint32_t sw = s.sc[nt][c >> 1];
                const h16x2 sv = __builtin_bit_cast(h16x2, sw);
                delta[nt * VW + c] = (float)((c & 1) ? sv.y : sv.x);
            }
#pragma unroll
        for (int ks = 0; ks < KSPG; ks++) {
            h16x8 a[MT];
#pragma unroll
            for (int mt = 0; mt < MT; mt++) a[mt] = permute_x(s.xa[ks][mt]);
#pragma unroll
            for (int nt = 0; nt < NT; nt++)
#pragma unroll
                for (int c = 0; c < VW; c++) {
                    const int t = nt * VW + c;
                    const h16x8 b = dequant_word(wword<VW>(s.w[ks][nt], c), neg_hi[t], neg_lo[t]);
#pragma unroll
                    for (int mt = 0; mt < MT; mt++)
                        accg[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], b, accg[mt][t], 0, 0, 0);
                }
        }
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int t = 0; t < NTILE; t++)
#pragma unroll
                for (int r = 0; r < 4; r++) acc[mt][t][r] = fmaf(delta[t], accg[mt][t][r], acc[mt][t][r]);
    };

    Stage sa, sb;
    if (g0 < g1) issue(sa, g0);
    for (int g = g0; g < g1; g += 2) {
        if (g + 1 < g1) issue(sb, g + 1);
        compute(sa);
        if (g + 1 < g1) {
            if (g + 2 < g1) issue(sa, g + 2);
            compute(sb);
        }
    }

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
            for (int c = 0; c < VW; c++) mypart[(size_t)e * VW + c] = v[c];
        }
    }
    if (split == 1) return;

    // ---- cross-workgroup: the last arrival adds the SPLIT partial tiles in split order
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) ticket_s = atomicAdd(&ws.tickets[tile], 1u);
    __syncthreads();
    if (ticket_s != (unsigned)(split - 1)) return;
    __threadfence();
    const float *base = ws.partial + (size_t)tile * split * TILE_FLOATS;
    for (int e = threadIdx.x; e < ITEMS; e += NW * 64) {
        const int l = e & 63, r = (e >> 6) & 3, nt = (e >> 8) % NT, mt = (e >> 8) / NT;
        float v[VW];
#pragma unroll
        for (int c = 0; c < VW; c++) v[c] = 0.f;
        for (int s = 0; s < split; s++)
#pragma unroll
            for (int c = 0; c < VW; c++) v[c] += __builtin_nontemporal_load(base + (size_t)s * TILE_FLOATS + (size_t)e * VW + c);
        const int m = mt * 16 + 4 * (l >> 4) + r;
        const int n = n0 + nt * 16 * VW + VW * (l & 15);
        if (m < M && n < N) {
            h16 *dst = y + (size_t)m * N + n;
#pragma unroll
            for (int c = 0; c < VW; c++) dst[c] = (h16)v[c];
        }
    }
    if (threadIdx.x == 0) ws.tickets[tile] = 0u;  // ready for the next launch on this stream
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

template <int MT, int VW, int NT, int NW, int KSPG>
int launch(int M, int N, int K, int split, const h16 *x, const uint32_t *packed, const h16 *scales,
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
    w4a16_decode_kernel<MT, VW, NT, NW, KSPG><<<dim3(tiles, split), NW * 64, 0, st>>>(M, N, K, x, packed, scales, zeros, y, ws);
    return sqp_launch_status();
}

struct Plan {
    int vw, nw, split;
};

// Pick strip width, waves per workgroup and K split so that the grid fills 256 compute
// units several times over while every wave still streams a few groups.
Plan make_plan(int M, int N, int K, int group)
{
    const int groups = K / group;
    Plan p;
    p.vw = 4;
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

template <int MT, int KSPG>
int dispatch_mt(const Plan &p, int M, int N, int K, const h16 *x, const uint32_t *packed, const h16 *scales,
                const uint8_t *zeros, h16 *y, hipStream_t st)
{
    return launch<MT, 4, 1, 4, KSPG>(M, N, K, p.split, x, packed, scales, zeros, y, st);
}

template <int KSPG>
int dispatch_kspg(const Plan &p, int M, int N, int K, const h16 *x, const uint32_t *packed, const h16 *scales,
                  const uint8_t *zeros, h16 *y, hipStream_t st)
{
    if (M <= 16) return dispatch_mt<1, KSPG>(p, M, N, K, x, packed, scales, zeros, y, st);
    if (M <= 32) return dispatch_mt<2, KSPG>(p, M, N, K, x, packed, scales, zeros, y, st);
    return dispatch_mt<4, KSPG>(p, M, N, K, x, packed, scales, zeros, y, st);
}

}  // namespace

// Test/benchmark hook: force the K split (0 = automatic).
static int g_force_split = 0;
extern "C" void sqp_debug_set_decode_split(int split) { g_force_split = split; }

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
    if (g_force_split > 0) {
        p.split = g_force_split;
        if (p.split > K / group) p.split = K / group;
    }
    switch (group) {
        case 32: return dispatch_kspg<1>(p, M, N, K, x, packed, scales, zeros, y, stream);
        case 64: return dispatch_kspg<2>(p, M, N, K, x, packed, scales, zeros, y, stream);
        case 128: return dispatch_kspg<4>(p, M, N, K, x, packed, scales, zeros, y, stream);
        case 256: return dispatch_kspg<8>(p, M, N, K, x, packed, scales, zeros, y, stream);
        default: return sqp_gemm_generic(M, N, K, group, x, packed, scales, zeros, y, stream);
    }
}

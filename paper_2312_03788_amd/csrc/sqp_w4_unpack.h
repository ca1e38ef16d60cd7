// Device helpers shared by the W4A16 GEMM kernels: 4-bit code unpack and the matching
// permutation of activations (Eq. 1 of arXiv 2312.03788, second line: (code - Z) * Delta).
#pragma once
#include "sqp_common.h"

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Constants of the nibble unpack, held in registers: v_and_or_b32 cannot take literals.
struct UnpackConsts {
    uint32_t mask_lo, mask_hi, magic_lo, magic_hi;
};
#define SQP_UNPACK_CONSTS {0x000f000fu, 0x00f000f0u, 0x64006400u, 0x54005400u}

// fp16 bit patterns of -(1024 + Z) and -(64 + Z), replicated into both halves:
// 1024 + Z is 0x6400 + Z and 64 + Z is 0x5400 + 16 Z for Z <= 15.
__device__ __forceinline__ h16x2 neg_hi_of(uint32_t z) { return __builtin_bit_cast(h16x2, z * 0x00010001u + 0xe400e400u); }
__device__ __forceinline__ h16x2 neg_lo_of(uint32_t z) { return __builtin_bit_cast(h16x2, z * 0x00100010u + 0xd400d400u); }

// packed word (8 codes of one column) -> 8 exact fp16 values (code - Z), in the order
// (k0,k4),(k1,k5),(k2,k6),(k3,k7): the nibbles are OR-ed into the mantissa of 1024.0
// (bits 3:0) or 64.0 (bits 7:4) and the offset is removed by an exact packed fp16 add.
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

// The same, times the step: the fp16 dequantised weights w_hat = fp16((code - Z) * Delta)
// themselves (one rounding, as Eq. 1 defines them).  4 more packed multiplies.
__device__ __forceinline__ h16x8 dequant_word_scaled(uint32_t w, h16x2 neg_hi, h16x2 neg_lo, h16x2 delta, const UnpackConsts &uc)
{
    const uint32_t w8 = w >> 8;
    uint32_t t0, t1, t2, t3;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t0) : "v"(w), "v"(uc.mask_lo), "v"(uc.magic_lo));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t1) : "v"(w), "v"(uc.mask_hi), "v"(uc.magic_hi));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t2) : "v"(w8), "v"(uc.mask_lo), "v"(uc.magic_lo));
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t3) : "v"(w8), "v"(uc.mask_hi), "v"(uc.magic_hi));
    h16x2 b0 = (__builtin_bit_cast(h16x2, t0) + neg_hi) * delta;
    h16x2 b1 = (__builtin_bit_cast(h16x2, t1) + neg_lo) * delta;
    h16x2 b2 = (__builtin_bit_cast(h16x2, t2) + neg_hi) * delta;
    h16x2 b3 = (__builtin_bit_cast(h16x2, t3) + neg_lo) * delta;
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

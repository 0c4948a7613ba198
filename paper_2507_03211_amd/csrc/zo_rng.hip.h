// Device-side random direction z (DistZO2, Eq. 1: z ~ N(0, I); App. A Alg. 1: every pass of a
// step re-draws the same z from the step's seed).
//
// z is addressed, not streamed: element i of tensor t under seed s is a pure function of
// (s, t, i), so "reset the generator to seed s" costs nothing and any kernel can regenerate
// exactly the values another one used.  Generator: Philox4x32-10 (Salmon et al., SC'11), one
// block per four consecutive elements.  Transform: pair-wise Box-Muller whose fp32 arithmetic
// is fixed operation by operation (only IEEE conversions, mul, fma, sqrt, integer ops and one
// lookup in a 512-entry table of fp32 constants), so the bits are the same on any IEEE-754
// machine.  Must be compiled with -ffp-contract=off.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "zo_ln_table.hip.h"

namespace zo {

struct u32x4 { uint32_t x, y, z, w; };

// a ^ b ^ k in one instruction (three-input bit operation, truth table 0x96); k is wave-uniform.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t k)
{
    uint32_t r;
    asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x96" : "=v"(r) : "v"(a), "v"(b), "s"(k));
    return r;
}

// (a & m) | o in one instruction; m and o are wave-uniform constants.
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t m, uint32_t o)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(m), "v"(o));
    return r;
}
// Bits of `a` where the wave-uniform mask m is set, bits of `b` elsewhere, in one instruction.
__device__ __forceinline__ uint32_t bit_select(uint32_t m, uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "s"(m), "v"(a), "v"(b));
    return r;
}

// Ten Philox-4x32 rounds.  One round maps (c0,c1,c2,c3) to
// (hi(B*c2)^c1^k0, lo(B*c2), hi(A*c0)^c3^k1, lo(A*c0)); the key advances by a Weyl step per round.
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1)
{
    constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
    constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t pa = (uint64_t)kMulA * c0;
        const uint64_t pb = (uint64_t)kMulB * c2;
        const uint32_t n0 = xor3((uint32_t)(pb >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(pa >> 32), c3, k1);
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
        k0 += kWeylA;
        k1 += kWeylB;
    }
    return u32x4{c0, c1, c2, c3};
}

// Words for elements 4j .. 4j+3 of tensor `tid`; tag 0 is the direction z.
__device__ __forceinline__ u32x4 philox_block(uint64_t seed, uint32_t tid, uint64_t j, uint32_t tag = 0u)
{
    return philox4x32_10((uint32_t)j, (uint32_t)(j >> 32), tid, tag, (uint32_t)seed, (uint32_t)(seed >> 32));
}

// Correctly rounded square root for the arguments the radius takes (t = -2 ln u with u = k 2^-24, k odd: 1.19e-7
// <= t <= 33.3, so no scaling for subnormals or huge values is needed, which is what makes the compiler's
// general sequence long): reciprocal square root estimate y, one Newton step for g = sqrt(t), and a final
// correction from the exact residual t - g^2 with the unrefined y/2 as 1/(2 sqrt(t)) (its error is far below
// what the correction can see).  Checked against the IEEE result for every one of the 2^23 arguments that can
// occur.
__device__ __forceinline__ float sqrt_rn(float t)
{
    const float y = __builtin_amdgcn_rsqf(t);
    float g = t * y;
    const float h = 0.5f * y;
    const float r = __builtin_fmaf(-h, g, 0.5f);
    g = __builtin_fmaf(g, r, g);
    const float d = __builtin_fmaf(-g, g, t);
    return __builtin_fmaf(d, h, g);
}

// The logarithm's pivot table in LDS: 512 {inv_i, l_i} pairs, 4 KiB.  Every kernel that draws normals copies it
// from constant memory once per workgroup (256 threads x 16 bytes) and synchronises before the first draw.
constexpr int kLnPivots = 512;
__device__ __forceinline__ void load_ln_pivots(float2 *tab /* LDS, kLnPivots entries */)
{
    for (int i = threadIdx.x; i < kLnPivots / 2; i += blockDim.x)
        ((float4 *)tab)[i] = ((const float4 *)kLnPivot)[i];
    __syncthreads();
}

// Two standard normals from two words.
//   radius  u = (2 (ra >> 9) + 1) 2^-24 in (0,1), rho = sqrt(-2 ln u)
//   angle   x = (float)(int32)rb 2^-31 in [-1, 1], a quarter turn either way
//   z1 = rho sin(pi x / 2);  z0 = -+rho cos(pi x / 2), negative when bit 8 of ra is set.
// The logarithm: uf = (float)(k 2^8) (exact) has the biased exponent E; u = m 4^n with n = (E >> 1) - 79 and m, the
// significand of uf under the exponent 126 + (E & 1), in [0.5, 2).  Bits 23..15 of uf select one of 512 significand
// intervals with pivot p_i (its midpoint; 1 for the interval that ends at m = 1); r = m inv_i - 1 is at most 2^-9 and
//   -2 ln u = n (-4 ln 2) + l_i + r (-2 + r (1 - (2/3) r))
// with {inv_i, l_i} = {fl(1 / p_i), fl(2 ln inv_i)} from the table.  A table lookup and three fused multiply-adds
// take the place of a ten-term logarithm polynomial; sign bits take the place of quadrant logic.
__device__ __forceinline__ void normal_pair(uint32_t ra, uint32_t rb, float &z0, float &z1, const float2 *tab)
{
    const float uf = (float)and_or(ra, 0xFFFFFE00u, 0x100u);
    const uint32_t b = __float_as_uint(uf);
    const float nf = (float)(b >> 24) - 79.0f;
    const float m = __uint_as_float((b & 0x00FFFFFFu) | 0x3F000000u);
    const float2 pv = tab[(b >> 15) & 0x1FFu];
    const float r = __builtin_fmaf(m, pv.x, -1.0f);
    const float base = __builtin_fmaf(nf, -0x1.62e430p+1f, pv.y);
    float p = __builtin_fmaf(r, -0x1.555556p-1f, 1.0f);
    p = __builtin_fmaf(p, r, -2.0f);
    const float rho = sqrt_rn(__builtin_fmaf(r, p, base));

    const float x = (float)(int32_t)rb * 0x1p-31f;
    const float w = x * x;
    float sp = 0x1.3e17cap-13f;                      // sin(pi x / 2) = x sp(w)
    sp = __builtin_fmaf(sp, w, -0x1.32535ap-8f);
    sp = __builtin_fmaf(sp, w, 0x1.4668f2p-4f);
    sp = __builtin_fmaf(sp, w, -0x1.4abbc4p-1f);
    sp = __builtin_fmaf(sp, w, 0x1.921fb6p+0f);
    float cp = -0x1.93c734p-16f;                     // cos(pi x / 2) = 1 + w cp(w)
    cp = __builtin_fmaf(cp, w, 0x1.e173cap-11f);
    cp = __builtin_fmaf(cp, w, -0x1.55d268p-6f);
    cp = __builtin_fmaf(cp, w, 0x1.03c1eep-2f);
    cp = __builtin_fmaf(cp, w, -0x1.3bd3ccp+0f);
    const float cs = __builtin_fmaf(w, cp, 1.0f);
    z1 = rho * (x * sp);
    // magnitude of rho cos with the sign taken from bit 8 of ra (one bit-field insert)
    z0 = __uint_as_float(bit_select(0x7FFFFFFFu, __float_as_uint(rho * cs), ra << 23));
}

__device__ __forceinline__ void normal4(const u32x4 &wd, float z[4], const float2 *tab)
{
    normal_pair(wd.x, wd.y, z[0], z[1], tab);
    normal_pair(wd.z, wd.w, z[2], z[3], tab);
}

}  // namespace zo

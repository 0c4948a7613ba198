// Device-side random direction z (DistZO2, Eq. 1: z ~ N(0, I); App. A Alg. 1: every pass of a
// step re-draws the same z from the step's seed).
//
// z is addressed, not streamed: element i of tensor t under seed s is a pure function of
// (s, t, i), so "reset the generator to seed s" costs nothing and any kernel can regenerate
// exactly the values another one used.  Generator: Philox4x32-10 (Salmon et al., SC'11), one
// block per four consecutive elements.  Transform: pair-wise Box-Muller whose fp32 arithmetic
// is fixed operation by operation (only IEEE add, mul, fma, sqrt and integer ops), so the bits
// are the same on any IEEE-754 machine.  Must be compiled with -ffp-contract=off.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zo {

struct u32x4 { uint32_t x, y, z, w; };

// a ^ b ^ k in one instruction (three-input bit operation, truth table 0x96); k is wave-uniform.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t k)
{
    uint32_t r;
    asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x96" : "=v"(r) : "v"(a), "v"(b), "s"(k));
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

// Two standard normals from two words.  u = (2 (ra>>9) + 1) 2^-24 in (0,1); the angle is
// (rb>>30) quarter turns plus the 24-bit fraction (rb>>6) of one.
__device__ __forceinline__ void normal_pair(uint32_t ra, uint32_t rb, float &z0, float &z1)
{
    // radius^2 = -2 ln u, with u = m 2^e and m in [sqrt(1/2), sqrt(2))
    // (the factor 2^-24 is taken off the exponent field instead of multiplied in: 24 << 23 = 0x0c000000)
    const float u24 = (float)(2u * (ra >> 9) + 1u);
    const uint32_t ix = __float_as_uint(u24) - (0x3f3504f3u + 0x0c000000u);
    const float ef = (float)((int32_t)ix >> 23);
    const float m = __uint_as_float((ix & 0x007fffffu) + 0x3f3504f3u);
    const float r = m - 1.0f;
    // The radius needs t = -2 ln u.  The factor -2 is carried through the sum instead of multiplied in at the end:
    // every coefficient below is -2 times that of ln(1+r) = r - r^2/2 + r^3 q(r), and a power of two scales
    // every intermediate exactly, so t has the bits of -2 * (e ln 2 + ln m) evaluated step by step.
    float q = 0x1.38b2a8p-3f;
    q = __builtin_fmaf(q, r, -0x1.055ad8p-2f);
    q = __builtin_fmaf(q, r, 0x1.0d8586p-2f);
    q = __builtin_fmaf(q, r, -0x1.22da36p-2f);
    q = __builtin_fmaf(q, r, 0x1.547240p-2f);
    q = __builtin_fmaf(q, r, -0x1.99a008p-2f);
    q = __builtin_fmaf(q, r, 0x1.000228p-1f);
    q = __builtin_fmaf(q, r, -0x1.555554p-1f);
    const float r2 = r * r;
    const float r3 = r2 * r;
    const float lnm = __builtin_fmaf(r3, q, __builtin_fmaf(-2.0f, r, r2));
    const float rho = sqrt_rn(__builtin_fmaf(ef, -0x1.62e430p+0f, lnm));

    // quarter-turn fraction folded at its middle: polynomials see [0, 1/2]
    const uint32_t k = (rb >> 6) & 0xFFFFFFu;
    const bool fold = k >= 0x800000u;
    const float f = (float)(fold ? 0x1000000u - k : k) * 0x1p-24f;
    const float w = f * f;
    float sp = -0x1.2d9302p-8f;                      // sin(pi f / 2) = f sp(w)
    sp = __builtin_fmaf(sp, w, 0x1.465e92p-4f);
    sp = __builtin_fmaf(sp, w, -0x1.4abbbap-1f);
    sp = __builtin_fmaf(sp, w, 0x1.921fb6p+0f);
    const float sn = f * sp;
    float cp = 0x1.d9f7b8p-11f;                      // cos(pi f / 2) = 1 + w cp(w)
    cp = __builtin_fmaf(cp, w, -0x1.55c664p-6f);
    cp = __builtin_fmaf(cp, w, 0x1.03c1dep-2f);
    cp = __builtin_fmaf(cp, w, -0x1.3bd3ccp+0f);
    const float cs = __builtin_fmaf(w, cp, 1.0f);
    // after the fold cos and sin trade places; an odd number of quarter turns trades them again
    const uint32_t quad = rb >> 30;
    const bool swap = fold != ((quad & 1u) != 0u);
    float c = swap ? sn : cs;
    float s = swap ? cs : sn;
    // signs per quadrant: (+,+), (-,+), (-,-), (+,-)
    const uint32_t csign = ((quad + 1u) & 2u) << 30;
    const uint32_t ssign = (quad & 2u) << 30;
    c = __uint_as_float(__float_as_uint(c) ^ csign);
    s = __uint_as_float(__float_as_uint(s) ^ ssign);
    z0 = rho * c;
    z1 = rho * s;
}

__device__ __forceinline__ void normal4(const u32x4 &wd, float z[4])
{
    normal_pair(wd.x, wd.y, z[0], z[1]);
    normal_pair(wd.z, wd.w, z[2], z[3]);
}

}  // namespace zo

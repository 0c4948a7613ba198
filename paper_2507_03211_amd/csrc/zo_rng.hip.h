// Device-side random direction z (DistZO2, Eq. 1: z ~ N(0, I); App. A Alg. 1: every pass of a
// step re-draws the same z from the step's seed).
//
// z is addressed, not streamed: element i of tensor t under seed s is a pure function of
// (s, t, i), so "reset the generator to seed s" costs nothing and any kernel can regenerate
// exactly the values another one used.  Generator: Philox4x32-10 (Salmon et al., SC'11), one
// block per four consecutive elements.  Transform: pair-wise Box-Muller whose fp32 arithmetic
// is fixed operation by operation (only IEEE conversions, add, mul, fma, integer ops and one
// lookup in a table of fp32 constants), so the bits are the same on any IEEE-754 machine.
// Must be compiled with -ffp-contract=off.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "zo_rayleigh_table.hip.h"

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

// The radius table in LDS.  `tab` is a virtual base: entries [kRayleighFirst, kRayleighLast) of it must be LDS that
// the workgroup owns (24 KiB); the entries below kRayleighFirst are never touched, so a kernel with other LDS data
// puts those in front of the table.  Every kernel that draws normals fills the table once per workgroup and
// synchronises before the first draw; workgroups are persistent so that this is paid once per CU slot and launch.
__device__ __forceinline__ void load_rayleigh_cells(float4 *tab)
{
    for (int i = kRayleighFirst + (int)threadIdx.x; i < kRayleighLast; i += (int)blockDim.x) tab[i] = kRayleighCell[i];
    __syncthreads();
}

// Two standard normals from two words.
//   radius  Rayleigh-distributed, by inversion: q = (2 j + 1) 2^-25 in (0, 1/2), j = bits 30..8 of ra; bit 4 of ra
//           clear: F = q, rho = sqrt(-2 ln(1 - q)); set: 1 - F = q, rho = sqrt(-2 ln q)
//   angle   x = (float)(int32)rb 2^-31 in [-1, 1], a quarter turn either way
//   z1 = rho sin(pi x / 2);  z0 = -+rho cos(pi x / 2), negative when bit 31 of ra is set.
// Neither logarithm nor square root is evaluated: both halves of the quantile are smooth in the relative position
// of q inside a binade, so qf = (float)((2 j + 1) 2^7) (exact) picks a cell by its exponent and top five fraction
// bits, and rho = a0 + d (a1 + d (a2 + d a3)) with d = qf - (the cell's midpoint), exact, and a_k the fp32 Taylor
// coefficients from the table.  Ten instructions for the radius: and-or, convert, and-or, subtract, three for the
// table address, three fused multiply-adds.
__device__ __forceinline__ void normal_pair(uint32_t ra, uint32_t rb, float &z0, float &z1, const float4 *tab)
{
    const float qf = (float)and_or(ra, 0x7FFFFF00u, 0x80u);
    const uint32_t b = __float_as_uint(qf);
    const float d = qf - __uint_as_float(and_or(b, 0xFFFC0000u, 0x00020000u));
    // entry 2 c + h, c = (b >> 18) mod 1024, 16 bytes each: byte offset ((b >> 13) & 0x7FE0) | (ra & 0x10)
    const float4 a = *(const float4 *)((const char *)tab + and_or(b >> 13, 0x7FE0u, ra & 0x10u));
    float rho = __builtin_fmaf(a.w, d, a.z);
    rho = __builtin_fmaf(rho, d, a.y);
    rho = __builtin_fmaf(rho, d, a.x);

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
    // magnitude of rho cos with the sign bit of ra (one bit-field insert)
    z0 = __uint_as_float(bit_select(0x7FFFFFFFu, __float_as_uint(rho * cs), ra));
}

__device__ __forceinline__ void normal4(const u32x4 &wd, float z[4], const float4 *tab)
{
    normal_pair(wd.x, wd.y, z[0], z[1], tab);
    normal_pair(wd.z, wd.w, z[2], z[3], tab);
}

}  // namespace zo

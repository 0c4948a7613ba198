// Storage / activation types of the three precisions and small device helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zo {

constexpr int kFP32 = 0, kBF16 = 1, kFP16 = 2;

// ---- scalar conversions (round to nearest even, as the perturbation is specified) ----
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    __bf16 b = (__bf16)f;      // v_cvt_pk_bf16_f32 on gfx950: nearest even
    uint16_t h;
    __builtin_memcpy(&h, &b, 2);
    return h;
}
__device__ __forceinline__ float f16_bits_to_f32(uint16_t h)
{
    _Float16 v;
    __builtin_memcpy(&v, &h, 2);
    return (float)v;
}
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f)
{
    _Float16 v = (_Float16)f;   // v_cvt_f16_f32: nearest even, subnormals kept
    uint16_t h;
    __builtin_memcpy(&h, &v, 2);
    return h;
}
// Same conversion for parameter storage.  The perturbation is specified as an fp32 fma (one rounding)
// followed by the rounding into the storage type (a second one).  Left alone, the compiler folds the
// two into v_fma_mixlo_f16, which rounds the exact fma result once, straight to fp16, and differs in
// rare ties.  The empty asm makes the fp32 value opaque so the fold cannot happen; it emits no
// instruction, so the compiler still sees (and pads) every hazard around the real ones.
__device__ __forceinline__ uint16_t f32_to_f16_bits_unfused(float f)
{
    asm volatile("" : "+v"(f));
    return f32_to_f16_bits(f);
}

// Stochastic rounding of an fp32 value into a 16-bit storage type (the opt-in rounding of the update of
// Eq. 2: round-to-nearest loses almost every update of a 16-bit weight at the paper's learning rates).
// |v| = (n + f) u with u the type's spacing at |v|: the magnitude becomes (n + 1) u when the word's top
// 24 bits are below floor(f 2^24), else n u; the sign is kept, representable values never move,
// non-finite values go the round-to-nearest way.
__device__ __forceinline__ uint16_t sr_to_bf16(float v, uint32_t word)
{
    const uint32_t bits = __float_as_uint(v), mag = bits & 0x7fffffffu;
    if (mag >= 0x7f800000u) return f32_to_bf16_bits(v);
    const uint32_t up = (word >> 8) < ((mag & 0xffffu) << 8) ? 1u : 0u;      // the dropped 16 bits are f
    return (uint16_t)(((bits >> 16) & 0x8000u) | ((mag >> 16) + up));
}
__device__ __forceinline__ uint16_t sr_to_f16(float v, uint32_t word)
{
    const uint32_t bits = __float_as_uint(v), mag = bits & 0x7fffffffu, sign = (bits >> 16) & 0x8000u;
    if (mag >= 0x7f800000u) return f32_to_f16_bits(v);
    const uint32_t e = mag >> 23;
    if (e >= 143u) return (uint16_t)(sign | 0x7c00u);                       // 2^16 and beyond
    // 24-bit significand and how many of its low bits lie below the half's last place: 13 for a normal
    // half, more below 2^-14 where the spacing stays 2^-24
    const uint32_t sig = (mag & 0x7fffffu) | (e ? 0x800000u : 0u);
    const uint32_t drop = e >= 113u ? 13u : (e ? 126u - e : 125u);
    const uint32_t expo = e >= 113u ? (e - 113u) << 10 : 0u;                // sig >> 13 carries the implicit one on top
    const uint32_t n = expo + (drop < 32u ? sig >> drop : 0u);
    uint32_t f24;
    if (drop <= 24u) f24 = (sig & ((1u << drop) - 1u)) << (24u - drop);
    else f24 = drop - 24u < 32u ? sig >> (drop - 24u) : 0u;
    return (uint16_t)(sign | (n + ((word >> 8) < f24 ? 1u : 0u)));
}

// Per-precision types.  W: parameter storage, A: activations between kernels, R: residual
// stream, Acc: accumulator / statistics.  fp32 parameters run with fp64 activations: g is a
// difference of two nearly equal losses, and fp32 activation rounding alone would eat the
// tolerance asked of that configuration.
template <int DT> struct Prec;
template <> struct Prec<kFP32> {
    using W = float; using A = double; using R = double; using Acc = double;
    static __device__ __forceinline__ float w2f(W v) { return v; }
    static __device__ __forceinline__ W f2w(float v) { return v; }
    static __device__ __forceinline__ Acc a2acc(A v) { return v; }
    static __device__ __forceinline__ A acc2a(Acc v) { return v; }
};
template <> struct Prec<kBF16> {
    using W = uint16_t; using A = uint16_t; using R = float; using Acc = float;
    static __device__ __forceinline__ float w2f(W v) { return bf16_bits_to_f32(v); }
    static __device__ __forceinline__ W f2w(float v) { return f32_to_bf16_bits(v); }
    static __device__ __forceinline__ Acc a2acc(A v) { return bf16_bits_to_f32(v); }
    static __device__ __forceinline__ A acc2a(Acc v) { return f32_to_bf16_bits(v); }
};
template <> struct Prec<kFP16> {
    using W = uint16_t; using A = uint16_t; using R = float; using Acc = float;
    static __device__ __forceinline__ float w2f(W v) { return f16_bits_to_f32(v); }
    static __device__ __forceinline__ W f2w(float v) { return f32_to_f16_bits_unfused(v); }
    static __device__ __forceinline__ Acc a2acc(A v) { return f16_bits_to_f32(v); }
    static __device__ __forceinline__ A acc2a(Acc v) { return f32_to_f16_bits(v); }
};

inline size_t elem_bytes(int dtype) { return dtype == kFP32 ? 4 : 2; }
inline size_t act_bytes(int dtype) { return dtype == kFP32 ? 8 : 2; }
inline size_t resid_bytes(int dtype) { return dtype == kFP32 ? 8 : 4; }
inline size_t acc_bytes(int dtype) { return dtype == kFP32 ? 8 : 4; }

// ---- block-wide reductions (blockDim.x multiple of 64, <= 1024) ----
template <typename T> __device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
template <typename T> __device__ __forceinline__ T wave_max(T v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { T t = __shfl_xor(v, o, 64); v = t > v ? t : v; }
    return v;
}
template <typename T> __device__ __forceinline__ T block_sum(T v, T *smem /* >= 16 */)
{
    v = wave_sum(v);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) smem[w] = v;
    __syncthreads();
    T t = 0;
    for (int i = 0; i < nw; ++i) t += smem[i];
    return t;
}
template <typename T> __device__ __forceinline__ T block_max(T v, T *smem)
{
    v = wave_max(v);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) smem[w] = v;
    __syncthreads();
    T t = smem[0];
    for (int i = 1; i < nw; ++i) t = smem[i] > t ? smem[i] : t;
    return t;
}

}  // namespace zo

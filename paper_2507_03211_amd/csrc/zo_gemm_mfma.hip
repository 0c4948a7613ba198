// Sign-batched linear layer on the matrix cores (bf16 / fp16 inputs, fp32 accumulate).
//
// This is where a ZO step spends its time: the paired forward passes of Eq. 1 (DistZO2,
// Preliminaries; PertP workflow Step 2 runs the two signs on two devices, here both signs are
// one launch on one device, rows [0, m_half) against W+ and rows [m_half, 2 m_half) against W-).
//
//   y[row, n] = sum_k x[row, k] wt[n, k]  (+ bias, ReLU, residual add)
//
// Both operands are K-contiguous ("TN"), which is what v_mfma_f32_32x32x16_{bf16,f16} wants:
// every lane feeds 8 consecutive k of one row.  The weight tile is the MFMA A operand and the
// activation tile the B operand, so a lane's 16 accumulators are 4 runs of 4 consecutive n of
// one output row, which makes the epilogue 8/16-byte stores.
//
// Tiling: 128 (rows) x 128 (n) x 64 (k) per workgroup of 4 waves (2 x 2, 64 x 64 each, i.e.
// 2 x 2 MFMA tiles of 32 x 32), LDS double-buffered, 16-byte chunks XOR-swizzled by row so
// that the 32 rows a fragment load touches spread over all banks.
#include "zo_kernels.h"
#include "zo_types.hip.h"

namespace zo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kChunksPerRow = BK / 8;       // 16-byte chunks per tile row

template <int DT> __device__ __forceinline__ f32x16 mfma32(const uint4 &a, const uint4 &b, const f32x16 &c)
{
    if constexpr (DT == kBF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// LDS tile: [rows][8 chunks] of uint4, chunk c of row r stored at c ^ (r & 7).
__device__ __forceinline__ int lds_slot(int r, int c) { return r * kChunksPerRow + (c ^ (r & 7)); }

template <int DT, int EPI>
__global__ __launch_bounds__(256) void linear_mfma_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ wt_p,
                                                          const uint16_t *__restrict__ wt_m, const uint16_t *__restrict__ b_p,
                                                          const uint16_t *__restrict__ b_m, void *__restrict__ y,
                                                          int m_half, int n, int k)
{
    __shared__ uint4 xs[2][BM * kChunksPerRow];
    __shared__ uint4 ws[2][BN * kChunksPerRow];
    const int sign = blockIdx.z;
    const uint16_t *xa = x + (size_t)sign * m_half * k;
    const uint16_t *wt = sign ? wt_m : wt_p;
    const uint16_t *bias = sign ? b_m : b_p;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // global -> LDS assignment: chunk c = tid % 8 of rows tid/8 + 32 i
    const int lc = tid & 7, lr = tid >> 3;
    const uint16_t *xg[4], *wg[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int xr = m0 + lr + 32 * i; xr = xr < m_half ? xr : m_half - 1;     // clamp: masked at the store
        int wr = n0 + lr + 32 * i; wr = wr < n ? wr : n - 1;
        xg[i] = xa + (size_t)xr * k + lc * 8;
        wg[i] = wt + (size_t)wr * k + lc * 8;
    }
    uint4 xreg[4], wreg[4];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            xreg[i] = *(const uint4 *)(xg[i] + k0);
            wreg[i] = *(const uint4 *)(wg[i] + k0);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            xs[buf][lds_slot(lr + 32 * i, lc)] = xreg[i];
            ws[buf][lds_slot(lr + 32 * i, lc)] = wreg[i];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    const int nk = k / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    const int fr = lane & 31, fh = lane >> 5;     // fragment row, k half
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_global((kt + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            uint4 wf[2], xf[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                wf[t] = ws[buf][lds_slot(wn * 64 + t * 32 + fr, ks * 2 + fh)];
                xf[t] = xs[buf][lds_slot(wm * 64 + t * 32 + fr, ks * 2 + fh)];
            }
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                for (int tm = 0; tm < 2; ++tm) acc[tn][tm] = mfma32<DT>(wf[tn], xf[tm], acc[tn][tm]);
        }
        if (kt + 1 < nk) store_lds(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds, for each (tn, tm), row m = .. + lane%32 and n = .. + 8 g + 4 (lane/32) + 0..3
#pragma unroll
    for (int tm = 0; tm < 2; ++tm) {
        const int mr = m0 + wm * 64 + tm * 32 + fr;
        if (mr >= m_half) continue;
        const size_t row = (size_t)sign * m_half + mr;
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int nc = n0 + wn * 64 + tn * 32 + 8 * g + 4 * fh;
                if (nc >= n) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[tn][tm][4 * g + e];
                if constexpr (EPI != 3) {
                    const uint2 braw = *(const uint2 *)(bias + nc);
                    const uint16_t bb[4] = {(uint16_t)(braw.x & 0xffff), (uint16_t)(braw.x >> 16),
                                            (uint16_t)(braw.y & 0xffff), (uint16_t)(braw.y >> 16)};
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += Prec<DT>::w2f(bb[e]);
                }
                if constexpr (EPI == 0 || EPI == 1) {
                    if constexpr (EPI == 1) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
                    }
                    uint2 o;
                    o.x = (uint32_t)Prec<DT>::acc2a(v[0]) | ((uint32_t)Prec<DT>::acc2a(v[1]) << 16);
                    o.y = (uint32_t)Prec<DT>::acc2a(v[2]) | ((uint32_t)Prec<DT>::acc2a(v[3]) << 16);
                    *(uint2 *)((uint16_t *)y + row * n + nc) = o;
                } else if constexpr (EPI == 2) {
                    float4 *p = (float4 *)((float *)y + row * n + nc);
                    float4 h = *p;
                    h.x += v[0]; h.y += v[1]; h.z += v[2]; h.w += v[3];
                    *p = h;
                } else {
                    *(float4 *)((float *)y + row * n + nc) = float4{v[0], v[1], v[2], v[3]};
                }
            }
        }
    }
}

template <int DT>
void launch_t(const void *x, const void *wt_p, const void *wt_m, const void *b_p, const void *b_m, void *y, int n_sign,
              int m_half, int n, int k, int epi, hipStream_t s)
{
    const dim3 grid((n + BN - 1) / BN, (m_half + BM - 1) / BM, n_sign), block(256);
#define ZO_L(E)                                                                                                   \
    linear_mfma_kernel<DT, E><<<grid, block, 0, s>>>((const uint16_t *)x, (const uint16_t *)wt_p, (const uint16_t *)wt_m, \
                                                     (const uint16_t *)b_p, (const uint16_t *)b_m, y, m_half, n, k)
    switch (epi) {
    case 0: ZO_L(0); break;
    case 1: ZO_L(1); break;
    case 2: ZO_L(2); break;
    default: ZO_L(3); break;
    }
#undef ZO_L
}

}  // namespace

bool mfma_linear_supported(int m_half, int n, int k) { return m_half >= 1 && n >= 8 && n % 8 == 0 && k >= BK && k % BK == 0; }

hipError_t launch_linear_mfma(const void *x, const void *wt_p, const void *wt_m, const void *b_p, const void *b_m, void *y,
                              int dtype, int n_sign, int m_half, int n, int k, int epilogue, hipStream_t s)
{
    if (!mfma_linear_supported(m_half, n, k) || (dtype != kBF16 && dtype != kFP16)) return hipErrorInvalidValue;
    if (dtype == kBF16) launch_t<kBF16>(x, wt_p, wt_m, b_p, b_m, y, n_sign, m_half, n, k, epilogue, s);
    else launch_t<kFP16>(x, wt_p, wt_m, b_p, b_m, y, n_sign, m_half, n, k, epilogue, s);
    return hipGetLastError();
}

}  // namespace zo

// Causal multi-head attention on the matrix cores (bf16 / fp16 in, fp32 softmax statistics),
// part of the paired forward passes of Eq. 1 (DistZO2, Preliminaries).  Both signs are just
// more sequences: the kernel sees n_seq = 2 * batch independent sequences.
//
// One workgroup = (128 query rows, one head, one sequence); 4 waves x 32 query rows.  Key /
// value tiles of 64 keys stream through LDS.  Everything is computed transposed so that a
// lane owns one query row:
//     S^T[key, q] = K Q^T        (MFMA A = K rows, B = Q rows; lane: column q, 16 keys)
//     O^T[c, q]  += V^T P^T      (MFMA A = V^T rows, B = P^T; lane: column q, 16 channels)
// so the online-softmax running maximum, normaliser and the rescaling of O are per-lane
// scalars, and the row reductions need one cross-half shuffle.  The contraction order of the
// P V product follows the accumulator layout of S^T (keys 16s + 4h + {0..3}, 16s + 8 + 4h +
// {0..3} for lane half h), which V^T is read with as well, so P never leaves registers.
#include "zo_kernels.h"
#include "zo_types.hip.h"

namespace zo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BQ = 128, BKV = 64;

template <int DT> __device__ __forceinline__ f32x16 mfma32(const uint4 &a, const uint4 &b, const f32x16 &c)
{
    if constexpr (DT == kBF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

template <int DT> __device__ __forceinline__ uint32_t pack2(float a, float b)
{
    return (uint32_t)Prec<DT>::acc2a(a) | ((uint32_t)Prec<DT>::acc2a(b) << 16);
}

template <int DT, int DH>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const uint16_t *__restrict__ qkv, uint16_t *__restrict__ out, int seq,
                                                        int n_heads)
{
    constexpr int CH = DH / 8;            // 16-byte chunks per K row
    constexpr int VLD = BKV + 4;          // padded V^T row: 34 banks, so 32 lanes reading 8 bytes each spread over all 64
    __shared__ uint4 ks[BKV * CH];        // K tile, chunk c of key r at c ^ kswz(r): 16 rows -> 16 distinct bank groups
    __shared__ __attribute__((aligned(16))) uint16_t vt[DH * VLD];   // V^T tile: [channel][key]

    auto kswz = [](int r) { return DH == 128 ? (r & 15) : ((r >> 1) & 7); };
    const int qt = (int)gridDim.x - 1 - (int)blockIdx.x;             // long rows first
    const int head = blockIdx.y, sq = blockIdx.z;
    const int d = n_heads * DH, ld = 3 * d;
    const uint16_t *base = qkv + (size_t)sq * seq * ld + head * DH;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fh = lane >> 5;
    const int q0 = qt * BQ + wave * 32;          // first query row of this wave
    const int qrow = q0 + fr;                    // this lane's query row
    const int qload = qrow < seq ? qrow : seq - 1;

    // Q fragments: B operand, lane = (row fr, k half fh), all DH/16 steps
    uint4 qf[DH / 16];
#pragma unroll
    for (int s = 0; s < DH / 16; ++s) qf[s] = *(const uint4 *)(base + (size_t)qload * ld + s * 16 + fh * 8);

    f32x16 oacc[DH / 32];
#pragma unroll
    for (int c = 0; c < DH / 32; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[c][i] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    const float sc = 1.4426950408889634f / __builtin_sqrtf((float)DH);    // log2(e) / sqrt(d_head)

    // global -> LDS assignment for a K/V tile: key = tid % 64, chunks tid / 64 + 4 i
    const int lkey = tid & 63, lch = tid >> 6;
    constexpr int NLD = CH / 4;
    uint4 kreg[NLD], vreg[NLD];
    auto load_tile = [&](int k0) {
        int kr = k0 + lkey; kr = kr < seq ? kr : seq - 1;
        const uint16_t *kp = base + (size_t)kr * ld + d;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            kreg[i] = *(const uint4 *)(kp + (lch + 4 * i) * 8);
            vreg[i] = *(const uint4 *)(kp + d + (lch + 4 * i) * 8);
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = lch + 4 * i;
            ks[lkey * CH + (c ^ kswz(lkey))] = kreg[i];
            const uint32_t w[4] = {vreg[i].x, vreg[i].y, vreg[i].z, vreg[i].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                vt[(c * 8 + 2 * e) * VLD + lkey] = (uint16_t)(w[e] & 0xffffu);
                vt[(c * 8 + 2 * e + 1) * VLD + lkey] = (uint16_t)(w[e] >> 16);
            }
        }
    };

    const int q_hi = qt * BQ + BQ - 1 < seq - 1 ? qt * BQ + BQ - 1 : seq - 1;   // last query row of the workgroup
    const int n_tiles = q_hi / BKV + 1;
    load_tile(0);
    for (int t = 0; t < n_tiles; ++t) {
        const int k0 = t * BKV;
        __syncthreads();                 // previous tile fully consumed
        store_tile();
        __syncthreads();
        if (t + 1 < n_tiles) load_tile(k0 + BKV);
        if (k0 > q0 + 31) continue;      // tile entirely in this wave's future (uniform per wave)

        // S^T tile: 64 keys x 32 queries = two 32 x 32 accumulators
        f32x16 sacc[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.0f;
#pragma unroll
            for (int s = 0; s < DH / 16; ++s) {
                const int r = kt * 32 + fr;
                const uint4 kf = ks[r * CH + ((2 * s + fh) ^ kswz(r))];
                sacc[kt] = mfma32<DT>(kf, qf[s], sacc[kt]);
            }
        }
        // scale, mask (key > query), tile maximum
        const bool diag = k0 + BKV - 1 > q0;
        float tmax = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float v = sacc[kt][i] * sc;
                if (diag) {
                    const int key = k0 + kt * 32 + 8 * (i >> 2) + 4 * fh + (i & 3);
                    if (key > qrow) v = -INFINITY;
                }
                sacc[kt][i] = v;
                tmax = v > tmax ? v : tmax;
            }
        const float other = __shfl_xor(tmax, 32, 64);
        tmax = other > tmax ? other : tmax;
        const float m_new = tmax > m_run ? tmax : m_run;      // finite: key k0 <= q0 <= qrow is never masked
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        float psum = 0.0f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(sacc[kt][i] - m_new);
                sacc[kt][i] = p;
                psum += p;
            }
        psum += __shfl_xor(psum, 32, 64);
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int c = 0; c < DH / 32; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[c][i] *= alpha;
        // O^T += V^T P^T : four contraction steps of 16 keys
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int kt = s >> 1, rb = (s & 1) * 8;
            uint4 pf;
            pf.x = pack2<DT>(sacc[kt][rb + 0], sacc[kt][rb + 1]);
            pf.y = pack2<DT>(sacc[kt][rb + 2], sacc[kt][rb + 3]);
            pf.z = pack2<DT>(sacc[kt][rb + 4], sacc[kt][rb + 5]);
            pf.w = pack2<DT>(sacc[kt][rb + 6], sacc[kt][rb + 7]);
            const int key_a = 16 * s + 4 * fh;       // keys key_a .. +3 and key_a + 8 .. +3
#pragma unroll
            for (int c = 0; c < DH / 32; ++c) {
                const uint16_t *vrow = vt + (c * 32 + fr) * VLD;
                const uint2 lo = *(const uint2 *)(vrow + key_a);
                const uint2 hi = *(const uint2 *)(vrow + key_a + 8);
                oacc[c] = mfma32<DT>(uint4{lo.x, lo.y, hi.x, hi.y}, pf, oacc[c]);
            }
        }
    }

    if (qrow < seq) {
        const float inv = 1.0f / l_run;
        uint16_t *o = out + ((size_t)sq * seq + qrow) * d + head * DH;
#pragma unroll
        for (int c = 0; c < DH / 32; ++c)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 v;
                v.x = pack2<DT>(oacc[c][4 * g] * inv, oacc[c][4 * g + 1] * inv);
                v.y = pack2<DT>(oacc[c][4 * g + 2] * inv, oacc[c][4 * g + 3] * inv);
                *(uint2 *)(o + c * 32 + 8 * g + 4 * fh) = v;
            }
    }
}

}  // namespace

bool mfma_attention_supported(int seq, int d_head) { return seq >= 1 && (d_head == 64 || d_head == 128); }

hipError_t launch_attention_mfma(const void *qkv, void *out, int dtype, int n_seq, int seq, int n_heads, int d_head,
                                 hipStream_t s)
{
    if (!mfma_attention_supported(seq, d_head) || (dtype != kBF16 && dtype != kFP16)) return hipErrorInvalidValue;
    const dim3 grid((seq + BQ - 1) / BQ, n_heads, n_seq), block(256);
    const uint16_t *q = (const uint16_t *)qkv;
    uint16_t *o = (uint16_t *)out;
    if (dtype == kBF16) {
        if (d_head == 64) attn_mfma_kernel<kBF16, 64><<<grid, block, 0, s>>>(q, o, seq, n_heads);
        else attn_mfma_kernel<kBF16, 128><<<grid, block, 0, s>>>(q, o, seq, n_heads);
    } else {
        if (d_head == 64) attn_mfma_kernel<kFP16, 64><<<grid, block, 0, s>>>(q, o, seq, n_heads);
        else attn_mfma_kernel<kFP16, 128><<<grid, block, 0, s>>>(q, o, seq, n_heads);
    }
    return hipGetLastError();
}

}  // namespace zo

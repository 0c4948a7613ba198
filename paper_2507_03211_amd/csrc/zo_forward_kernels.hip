// Forward-pass kernels that are not matrix-core bound: embedding gather, LayerNorm, the
// cross-entropy reduction, the loss / projected-gradient scalars (DistZO2 Eq. 1), and the
// plain (non-MFMA) linear and attention kernels that serve the fp32-parameter precision,
// which runs with fp64 activations, and shapes the MFMA tilings do not cover.
//
// Row layout everywhere: row = sign * m_half + b * seq + t, sign 0 = theta + eps z,
// sign 1 = theta - eps z; each sign reads its own copy of every parameter.
#include "zo_kernels.h"
#include "zo_types.hip.h"

namespace zo {

// ------------------------------------------------------------------ embedding
// h[row, :] = E_sign[token] + Pos_sign[t];  target[row] = next token (or -1 at t = seq-1).
template <int DT>
__global__ __launch_bounds__(256) void embed_kernel(const int32_t *__restrict__ tokens, const void *e_p, const void *e_m,
                                                    const void *pos_p, const void *pos_m, void *resid,
                                                    int32_t *__restrict__ target, uint32_t *flags, int batch, int seq,
                                                    int d, int vocab)
{
    using P = Prec<DT>;
    const int m_half = batch * seq;
    const int row = blockIdx.x;
    const int sign = row / m_half, bt = row % m_half, t = bt % seq;
    const int tok = tokens[bt];
    const bool ok = tok >= 0 && tok < vocab;
    if (threadIdx.x == 0) {
        int tg = -1;
        if (t + 1 < seq) {
            tg = tokens[bt + 1];
            if (tg < 0 || tg >= vocab) { tg = -2; atomicOr(flags, 2u); }   // -2: poisons the row loss
        }
        target[row] = tg;
        if (!ok) atomicOr(flags, 2u);
    }
    const typename P::W *e = (const typename P::W *)(sign ? e_m : e_p) + (size_t)(ok ? tok : 0) * d;
    const typename P::W *p = (const typename P::W *)(sign ? pos_m : pos_p) + (size_t)t * d;
    typename P::R *h = (typename P::R *)resid + (size_t)row * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        typename P::R v = (typename P::R)P::w2f(e[c]) + (typename P::R)P::w2f(p[c]);
        if (!ok) v = (typename P::R)__builtin_nanf("");
        h[c] = v;
    }
}

// ------------------------------------------------------------------ LayerNorm
// One workgroup per row; mean and (biased) variance by two passes over the row.
template <int DT>
__global__ __launch_bounds__(256) void layernorm_kernel(const void *resid, const void *g_p, const void *g_m,
                                                        const void *b_p, const void *b_m, void *y, int m_half, int d,
                                                        float eps)
{
    using P = Prec<DT>;
    using Acc = typename P::Acc;
    __shared__ Acc red[16];
    const int row = blockIdx.x;
    const int sign = row / m_half;
    const typename P::R *h = (const typename P::R *)resid + (size_t)row * d;
    const typename P::W *g = (const typename P::W *)(sign ? g_m : g_p);
    const typename P::W *b = (const typename P::W *)(sign ? b_m : b_p);
    typename P::A *out = (typename P::A *)y + (size_t)row * d;
    Acc s = 0;
    for (int c = threadIdx.x; c < d; c += blockDim.x) s += (Acc)h[c];
    const Acc mean = block_sum(s, red) / (Acc)d;
    Acc v = 0;
    for (int c = threadIdx.x; c < d; c += blockDim.x) { const Acc t = (Acc)h[c] - mean; v += t * t; }
    const Acc var = block_sum(v, red) / (Acc)d;
    Acc rstd;
    if constexpr (sizeof(Acc) == 8) rstd = 1.0 / __builtin_sqrt(var + (double)eps);
    else rstd = 1.0f / __builtin_sqrtf(var + eps);
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        const Acc t = ((Acc)h[c] - mean) * rstd * (Acc)P::w2f(g[c]) + (Acc)P::w2f(b[c]);
        out[c] = P::acc2a(t);
    }
}


// Fast path for 2-byte activations and rows of up to 2048 elements: one wavefront per row, the row held in registers
// (NV float4 per lane), so the residual stream is read once; statistics by wavefront shuffles only.  d % 4 == 0.
template <int DT, int NV>
__global__ __launch_bounds__(256) void layernorm_wave_kernel(const float *__restrict__ resid, const uint16_t *__restrict__ g_p,
                                                             const uint16_t *__restrict__ g_m, const uint16_t *__restrict__ b_p,
                                                             const uint16_t *__restrict__ b_m, uint16_t *__restrict__ y, int rows,
                                                             int m_half, int d, float eps)
{
    using P = Prec<DT>;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= rows) return;
    const int sign = row / m_half;
    const float4 *h = (const float4 *)(resid + (size_t)row * d);
    const uint2 *g = (const uint2 *)(sign ? g_m : g_p), *b = (const uint2 *)(sign ? b_m : b_p);
    uint2 *out = (uint2 *)(y + (size_t)row * d);
    const int nvec = d >> 2;
    float4 v[NV];
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + 64 * i;
        v[i] = c < nvec ? h[c] : float4{0.0f, 0.0f, 0.0f, 0.0f};
        s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
    const float mean = wave_sum(s) / (float)d;
    float q = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (lane + 64 * i < nvec) {
            const float a = v[i].x - mean, bb = v[i].y - mean, c = v[i].z - mean, dd = v[i].w - mean;
            q += (a * a + bb * bb) + (c * c + dd * dd);
        }
    }
    const float rstd = 1.0f / __builtin_sqrtf(wave_sum(q) / (float)d + eps);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + 64 * i;
        if (c < nvec) {
            const uint2 gr = g[c], br = b[c];
            const float g0 = P::w2f((uint16_t)(gr.x & 0xffff)), g1 = P::w2f((uint16_t)(gr.x >> 16));
            const float g2 = P::w2f((uint16_t)(gr.y & 0xffff)), g3 = P::w2f((uint16_t)(gr.y >> 16));
            const float b0 = P::w2f((uint16_t)(br.x & 0xffff)), b1 = P::w2f((uint16_t)(br.x >> 16));
            const float b2 = P::w2f((uint16_t)(br.y & 0xffff)), b3 = P::w2f((uint16_t)(br.y >> 16));
            const float o0 = (v[i].x - mean) * rstd * g0 + b0, o1 = (v[i].y - mean) * rstd * g1 + b1;
            const float o2 = (v[i].z - mean) * rstd * g2 + b2, o3 = (v[i].w - mean) * rstd * g3 + b3;
            uint2 o;
            o.x = (uint32_t)P::acc2a(o0) | ((uint32_t)P::acc2a(o1) << 16);
            o.y = (uint32_t)P::acc2a(o2) | ((uint32_t)P::acc2a(o3) << 16);
            out[c] = o;
        }
    }
}

// The same for longer rows: one workgroup of 256 threads per row, NV float4 per thread, the two sums across the four
// wavefronts through LDS.  d % 4 == 0, d <= 1024 NV.  Measured against the wavefront-per-row kernel (8192 rows):
// 5.4 against 4.7 TB/s at d = 4096 and 5120, 5.5 against 2.7 at 12288 (48 float4 per lane leave a SIMD two waves),
// 5.5 against 5.9 at 2048, 4.3 against 5.6 at 1280: hence the switch at 2048.
template <int DT, int NV>
__global__ __launch_bounds__(256) void layernorm_block_kernel(const float *__restrict__ resid, const uint16_t *__restrict__ g_p,
                                                              const uint16_t *__restrict__ g_m, const uint16_t *__restrict__ b_p,
                                                              const uint16_t *__restrict__ b_m, uint16_t *__restrict__ y, int m_half,
                                                              int d, float eps)
{
    using P = Prec<DT>;
    __shared__ float red[16];
    const int row = blockIdx.x, tid = threadIdx.x;
    const int sign = row / m_half;
    const float4 *h = (const float4 *)(resid + (size_t)row * d);
    const uint2 *g = (const uint2 *)(sign ? g_m : g_p), *b = (const uint2 *)(sign ? b_m : b_p);
    uint2 *out = (uint2 *)(y + (size_t)row * d);
    const int nvec = d >> 2;
    float4 v[NV];
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = tid + 256 * i;
        v[i] = c < nvec ? h[c] : float4{0.0f, 0.0f, 0.0f, 0.0f};
        s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
    const float mean = block_sum(s, red) / (float)d;
    float q = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (tid + 256 * i < nvec) {
            const float a = v[i].x - mean, bb = v[i].y - mean, c = v[i].z - mean, dd = v[i].w - mean;
            q += (a * a + bb * bb) + (c * c + dd * dd);
        }
    }
    const float rstd = 1.0f / __builtin_sqrtf(block_sum(q, red) / (float)d + eps);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = tid + 256 * i;
        if (c < nvec) {
            const uint2 gr = g[c], br = b[c];
            const float g0 = P::w2f((uint16_t)(gr.x & 0xffff)), g1 = P::w2f((uint16_t)(gr.x >> 16));
            const float g2 = P::w2f((uint16_t)(gr.y & 0xffff)), g3 = P::w2f((uint16_t)(gr.y >> 16));
            const float b0 = P::w2f((uint16_t)(br.x & 0xffff)), b1 = P::w2f((uint16_t)(br.x >> 16));
            const float b2 = P::w2f((uint16_t)(br.y & 0xffff)), b3 = P::w2f((uint16_t)(br.y >> 16));
            const float o0 = (v[i].x - mean) * rstd * g0 + b0, o1 = (v[i].y - mean) * rstd * g1 + b1;
            const float o2 = (v[i].z - mean) * rstd * g2 + b2, o3 = (v[i].w - mean) * rstd * g3 + b3;
            uint2 o;
            o.x = (uint32_t)P::acc2a(o0) | ((uint32_t)P::acc2a(o1) << 16);
            o.y = (uint32_t)P::acc2a(o2) | ((uint32_t)P::acc2a(o3) << 16);
            out[c] = o;
        }
    }
}

// ------------------------------------------------------------------ plain linear layer
// y[row, n] = sum_k x[row, k] wt[n, k] (+ bias).  64 x 64 output tile, 16-deep LDS slabs,
// 4 x 4 outputs per thread.  blockIdx.z selects the sign.
template <int DT, int EPI>
__global__ __launch_bounds__(256) void linear_plain_kernel(const void *x, const void *wt_p, const void *wt_m,
                                                           const void *b_p, const void *b_m, void *y, int m_half, int n,
                                                           int k)
{
    using P = Prec<DT>;
    using Acc = typename P::Acc;
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ Acc xs[BK][BM + 1];
    __shared__ Acc ws[BK][BN + 1];
    const int sign = blockIdx.z;
    const typename P::A *xa = (const typename P::A *)x + (size_t)sign * m_half * k;
    const typename P::W *wt = (const typename P::W *)(sign ? wt_m : wt_p);
    const typename P::W *bias = (const typename P::W *)(sign ? b_m : b_p);
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    Acc acc[4][4] = {};
    for (int k0 = 0; k0 < k; k0 += BK) {
        // 64 rows x 16 k = 1024 values per operand, 4 per thread
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = threadIdx.x + 256 * i;
            const int r = idx / BK, kk = idx % BK;
            const bool kin = k0 + kk < k;
            xs[kk][r] = (kin && m0 + r < m_half) ? P::a2acc(xa[(size_t)(m0 + r) * k + k0 + kk]) : (Acc)0;
            ws[kk][r] = (kin && n0 + r < n) ? (Acc)P::w2f(wt[(size_t)(n0 + r) * k + k0 + kk]) : (Acc)0;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            Acc a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = xs[kk][ty * 4 + i]; b[i] = ws[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = m0 + ty * 4 + i;
        if (r >= m_half) continue;
        const size_t row = (size_t)sign * m_half + r;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = n0 + tx * 4 + j;
            if (c >= n) continue;
            Acc v = acc[i][j];
            if constexpr (EPI != 3) v += (Acc)P::w2f(bias[c]);
            if constexpr (EPI == 0) ((typename P::A *)y)[row * n + c] = P::acc2a(v);
            if constexpr (EPI == 1) ((typename P::A *)y)[row * n + c] = P::acc2a(v > 0 ? v : (Acc)0);
            if constexpr (EPI == 2) ((typename P::R *)y)[row * n + c] += (typename P::R)v;
            if constexpr (EPI == 3) ((Acc *)y)[row * n + c] = v;
        }
    }
}

// ------------------------------------------------------------------ plain causal attention
// One workgroup per (query row, head, sequence): scores into LDS, softmax, then P V.
template <int DT>
__global__ __launch_bounds__(128) void attention_plain_kernel(const void *qkv_, void *out_, int seq, int n_heads,
                                                              int d_head)
{
    using P = Prec<DT>;
    using Acc = typename P::Acc;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Acc *sc = (Acc *)smem_raw;          // [seq]
    Acc *qs = sc + seq;                 // [d_head]
    Acc *red = qs + d_head;             // [16]
    const int t = blockIdx.x, head = blockIdx.y, sq = blockIdx.z;
    const int d = n_heads * d_head;
    const typename P::A *qkv = (const typename P::A *)qkv_ + (size_t)sq * seq * 3 * d;
    const typename P::A *q = qkv + (size_t)t * 3 * d + head * d_head;
    for (int c = threadIdx.x; c < d_head; c += blockDim.x) qs[c] = P::a2acc(q[c]);
    __syncthreads();
    Acc scale;
    if constexpr (sizeof(Acc) == 8) scale = 1.0 / __builtin_sqrt((double)d_head);
    else scale = 1.0f / __builtin_sqrtf((float)d_head);
    Acc mx = -INFINITY;
    for (int j = threadIdx.x; j <= t; j += blockDim.x) {
        const typename P::A *kr = qkv + (size_t)j * 3 * d + d + head * d_head;
        Acc s = 0;
        for (int c = 0; c < d_head; ++c) s += qs[c] * P::a2acc(kr[c]);
        s *= scale;
        sc[j] = s;
        mx = s > mx ? s : mx;
    }
    mx = block_max(mx, red);
    Acc sum = 0;
    for (int j = threadIdx.x; j <= t; j += blockDim.x) {
        Acc e;
        if constexpr (sizeof(Acc) == 8) e = exp(sc[j] - mx); else e = __expf(sc[j] - mx);
        sc[j] = e;
        sum += e;
    }
    sum = block_sum(sum, red);
    __syncthreads();
    typename P::A *o = (typename P::A *)out_ + ((size_t)sq * seq + t) * d + head * d_head;
    for (int c = threadIdx.x; c < d_head; c += blockDim.x) {
        Acc a = 0;
        for (int j = 0; j <= t; ++j) a += sc[j] * P::a2acc(qkv[(size_t)j * 3 * d + 2 * d + head * d_head + c]);
        o[c] = P::acc2a(a / sum);
    }
}

// ------------------------------------------------------------------ cross entropy over stored logits
// row_loss[r] = logsumexp(logits[r, :]) - logits[r, target[r]]; 0 for target -1, NaN for -2.
template <typename Acc>
__global__ __launch_bounds__(256) void ce_rows_kernel(const Acc *__restrict__ logits, const int32_t *__restrict__ target,
                                                      double *__restrict__ row_loss, int vocab)
{
    __shared__ double red[16];
    const int r = blockIdx.x;
    const int tg = target[r];
    if (tg == -1) { if (threadIdx.x == 0) row_loss[r] = 0.0; return; }
    const Acc *lg = logits + (size_t)r * vocab;
    double mx = -INFINITY;
    for (int c = threadIdx.x; c < vocab; c += blockDim.x) { const double v = (double)lg[c]; mx = v > mx ? v : mx; }
    mx = block_max(mx, red);
    double s = 0;
    for (int c = threadIdx.x; c < vocab; c += blockDim.x) s += exp((double)lg[c] - mx);
    s = block_sum(s, red);
    if (threadIdx.x == 0) row_loss[r] = tg >= 0 ? (log(s) + mx - (double)lg[tg]) : (double)__builtin_nan("");
}

// Merge the (max, sum-exp) pairs the fused LM-head epilogue left for a row: one wavefront per row.
__global__ __launch_bounds__(256) void ce_finish_kernel(const float2 *__restrict__ partials, int n_partial,
                                                        const float *__restrict__ target_logit,
                                                        const int32_t *__restrict__ target, double *__restrict__ row_loss,
                                                        int rows)
{
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (r >= rows) return;
    const int tg = target[r];
    if (tg == -1) { if (lane == 0) row_loss[r] = 0.0; return; }
    const float2 *p = partials + (size_t)r * n_partial;
    float mx = -INFINITY;
    for (int i = lane; i < n_partial; i += 64) mx = p[i].x > mx ? p[i].x : mx;
    mx = wave_max(mx);
    double s = 0.0;
    for (int i = lane; i < n_partial; i += 64)
        if (p[i].x > -INFINITY) s += (double)p[i].y * exp((double)p[i].x - (double)mx);
    s = wave_sum(s);
    if (lane == 0) row_loss[r] = tg >= 0 ? (log(s) + (double)mx - (double)target_logit[r]) : (double)__builtin_nan("");
}

// L+- = sum of the sign's row losses / count, in a fixed order (deterministic).
__global__ __launch_bounds__(1024) void loss_reduce_kernel(const double *__restrict__ row_loss, int m_half, int count,
                                                           double *__restrict__ loss_pm)
{
    __shared__ double red[16];
    const int sign = blockIdx.x;
    const double *r = row_loss + (size_t)sign * m_half;
    double s = 0;
    for (int i = threadIdx.x; i < m_half; i += blockDim.x) s += r[i];
    s = block_sum(s, red);
    if (threadIdx.x == 0) loss_pm[sign] = s / (double)count;
}

// Eq. 1 and the scalar of Eq. 2: g = (l+ - l-) / (2 eps), s = -(lr g) rounded once to fp32.
__global__ void g_scalar_kernel(const double *loss_pm, float eps, float lr, double *g_out, float *s_out, uint32_t *flags)
{
    const double g = (loss_pm[0] - loss_pm[1]) / (2.0 * (double)eps);
    float s = (float)(-((double)lr * g));
    if (!(g == g) || g - g != 0.0) { s = 0.0f; atomicOr(flags, 1u); }
    *g_out = g;
    *s_out = s;
}

// ------------------------------------------------------------------ launchers
#define ZO_DISPATCH_DT(dtype, CALL)                  \
    switch (dtype) {                                 \
    case kFP32: { constexpr int DT = kFP32; CALL; } break; \
    case kBF16: { constexpr int DT = kBF16; CALL; } break; \
    case kFP16: { constexpr int DT = kFP16; CALL; } break; \
    default: return hipErrorInvalidValue;            \
    }

hipError_t launch_embed(const int32_t *tokens, const void *e_p, const void *e_m, const void *pos_p, const void *pos_m,
                        void *resid, int32_t *target, uint32_t *flags, int dtype, int n_sign, int batch, int seq, int d,
                        int vocab, hipStream_t s)
{
    const dim3 grid(n_sign * batch * seq), block(256);
    ZO_DISPATCH_DT(dtype, (embed_kernel<DT><<<grid, block, 0, s>>>(tokens, e_p, e_m, pos_p, pos_m, resid, target, flags,
                                                                   batch, seq, d, vocab)));
    return hipGetLastError();
}

hipError_t launch_layernorm(const void *resid, const void *g_p, const void *g_m, const void *b_p, const void *b_m,
                            void *y, int dtype, int n_sign, int m_half, int d, float eps, hipStream_t s)
{
    const int rows = n_sign * m_half;
    if (dtype != kFP32 && d % 4 == 0 && d <= 12288) {
        const dim3 wgrid((rows + 3) / 4), wblock(256);
#define ZO_LNW(DT, NV)                                                                                                        \
    layernorm_wave_kernel<DT, NV><<<wgrid, wblock, 0, s>>>((const float *)resid, (const uint16_t *)g_p, (const uint16_t *)g_m, \
                                                           (const uint16_t *)b_p, (const uint16_t *)b_m, (uint16_t *)y, rows,   \
                                                           m_half, d, eps)
#define ZO_LNB(DT, NV)                                                                                                        \
    layernorm_block_kernel<DT, NV><<<dim3(rows), dim3(256), 0, s>>>((const float *)resid, (const uint16_t *)g_p,              \
                                                                    (const uint16_t *)g_m, (const uint16_t *)b_p,             \
                                                                    (const uint16_t *)b_m, (uint16_t *)y, m_half, d, eps)
#define ZO_LNW_D(DT)                          \
    if (d <= 1024) ZO_LNW(DT, 4);             \
    else if (d <= 2048) ZO_LNW(DT, 8);        \
    else if (d <= 4096) ZO_LNB(DT, 4);        \
    else if (d <= 5120) ZO_LNB(DT, 5);        \
    else if (d <= 8192) ZO_LNB(DT, 8);        \
    else ZO_LNB(DT, 12);
        if (dtype == kBF16) { ZO_LNW_D(kBF16) } else { ZO_LNW_D(kFP16) }
#undef ZO_LNB
#undef ZO_LNW_D
#undef ZO_LNW
        return hipGetLastError();
    }
    const dim3 grid(rows), block(256);
    ZO_DISPATCH_DT(dtype, (layernorm_kernel<DT><<<grid, block, 0, s>>>(resid, g_p, g_m, b_p, b_m, y, m_half, d, eps)));
    return hipGetLastError();
}

template <int DT>
static void linear_plain_launch(const void *x, const void *wt_p, const void *wt_m, const void *b_p, const void *b_m,
                                void *y, int n_sign, int m_half, int n, int k, int epi, hipStream_t s)
{
    const dim3 grid((n + 63) / 64, (m_half + 63) / 64, n_sign), block(256);
    switch (epi) {
    case 0: linear_plain_kernel<DT, 0><<<grid, block, 0, s>>>(x, wt_p, wt_m, b_p, b_m, y, m_half, n, k); break;
    case 1: linear_plain_kernel<DT, 1><<<grid, block, 0, s>>>(x, wt_p, wt_m, b_p, b_m, y, m_half, n, k); break;
    case 2: linear_plain_kernel<DT, 2><<<grid, block, 0, s>>>(x, wt_p, wt_m, b_p, b_m, y, m_half, n, k); break;
    default: linear_plain_kernel<DT, 3><<<grid, block, 0, s>>>(x, wt_p, wt_m, b_p, b_m, y, m_half, n, k); break;
    }
}

hipError_t launch_linear(const void *x, const void *wt_p, const void *wt_m, const void *b_p, const void *b_m, void *y,
                         int dtype, int n_sign, int m_half, int n, int k, int epilogue, bool allow_mfma, hipStream_t s)
{
    if (allow_mfma && dtype != kFP32 && mfma_linear_supported(m_half, n, k))
        return launch_linear_mfma(x, wt_p, wt_m, b_p, b_m, y, dtype, n_sign, m_half, n, k, epilogue, s);
    ZO_DISPATCH_DT(dtype, (linear_plain_launch<DT>(x, wt_p, wt_m, b_p, b_m, y, n_sign, m_half, n, k, epilogue, s)));
    return hipGetLastError();
}

hipError_t launch_attention(const void *qkv, void *out, int dtype, int n_seq, int seq, int n_heads, int d_head,
                            bool allow_mfma, hipStream_t s)
{
    if (allow_mfma && dtype != kFP32 && mfma_attention_supported(seq, d_head))
        return launch_attention_mfma(qkv, out, dtype, n_seq, seq, n_heads, d_head, s);
    const dim3 grid(seq, n_heads, n_seq), block(128);
    const size_t smem = (size_t)(seq + d_head + 16) * acc_bytes(dtype);
    ZO_DISPATCH_DT(dtype, (attention_plain_kernel<DT><<<grid, block, smem, s>>>(qkv, out, seq, n_heads, d_head)));
    return hipGetLastError();
}

hipError_t launch_ce_rows(const void *logits, const int32_t *target, double *row_loss, int dtype, int rows, int vocab,
                          hipStream_t s)
{
    if (rows == 0) return hipSuccess;
    if (dtype == kFP32) ce_rows_kernel<double><<<dim3(rows), dim3(256), 0, s>>>((const double *)logits, target, row_loss, vocab);
    else ce_rows_kernel<float><<<dim3(rows), dim3(256), 0, s>>>((const float *)logits, target, row_loss, vocab);
    return hipGetLastError();
}

hipError_t launch_ce_finish(const void *partials, int n_partial, const float *target_logit, const int32_t *target,
                            double *row_loss, int rows, hipStream_t s)
{
    if (rows == 0) return hipSuccess;
    ce_finish_kernel<<<dim3((rows + 3) / 4), dim3(256), 0, s>>>((const float2 *)partials, n_partial, target_logit, target, row_loss,
                                                                rows);
    return hipGetLastError();
}

hipError_t launch_loss_reduce(const double *row_loss, int n_sign, int m_half, int count_per_sign, double *loss_pm,
                              hipStream_t s)
{
    loss_reduce_kernel<<<dim3(n_sign), dim3(1024), 0, s>>>(row_loss, m_half, count_per_sign, loss_pm);
    return hipGetLastError();
}

hipError_t launch_g_scalar(const double *loss_pm, float eps, float lr, double *g_out, float *s_out, uint32_t *flags,
                           hipStream_t s)
{
    g_scalar_kernel<<<dim3(1), dim3(1), 0, s>>>(loss_pm, eps, lr, g_out, s_out, flags);
    return hipGetLastError();
}

}  // namespace zo

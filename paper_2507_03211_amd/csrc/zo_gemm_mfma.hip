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
// Two tilings:
//  * 256 x 256 x 64, 4 waves of 128 x 128 (4 x 4 MFMA tiles, 256 accumulator registers), one persistent
//    workgroup per CU that walks its XCD's share of the tile list.  Operand tiles go from global memory
//    straight into LDS (global_load_lds_dwordx4, no register staging), whole 128-byte lines per tile row; the
//    160 KiB of LDS hold three stages of the activation tile and two of the weight tile, and the pipeline
//    runs on from one tile into the next.  16-byte chunks are XOR-swizzled on the global side so that
//    fragment reads are free of bank conflicts.  Tiles are numbered so that each XCD (its own L2) owns a
//    contiguous band of 8 tile-rows and walks it column by column.  Outputs leave through LDS as whole rows.
//  * 128 x 128 x 64, 4 waves of 64 x 64, register-staged double buffer: for shapes with fewer than 128
//    256-tiles, K below three slabs, and ragged small cases.
#include "zo_kernels.h"
#include "zo_types.hip.h"

namespace zo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vector: arrays of it stay in registers
typedef float f32x4 __attribute__((ext_vector_type(4)));

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


// One lane's run of 4 consecutive n of one output row.
template <int DT, int EPI>
__device__ __forceinline__ void epilogue_store(float (&v)[4], const uint16_t *__restrict__ bias, void *__restrict__ y, size_t row,
                                               int n, int nc)
{
    if constexpr (EPI != 3) {
        const uint2 braw = *(const uint2 *)(bias + nc);
        const uint16_t bb[4] = {(uint16_t)(braw.x & 0xffff), (uint16_t)(braw.x >> 16), (uint16_t)(braw.y & 0xffff),
                                (uint16_t)(braw.y >> 16)};
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


// Epilogue 4 (tied LM head fused with the cross-entropy reduction): nothing of the logits is stored.  A lane
// holds TN * 16 logits of one row (4 runs of 4 consecutive columns per MFMA tile); it reduces them to a
// (maximum, sum of exp) pair, merges with the other lane half (the remaining columns of the wave's range)
// and the wave writes one pair per row and per wave-column-range; the lane that holds the target column
// stores that logit.  A last small kernel merges the pairs of a row into logsumexp - target logit.
// Argument reuse for this epilogue: bias_p -> int32 target[rows], bias_m -> float target_logit[rows],
// y -> float2 partial[rows][n_partial].
template <int TN>
__device__ __forceinline__ void ce_partial_row(const f32x16 (&a)[TN], int col0, int fh, int n, bool live, int tg,
                                               float *tgt_logit_row, float2 *partial_slot)
{
    // `live` false: a row past the ragged end of the tile.  It takes part (the two halves of the wave exchange their
    // results below) and stores nothing; its pointers are those of the last valid row.
    //
    // A lane's 16 TN logits in register order k = 16 tn + i sit at columns col0 + 32 tn + 8 (i / 4) + 4 fh + i % 4,
    // which grow with k.  Nothing here keeps one compare result per element alive (64 of them, the same for every
    // row block, is what the compiler would hoist and then spill): the ragged strip of the vocabulary is masked by
    // arithmetic, the target logit is picked by a tree of selects on the bits of its register number.
    constexpr int NE = 16 * TN;
    float v[NE];
#pragma unroll
    for (int k = 0; k < NE; ++k) v[k] = a[k / 16][k % 16];
    if (col0 + 32 * TN > n) {                      // wave-uniform: only the last strip of the vocabulary
        // number of this lane's registers that lie inside the vocabulary
        int kmax = 0;
#pragma unroll
        for (int g = 0; g < 4 * TN; ++g) {         // runs of 4 columns: col0 + 32 (g / 4) + 8 (g % 4) + 4 fh + 0..3
            const int c0 = col0 + 32 * (g / 4) + 8 * (g % 4) + 4 * fh, left = n - c0;
            kmax += left < 0 ? 0 : left > 4 ? 4 : left;
        }
        const float kf = (float)kmax - 0.5f;
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            // (kf - k) * inf is +inf for registers inside, -inf outside (never 0 * inf); min(., 0) makes it 0 or -inf
            const float pen = __builtin_fminf((kf - (float)k) * INFINITY, 0.0f);
            v[k] += pen;
        }
    }
    float mx = v[0];
#pragma unroll
    for (int k = 1; k < NE; ++k) mx = __builtin_fmaxf(mx, v[k]);
    const float ms = mx > -INFINITY ? mx : 0.0f;      // a strip that lies wholly past the vocabulary: exp(-inf - 0) = 0
    float sum = 0.0f;
#pragma unroll
    for (int k = 0; k < NE; ++k) sum += __expf(v[k] - ms);
    // the target column, if it is one of this lane's: register 16 (rel / 32) + 4 (rel / 8 % 4) + rel % 4 of the lane
    // half rel / 4 % 2
    const int rel = tg - col0;
    const bool mine = rel >= 0 && rel < 32 * TN && ((rel >> 2) & 1) == fh;
    const int which = (rel >> 5) * 16 + ((rel >> 3) & 3) * 4 + (rel & 3);
    float t[NE];
#pragma unroll
    for (int k = 0; k < NE; ++k) t[k] = v[k];
#pragma unroll
    for (int bit = 0, cnt = NE; cnt > 1; ++bit, cnt >>= 1) {
        const bool odd = (which >> bit) & 1;
#pragma unroll
        for (int k = 0; k < cnt / 2; ++k) t[k] = odd ? t[2 * k + 1] : t[2 * k];
    }
    if (live && mine) *tgt_logit_row = t[0];
    const float mo = __shfl_xor(mx, 32, 64), so = __shfl_xor(sum, 32, 64);
    const float m2 = mx > mo ? mx : mo;
    const float s2 = (mx > -INFINITY ? sum * __expf(mx - m2) : 0.0f) + (mo > -INFINITY ? so * __expf(mo - m2) : 0.0f);
    if (live && fh == 0) *partial_slot = float2{m2, s2};
}

// LDS tile: [rows][8 chunks] of uint4, chunk c of row r stored at c ^ ((r >> 1) & 7): the LDS has 64
// four-byte banks, so 16 lanes (16 consecutive rows, one logical chunk) must land on 16 distinct 16-byte
// positions of a 256-byte window, i.e. on distinct (row parity, slot) pairs.
__device__ __forceinline__ int lds_slot(int r, int c) { return r * kChunksPerRow + (c ^ ((r >> 1) & 7)); }

template <int DT, int EPI>
__global__ __launch_bounds__(256) void linear_mfma_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ wt_p,
                                                          const uint16_t *__restrict__ wt_m, const uint16_t *__restrict__ b_p,
                                                          const uint16_t *__restrict__ b_m, void *__restrict__ y,
                                                          int m_half, int n, int k)
{
    __shared__ u32x4 xs[2][BM * kChunksPerRow];
    __shared__ u32x4 ws[2][BN * kChunksPerRow];
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
    u32x4 xreg[4], wreg[4];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            xreg[i] = *(const u32x4 *)(xg[i] + k0);
            wreg[i] = *(const u32x4 *)(wg[i] + k0);
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
                wf[t] = __builtin_bit_cast(uint4, ws[buf][lds_slot(wn * 64 + t * 32 + fr, ks * 2 + fh)]);
                xf[t] = __builtin_bit_cast(uint4, xs[buf][lds_slot(wm * 64 + t * 32 + fr, ks * 2 + fh)]);
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
    if constexpr (EPI == 4) {
        const int n_partial = 2 * (int)gridDim.x;
#pragma unroll
        for (int tm = 0; tm < 2; ++tm) {
            const int mr = m0 + wm * 64 + tm * 32 + fr;
            const size_t row = (size_t)sign * m_half + (mr < m_half ? mr : m_half - 1);
            const f32x16 a[2] = {acc[0][tm], acc[1][tm]};
            ce_partial_row<2>(a, n0 + wn * 64, fh, n, mr < m_half, ((const int32_t *)b_p)[row], (float *)b_m + row,
                              (float2 *)y + row * n_partial + (blockIdx.x * 2 + wn));
        }
        return;
    }
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
                epilogue_store<DT, EPI>(v, bias, y, row, n, nc);
            }
        }
    }
}

// ------------------------------------------------------------------ 256 x 256 x 64 tiling
namespace big {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int STX = 3, STW = 2;                 // LDS stages of the activation tile / of the weight tile
constexpr int kTileU4 = BM * (BK / 8);          // uint4 per operand tile (2048 = 32 KiB)
constexpr int kLdsBytes = (STX + STW) * kTileU4 * 16;   // 160 KiB: all of a CU's LDS
constexpr int kGroupM = 8;                      // tile-rows per band

// 16 bytes per lane from global memory straight into LDS: lane L lands at lds_off + 16 L.
// Issued from asm so that the waits are ours: the compiler would otherwise drain every
// outstanding load before the next LDS read, which defeats the overlap.
// The address is a wave-uniform 64-bit base (scalar registers: the k advance of the pipeline costs no vector
// instruction) plus a 32-bit per-lane byte offset that stays the same for the whole tile.
__device__ __forceinline__ void gload_lds16(uint64_t base, uint32_t lane_off, uint32_t lds_off)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_off) : "memory", "m0");
}
__device__ __forceinline__ uint64_t uniform64(uint64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

template <int DT, int EPI>
__global__ __launch_bounds__(256) void linear_mfma256_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ wt_p,
                                                             const uint16_t *__restrict__ wt_m, const uint16_t *__restrict__ b_p,
                                                             const uint16_t *__restrict__ b_m, void *__restrict__ y, int m_half,
                                                             int n, int k, int n_sign, int tiles_m, int tiles_n, int total)
{
    extern __shared__ __attribute__((aligned(16))) uint4 smem[];
    // Persistent workgroups, one per CU: the hardware deals consecutive workgroup ids round-robin to the 8 XCDs,
    // so workgroup b sits on XCD b % 8 and is that XCD's slot b / 8; it walks the XCD's contiguous share of the
    // tile list, slot, slot + slots, ...  The software pipeline does not stop between tiles: while the last two
    // slabs of a tile are multiplied the first two slabs of the next tile are already being loaded, and they land
    // during the epilogue.
    const int per_xcd = (total + 7) / 8, slots = (int)gridDim.x / 8;
    const int xcd = (int)blockIdx.x % 8, slot0 = (int)blockIdx.x / 8;
    auto tile_lin = [&](int it) {                                   // -1: no such tile
        const int sl = slot0 + slots * it, lin = xcd * per_xcd + sl;
        return (sl < per_xcd && lin < total) ? lin : -1;
    };
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int rows_total = n_sign * tiles_m;            // tile-rows over both signs

    // Load assignment: one wave instruction moves 8 tile rows x 128 bytes (whole cache lines); wave w,
    // instruction i covers rows (8 w + i) * 8 .. + 7; lane -> (row, 16-byte slot).  The slot holds logical
    // chunk slot ^ (row / 2 mod 8): 16 consecutive rows of one logical chunk then sit on 16 distinct
    // 16-byte positions of the 64-bank (256-byte wide) LDS, so fragment reads are conflict-free.
    const int lrow = lane >> 3, lslot = lane & 7;
    struct Tile {
        int sign, m0, n0, tcol;
        uint64_t xbase, wbase;          // first row of the tile in x / in the sign's weights (wave-uniform)
        uint32_t xg[8], wg[8];          // byte offsets of this lane's 8 + 8 loads from those (clamped at ragged edges)
    };
    auto setup = [&](int lin, Tile &t) {
        const int band = lin / (kGroupM * tiles_n), rem = lin % (kGroupM * tiles_n);
        const int band_rows = rows_total - band * kGroupM < kGroupM ? rows_total - band * kGroupM : kGroupM;
        const int trow = band * kGroupM + rem % band_rows;
        t.tcol = rem / band_rows;
        t.sign = trow / tiles_m;
        t.m0 = (trow % tiles_m) * BM;
        t.n0 = t.tcol * BN;
        const uint16_t *xa = x + (size_t)t.sign * m_half * k;
        const uint16_t *wt = t.sign ? wt_m : wt_p;
        t.xbase = uniform64((uint64_t)(uintptr_t)(xa + (size_t)t.m0 * k));
        t.wbase = uniform64((uint64_t)(uintptr_t)(wt + (size_t)t.n0 * k));
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = (wave * 8 + i) * 8 + lrow;
            const int chunk = lslot ^ ((row >> 1) & 7);
            int xr = t.m0 + row; xr = xr < m_half ? xr : m_half - 1;       // clamp: masked at the store
            int wr = t.n0 + row; wr = wr < n ? wr : n - 1;
            t.xg[i] = ((uint32_t)(xr - t.m0) * (uint32_t)k + chunk * 8) * 2u;
            t.wg[i] = ((uint32_t)(wr - t.n0) * (uint32_t)k + chunk * 8) * 2u;
        }
    };
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)smem;
    const int nk = k / BK;                              // >= 3 (the launcher sees to it)
    // Slabs are numbered through all the tiles of this workgroup.  x slab g lives in x stage g % 3, w slab g in w
    // stage g % 2 (after the three x stages); the stages of slabs g, g+1, g+2 are kept as rotating scalars (uint4
    // index into smem) instead of being worked out from g every time.
    constexpr uint32_t kStage = kTileU4;                 // uint4 per stage
    uint32_t xs0 = 0, xs1 = kStage, xs2 = 2 * kStage;    // x stages of slabs g, g+1, g+2
    uint32_t ws0 = STX * kStage, ws1 = (STX + 1) * kStage;   // w stages of slabs g (and g+2), g+1
    auto lds_of = [&](uint32_t stage) { return lds_base + stage * 16u + (uint32_t)wave * 8192u; };   // this wave's slice

    f32x16 acc[4][4];
    const int fr = lane & 31, fh = lane >> 5, sw = (fr >> 1) & 7;
    const int xrow = (wm * 128 + fr) * 8, wrow = (wn * 128 + fr) * 8;     // uint4 index of the lane's first rows
    uint4 wfa[4], xfa[4], wfb[4], xfb[4];                                 // two fragment sets: one multiplies while one loads
    // One fragment of set (wf, xf) for k-step ks of the slab in stages (xst, wst), in the order the multiplies need them:
    // wf0, xf0, xf1, xf2, xf3, wf1, wf2, wf3.
    auto frag1 = [&](uint32_t xst, uint32_t wst, int ks, int idx, uint4 (&wf)[4], uint4 (&xf)[4]) {
        const uint4 *xs = smem + xst;
        const uint4 *ws = smem + wst;
        const int slot = (2 * ks + fh) ^ sw;
        if (idx == 0) wf[0] = ws[wrow + slot];
        else if (idx <= 4) xf[idx - 1] = xs[xrow + (idx - 1) * 256 + slot];
        else wf[idx - 4] = ws[wrow + (idx - 4) * 256 + slot];
    };
    // Multiplies j0 .. j1-1 of the 4 x 4 fragment product of set (wf, xf).  Before multiply j:
    //  * fragments rper (j - rj0) / revery .. + rper - 1 of set (nwf, nxf) are read for k-step nks of the slab in
    //    stages (nxst, nwst), when that divides;
    //  * load lfirst + (j - lj0) / levery (lane offsets `offs` from the scalar base `gbase`) goes out into LDS at
    //    `st`, when that divides, `nload` in all.
    //  `first`: the product starts the accumulators (first quarter of a tile's first slab) instead of adding to them.
    auto mma_rl = [&](const uint4 (&wf)[4], const uint4 (&xf)[4], int j0, int j1, uint4 (&nwf)[4], uint4 (&nxf)[4], uint32_t nxst,
                      uint32_t nwst, int nks, int rj0, int revery, int rper, const uint32_t (&offs)[8], uint64_t gbase, uint32_t st,
                      int lfirst, int nload, int lj0, int levery, bool first = false) {
#pragma unroll
        for (int j = j0; j < j1; ++j) {
            if (j >= rj0 && (j - rj0) % revery == 0 && (j - rj0) / revery * rper < 8) {
#pragma unroll
                for (int r = 0; r < rper; ++r) frag1(nxst, nwst, nks, (j - rj0) / revery * rper + r, nwf, nxf);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (j >= lj0 && (j - lj0) % levery == 0 && (j - lj0) / levery < nload) {
                const int q = lfirst + (j - lj0) / levery;
                gload_lds16(gbase, offs[q], st + q * 1024u);
                __builtin_amdgcn_sched_barrier(0);
            }
            // back and forth over the activation fragments, so that one operand changes from one multiply to
            // the next, not both (a little less switching on a chip whose clock is set by its power)
            const int xi = ((j >> 2) & 1) ? 3 - (j & 3) : (j & 3);
            if (first) {
                f32x16 zero;
#pragma unroll
                for (int i = 0; i < 16; ++i) zero[i] = 0.0f;
                acc[j >> 2][xi] = mfma32<DT>(wf[j >> 2], xf[xi], zero);
            } else {
                acc[j >> 2][xi] = mfma32<DT>(wf[j >> 2], xf[xi], acc[j >> 2][xi]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // Software pipeline.  The 160 KiB of LDS hold three stages of the activation tile and two of the weight
    // tile, so half of every slab's loads are issued two slab-times ahead and only the other half one ahead:
    // with a single slab of lookahead for everything the multiplies wait on memory latency.  One wave per SIMD
    // means nothing else hides an instruction that is slow to issue, so neither the global->LDS loads nor the
    // LDS fragment reads come in bursts: each sits alone between two multiplies and issues while the matrix
    // pipe works on the one before.  The fragments of a quarter slab (16 multiplies) are read during the quarter
    // before it, into the set of registers the quarter before that used.  The barrier sits in the middle of
    // the third quarter, once this wave's last LDS reads of slab g are in registers.
    // sched_barrier(0) pins the order (the compiler would sink each LDS read down to its first use).
    //
    // One slab: multiplies slab g (fragment set A holds its first quarter), loads slab g + 2 from (xb, wb) with
    // the lane offsets (xo, wo).  x(g+2) goes into the activation stage that slab g-1 left at the previous barrier:
    // its 8 loads sit under the 40 multiplies before this slab's barrier; w(g+2) can only follow the barrier: its
    // 8 loads sit under the 24 multiplies after it.
    auto slab = [&](uint64_t xb, uint64_t wb, const uint32_t (&xo)[8], const uint32_t (&wo)[8], bool first) {
        const uint32_t stx = lds_of(xs2), stw = lds_of(ws0);
        mma_rl(wfa, xfa, 0, 16, wfb, xfb, xs0, ws0, 1, 1, 2, 1, xo, xb, stx, 0, 3, 0, 6, first);
        mma_rl(wfb, xfb, 0, 16, wfa, xfa, xs0, ws0, 2, 1, 2, 1, xo, xb, stx, 3, 3, 0, 6);
        // the last fragments of slab g, two reads at a time, so that they have landed when the barrier's wait comes
        mma_rl(wfa, xfa, 0, 8, wfb, xfb, xs0, ws0, 3, 0, 1, 2, xo, xb, stx, 6, 2, 4, 2);
        // slab g+1 landed (only x(g+2), the 8 newest loads, may still be out); slab g fully in registers
        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        mma_rl(wfa, xfa, 8, 16, wfb, xfb, xs0, ws0, 3, 99, 1, 1, wo, wb, stw, 0, 3, 8, 3);
        // the first fragments of slab g+1 early in the quarter: the loop's back edge waits for all LDS reads
        mma_rl(wfb, xfb, 0, 16, wfa, xfa, xs1, ws1, 0, 0, 1, 1, wo, wb, stw, 3, 5, 0, 3);
        // on to the next slab: the stage this one leaves is the one that slab g+3 will be loaded into
        const uint32_t tx = xs0, tw = ws0;
        xs0 = xs1; xs1 = xs2; xs2 = tx;
        ws0 = ws1; ws1 = tw;
    };

    Tile cur, nxt;
    int lin = tile_lin(0);
    if (lin < 0) return;
    setup(lin, cur);
    int it = 0;                                         // tile number of this workgroup
    // prologue of the first tile only: slabs 0 and 1, fragments of the first quarter
#pragma unroll
    for (int i = 0; i < 8; ++i) gload_lds16(cur.xbase, cur.xg[i], lds_of(xs0) + i * 1024u);
#pragma unroll
    for (int i = 0; i < 8; ++i) gload_lds16(cur.wbase, cur.wg[i], lds_of(ws0) + i * 1024u);
#pragma unroll
    for (int i = 0; i < 8; ++i) gload_lds16(cur.xbase + 2u * BK, cur.xg[i], lds_of(xs1) + i * 1024u);
#pragma unroll
    for (int i = 0; i < 8; ++i) gload_lds16(cur.wbase + 2u * BK, cur.wg[i], lds_of(ws1) + i * 1024u);
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");               // slab 0 landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int idx = 0; idx < 8; ++idx) frag1(xs0, ws0, 0, idx, wfa, xfa);

    for (;;) {
        const int lin_next = tile_lin(it + 1);
        const bool has_next = lin_next >= 0;
        if (has_next) {
            setup(lin_next, nxt);
        } else {
            // no successor: the two slabs loaded ahead are this tile's last two over again, which nothing reads
            nxt = cur;
            nxt.xbase += 2u * (uint32_t)((nk - 2) * BK);
            nxt.wbase += 2u * (uint32_t)((nk - 2) * BK);
        }
        // all slabs but the last two load two slabs ahead in this tile; the first one starts the accumulators
        slab(cur.xbase + 2u * (uint32_t)(2 * BK), cur.wbase + 2u * (uint32_t)(2 * BK), cur.xg, cur.wg, true);
        for (int kt = 1; kt < nk - 2; ++kt)
            slab(cur.xbase + 2u * (uint32_t)((kt + 2) * BK), cur.wbase + 2u * (uint32_t)((kt + 2) * BK), cur.xg, cur.wg, false);
        // the last two load the first two slabs of the next tile
        slab(nxt.xbase, nxt.wbase, nxt.xg, nxt.wg, false);
        slab(nxt.xbase + 2u * BK, nxt.wbase + 2u * BK, nxt.xg, nxt.wg, false);

        // ---- epilogue of tile `cur`
        const int sign = cur.sign, m0 = cur.m0, n0 = cur.n0;
        const uint16_t *bias = sign ? b_m : b_p;
        if constexpr (EPI == 4) {
            const int n_partial = 2 * tiles_n;
#pragma unroll
            for (int tm = 0; tm < 4; ++tm) {
                const int mr = m0 + wm * 128 + tm * 32 + fr;
                const size_t row = (size_t)sign * m_half + (mr < m_half ? mr : m_half - 1);
                const f32x16 a[4] = {acc[0][tm], acc[1][tm], acc[2][tm], acc[3][tm]};
                ce_partial_row<4>(a, n0 + wn * 128, fh, n, mr < m_half, ((const int32_t *)b_p)[row], (float *)b_m + row,
                                  (float2 *)y + row * n_partial + (cur.tcol * 2 + wn));
            }
        } else {
            // Output through LDS so that global stores are whole rows: in the MFMA layout a lane holds runs of 4
            // consecutive columns of ONE row and a wave instruction would touch 32 rows with 16 or 32 bytes each.
            // A wave stages 8 KiB at a time (32 rows x 128 two-byte columns, or 16 rows of fp32) in its own slice
            // of the activation stage that the tile's last slab has just left: every wave finished reading that
            // stage before the slab's barrier, and the next loads into the slice are this wave's own, issued after
            // the epilogue.  No workgroup barrier.  XOR-swizzled so that both the run-wise writes and the row-wise
            // 16-byte reads are free of bank conflicts.
            constexpr bool kOut16 = (EPI == 0 || EPI == 1);              // 2-byte outputs; else fp32
            constexpr int RP = kOut16 ? 32 : 16;                         // rows per pass
            constexpr int NPASS = 128 / RP;
            char *stage = (char *)(smem + xs2) + wave * 8192;        // xs2: the stage the tile's last slab has just left
            const int ncol0 = n0 + wn * 128;
            // Bias: 2-byte outputs take it before the rounding, so per run of the MFMA layout (the same 16 runs
            // for every row block); fp32 outputs take it after the LDS pass, where a lane always holds the same
            // 4 columns.
            // They come through the scalar cache (a wave-uniform address in the constant address space: 16 bytes
            // = the 8 columns of a run pair, of which the lane half keeps its 4): a vector load here would make
            // the compiler wait for every outstanding vector memory operation, the next tile's loads included.
            float bvals[kOut16 ? 4 : 1][4][4];
            if constexpr (kOut16) {
                typedef const __attribute__((address_space(4))) u32x4 *cptr;
                const uint64_t bbase = uniform64((uint64_t)(uintptr_t)bias);
#pragma unroll
                for (int tn = 0; tn < 4; ++tn)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        int c8 = ncol0 + tn * 32 + 8 * g;               // wave-uniform; clamped: columns >= n are never stored
                        c8 = c8 + 8 <= n ? c8 : n - 8;
                        const u32x4 raw = *(cptr)(uintptr_t)(bbase + 2u * (uint32_t)c8);
                        const uint32_t lo = fh ? raw.z : raw.x, hi = fh ? raw.w : raw.y;
                        bvals[tn][g][0] = Prec<DT>::w2f((uint16_t)(lo & 0xffff));
                        bvals[tn][g][1] = Prec<DT>::w2f((uint16_t)(lo >> 16));
                        bvals[tn][g][2] = Prec<DT>::w2f((uint16_t)(hi & 0xffff));
                        bvals[tn][g][3] = Prec<DT>::w2f((uint16_t)(hi >> 16));
                    }
            }
            // Residual epilogue: the 8 reads of the running sum that a pass needs are all issued one pass ahead
            // (a load may not overtake an earlier store that the compiler cannot tell apart from it).  Reading
            // further ahead (two passes, which is what the registers allow) changes nothing: what the tile waits
            // for is the bandwidth of all workgroups' read-modify-write bursts arriving together, not one latency.
            float4 hres[2][8];
            auto load_res = [&](int pass, float4 (&h)[8]) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int r = 2 * i + (lane >> 5), c = lane & 31;
                    const int mr = m0 + wm * 128 + pass * 16 + r, nc = ncol0 + c * 4;
                    h[i] = float4{0.f, 0.f, 0.f, 0.f};
                    if (mr < m_half && nc < n) {
                        // read once, written once: neither the running sum nor any output is worth an L2 line that
                        // an operand slab could keep (non-temporal loads and stores)
                        const f32x4 t = __builtin_nontemporal_load((const f32x4 *)((const float *)y + ((size_t)sign * m_half + mr) * n + nc));
                        h[i] = float4{t.x, t.y, t.z, t.w};
                    }
                }
            };
            float bias4[4] = {0.f, 0.f, 0.f, 0.f};
            if constexpr (EPI == 2) {
                load_res(0, hres[0]);
                const int nc = ncol0 + (lane & 31) * 4;
                if (nc < n) {
                    const uint2 braw = *(const uint2 *)(bias + nc);
                    bias4[0] = Prec<DT>::w2f((uint16_t)(braw.x & 0xffff));
                    bias4[1] = Prec<DT>::w2f((uint16_t)(braw.x >> 16));
                    bias4[2] = Prec<DT>::w2f((uint16_t)(braw.y & 0xffff));
                    bias4[3] = Prec<DT>::w2f((uint16_t)(braw.y >> 16));
                }
            }
#pragma unroll
            for (int pass = 0; pass < NPASS; ++pass) {
                const int tm = pass * RP / 32;                          // MFMA row block of this pass
                if constexpr (EPI == 2) {
                    if (pass + 1 < NPASS) load_res(pass + 1, hres[(pass + 1) & 1]);
                }
                // fp32: the pass covers rows 16 (pass % 2) .. + 15 of the block, held by the lanes with that fr / 16
                if (kOut16 || (fr >> 4) == (pass & 1)) {
#pragma unroll
                    for (int tn = 0; tn < 4; ++tn)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            float v[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                v[e] = acc[tn][tm][4 * g + e];
                                if constexpr (kOut16) v[e] += bvals[tn][g][e];
                                if constexpr (EPI == 1) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
                            }
                            const int run = tn * 8 + 2 * g + fh;         // which run of 4 columns (0..31) of the row
                            if constexpr (kOut16) {
                                // two outputs per conversion instruction (round to nearest even, as the single one does)
                                auto pack2 = [](float lo, float hi) {
                                    const f32x2 pr = {lo, hi};
                                    if constexpr (DT == kBF16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
                                    else return __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, f16x2));
                                };
                                uint2 o;
                                o.x = pack2(v[0], v[1]);
                                o.y = pack2(v[2], v[3]);
                                *(uint2 *)(stage + fr * 256 + ((run ^ fr) << 3)) = o;      // 8-byte slots, XOR by the row
                            } else {
                                *(float4 *)(stage + (fr & 15) * 512 + ((run ^ (fr & 15)) << 4)) = float4{v[0], v[1], v[2], v[3]};
                            }
                        }
                }
                const int mbase = m0 + wm * 128 + pass * RP;
                asm volatile("" ::: "memory");      // the wave's LDS operations execute in order; keep the compiler to it too
                if constexpr (kOut16) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int r = 4 * i + (lane >> 4), c16 = lane & 15;           // 16 lanes x 16 bytes = one 256-byte row
                        uint4 q = *(const uint4 *)(stage + r * 256 + ((c16 ^ (r >> 1)) << 4));
                        if (r & 1) q = uint4{q.z, q.w, q.x, q.y};                    // odd rows hold the two runs swapped
                        const int mr = mbase + r, nc = ncol0 + c16 * 8;
                        if (mr < m_half && nc < n) __builtin_nontemporal_store(__builtin_bit_cast(u32x4, q), (u32x4 *)((uint16_t *)y + ((size_t)sign * m_half + mr) * n + nc));
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int r = 2 * i + (lane >> 5), c = lane & 31;             // 32 lanes x 16 bytes = one 512-byte row
                        const float4 q = *(const float4 *)(stage + r * 512 + ((c ^ r) << 4));
                        const int mr = mbase + r, nc = ncol0 + c * 4;
                        if (mr < m_half && nc < n) {
                            float4 *p = (float4 *)((float *)y + ((size_t)sign * m_half + mr) * n + nc);
                            if constexpr (EPI == 2) {
                                float4 h = hres[pass & 1][i];
                                h.x += q.x + bias4[0]; h.y += q.y + bias4[1]; h.z += q.z + bias4[2]; h.w += q.w + bias4[3];
                                __builtin_nontemporal_store(f32x4{h.x, h.y, h.z, h.w}, (f32x4 *)p);
                            } else {
                                *p = q;
                            }
                        }
                    }
                }
                asm volatile("" ::: "memory");
            }
        }
        if (!has_next) break;
        cur = nxt;
        ++it;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                 // the tail loads land before LDS is released
}

}  // namespace big

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
    case 4: ZO_L(4); break;
    default: ZO_L(3); break;
    }
#undef ZO_L
}

template <int DT>
hipError_t launch_big_t(const void *x, const void *wt_p, const void *wt_m, const void *b_p, const void *b_m, void *y, int n_sign,
                        int m_half, int n, int k, int epi, hipStream_t s)
{
    const int tiles_m = (m_half + big::BM - 1) / big::BM, tiles_n = (n + big::BN - 1) / big::BN;
    const int total = n_sign * tiles_m * tiles_n;
    // persistent workgroups: one per CU (the 160 KiB of LDS allow no second one), a multiple of the 8 XCDs
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        n_cu = v >= 8 ? v / 8 * 8 : 8;
    }
    const int want = (total + 7) / 8 * 8;
    const dim3 grid(want < n_cu ? want : n_cu), block(256);
#define ZO_B(E)                                                                                                                  \
    {                                                                                                                            \
        auto kern = big::linear_mfma256_kernel<DT, E>;                                                                           \
        static bool attr_set = false;                                                                                            \
        if (!attr_set) {                                                                                                         \
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, big::kLdsBytes);  \
            if (e != hipSuccess) return e;                                                                                       \
            attr_set = true;                                                                                                     \
        }                                                                                                                        \
        kern<<<grid, block, big::kLdsBytes, s>>>((const uint16_t *)x, (const uint16_t *)wt_p, (const uint16_t *)wt_m,            \
                                                 (const uint16_t *)b_p, (const uint16_t *)b_m, y, m_half, n, k, n_sign, tiles_m,  \
                                                 tiles_n, total);                                                                         \
    }
    switch (epi) {
    case 0: ZO_B(0) break;
    case 1: ZO_B(1) break;
    case 2: ZO_B(2) break;
    case 4: ZO_B(4) break;
    default: ZO_B(3) break;
    }
#undef ZO_B
    return hipGetLastError();
}

// The big tiling pays once its tiles occupy about half of the 256 CUs: measured at 192 tiles it is 1.5 times as
// fast as the small tiling although a quarter of the CUs idle.
bool use_big(int n_sign, int m_half, int n, int k)
{
    if (k % big::BK || k < 3 * big::BK) return false;      // the pipeline runs two slabs ahead, and the first slab of a tile is special
    const long tiles = (long)n_sign * ((m_half + big::BM - 1) / big::BM) * ((n + big::BN - 1) / big::BN);
    return tiles >= 128;
}

}  // namespace

int mfma_ce_partials(int n_sign, int m_half, int n, int k)
{
    return use_big(n_sign, m_half, n, k) ? 2 * ((n + big::BN - 1) / big::BN) : 2 * ((n + BN - 1) / BN);
}

bool mfma_linear_supported(int m_half, int n, int k) { return m_half >= 1 && n >= 8 && n % 8 == 0 && k >= BK && k % BK == 0; }

hipError_t launch_linear_mfma(const void *x, const void *wt_p, const void *wt_m, const void *b_p, const void *b_m, void *y,
                              int dtype, int n_sign, int m_half, int n, int k, int epilogue, hipStream_t s)
{
    if (!mfma_linear_supported(m_half, n, k) || (dtype != kBF16 && dtype != kFP16)) return hipErrorInvalidValue;
    // 16-byte pieces everywhere (operand loads, row-wise stores, bias through the scalar cache)
    if ((uintptr_t)x % 16 || (uintptr_t)wt_p % 16 || (uintptr_t)wt_m % 16 || (uintptr_t)y % 16) return hipErrorInvalidValue;
    if (epilogue != 3 && epilogue != 4 && ((uintptr_t)b_p % 16 || (uintptr_t)b_m % 16)) return hipErrorInvalidValue;
    if (use_big(n_sign, m_half, n, k)) {
        return dtype == kBF16 ? launch_big_t<kBF16>(x, wt_p, wt_m, b_p, b_m, y, n_sign, m_half, n, k, epilogue, s)
                              : launch_big_t<kFP16>(x, wt_p, wt_m, b_p, b_m, y, n_sign, m_half, n, k, epilogue, s);
    }
    if (dtype == kBF16) launch_t<kBF16>(x, wt_p, wt_m, b_p, b_m, y, n_sign, m_half, n, k, epilogue, s);
    else launch_t<kFP16>(x, wt_p, wt_m, b_p, b_m, y, n_sign, m_half, n, k, epilogue, s);
    return hipGetLastError();
}

}  // namespace zo

// Perturb / update streams (DistZO2 App. A, Alg. 1: PerturbParameters and UpdateParameters;
// Eq. 2) and the out-of-place staging of W+- = rn(theta +- eps z) (PertP workflow, Step 2).
//
// All of them are one pass over the parameters with z regenerated in registers from its
// counter: 16-byte coalesced loads and stores, independent Philox blocks per thread for
// instruction-level parallelism.  The normal transform reads its radius from a 24 KiB table in
// LDS, so the workgroups are persistent: a few per CU, each filling the table once and then
// walking chunks (tiles) blockIdx.x, blockIdx.x + gridDim.x, ...
#include <type_traits>

#include "zo_kernels.h"
#include "zo_rng.hip.h"
#include "zo_types.hip.h"

namespace zo {

// ------------------------------------------------------------------ z only (verification)
__global__ __launch_bounds__(256) void z_kernel(float *out, uint64_t n, uint64_t seed, uint32_t tid, uint64_t first)
{
    __shared__ float4 ln_tab[kRayleighLast];
    load_rayleigh_cells(ln_tab);
    // one Philox block per thread; blocks first/4 .. (first+n-1)/4
    const uint64_t j = first / 4 + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (4 * j >= first + n) return;
    float z[4];
    normal4(philox_block(seed, tid, j), z, ln_tab);
#pragma unroll
    for (int l = 0; l < 4; ++l) {
        const uint64_t i = 4 * j + l;
        if (i >= first && i < first + n) out[i - first] = z[l];
    }
}

__global__ __launch_bounds__(256) void normal_pairs_kernel(const uint32_t *words, float *z, uint64_t n_pairs)
{
    __shared__ float4 ln_tab[kRayleighLast];
    load_rayleigh_cells(ln_tab);
    const uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n_pairs) return;
    float a, b;
    normal_pair(words[2 * p], words[2 * p + 1], a, b, ln_tab);
    z[2 * p] = a;
    z[2 * p + 1] = b;
}

// ------------------------------------------------------------------ in-place axpy with z
template <int DT> struct Vec16;   // 16 bytes of storage elements
template <> struct Vec16<kFP32> { static constexpr int N = 4; };
template <> struct Vec16<kBF16> { static constexpr int N = 8; };
template <> struct Vec16<kFP16> { static constexpr int N = 8; };

template <int DT> __device__ __forceinline__ void unpack16(const uint4 &v, float *f)
{
    if constexpr (DT == kFP32) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = Prec<DT>::w2f((uint16_t)(w[i] & 0xffffu));
            f[2 * i + 1] = Prec<DT>::w2f((uint16_t)(w[i] >> 16));
        }
    }
}
// The same with the stochastic rounding; word e serves element e (16-bit types only).
template <int DT> __device__ __forceinline__ uint4 pack16_sr(const float *f, const uint32_t *word)
{
    static_assert(DT != kFP32, "stochastic rounding is for the 16-bit storage types");
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t lo = DT == kBF16 ? sr_to_bf16(f[2 * i], word[2 * i]) : sr_to_f16(f[2 * i], word[2 * i]);
        const uint32_t hi = DT == kBF16 ? sr_to_bf16(f[2 * i + 1], word[2 * i + 1]) : sr_to_f16(f[2 * i + 1], word[2 * i + 1]);
        w[i] = lo | (hi << 16);
    }
    return uint4{w[0], w[1], w[2], w[3]};
}
template <int DT> __device__ __forceinline__ uint4 pack16(const float *f)
{
    if constexpr (DT == kFP32) {
        return uint4{__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3])};
    } else {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (DT == kBF16) {
                // both halves of a word in one conversion instruction (round to nearest even, as f2w does one by one)
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                const bf16x2 pk = __builtin_convertvector(f32x2{f[2 * i], f[2 * i + 1]}, bf16x2);
                w[i] = __builtin_bit_cast(uint32_t, pk);
            } else {
                w[i] = (uint32_t)Prec<DT>::f2w(f[2 * i]) | ((uint32_t)Prec<DT>::f2w(f[2 * i + 1]) << 16);
            }
        }
        return uint4{w[0], w[1], w[2], w[3]};
    }
}

// Descriptor i of a table in device memory, fetched through the scalar cache: the index is the same for every lane
// of the workgroup (it depends on blockIdx and the loop count alone), which the compiler cannot see by itself; a
// vector load here would put a memory round trip per lane in front of every chunk's address.
typedef const __attribute__((address_space(4))) TensorDesc *DescTable;
__device__ __forceinline__ DescTable desc_table(const TensorDesc *p) { return (DescTable)(uintptr_t)p; }
__device__ __forceinline__ TensorDesc desc_at(DescTable t, int i)
{
    const int u = __builtin_amdgcn_readfirstlane(i);
    TensorDesc d;
    d.src = t[u].src; d.dst = t[u].dst; d.numel = t[u].numel; d.first_chunk = t[u].first_chunk; d.tid = t[u].tid; d.pad = 0;
    return d;
}
__device__ __forceinline__ uint64_t desc_first_chunk(DescTable t, int i) { return t[__builtin_amdgcn_readfirstlane(i)].first_chunk; }

// One chunk = kAxpyChunk consecutive elements of one tensor; workgroup w of a launch takes chunks w, w + gridDim.x, ...
// of the launch's `total_chunks`.  SR: stochastic instead of nearest rounding into the storage type, with the random
// word of element i taken from word i % 4 of the Philox block (i / 4, tensor, tag 3) under the same seed.
#ifndef ZO_STREAM_THREADS
#define ZO_STREAM_THREADS 512
#endif
#ifndef ZO_AXPY_PER_CU
#define ZO_AXPY_PER_CU 4
#endif
constexpr int kStreamThreads = ZO_STREAM_THREADS;      // 4 workgroups of 8 waves fill a CU's 32 wave slots; 30 KiB of LDS each
template <int DT, bool SR>
__global__ __launch_bounds__(kStreamThreads) void axpy_z_kernel(const TensorDesc *__restrict__ descs, int n_desc, TensorDesc single,
                                                                uint64_t chunk_offset, uint32_t total_chunks, uint64_t seed, float scale,
                                                                const float *__restrict__ dev_scale)
{
    using W = typename Prec<DT>::W;
    constexpr int VN = Vec16<DT>::N;
    constexpr int kIter = kAxpyChunk / (kStreamThreads * VN);
    static_assert(kIter >= 1 && kIter * kStreamThreads * VN == (int)kAxpyChunk, "a chunk is a whole number of 16-byte pieces per thread");
    __shared__ float4 ln_tab[kRayleighLast];
    load_rayleigh_cells(ln_tab);
    const float sc = dev_scale ? *dev_scale : scale;
    int di = 0;
    if (descs) {
        // last descriptor whose first_chunk <= this workgroup's first chunk; later chunks only ever move forward from it
        const uint64_t chunk = (uint64_t)blockIdx.x + chunk_offset;
        int lo = 0, hi = n_desc - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (desc_first_chunk(desc_table(descs), mid) <= chunk) lo = mid; else hi = mid - 1;
        }
        di = lo;
    }
    auto desc_of = [&](uint64_t chunk) {
        if (!descs) return single;
        while (di + 1 < n_desc && desc_first_chunk(desc_table(descs), di + 1) <= chunk) ++di;
        return desc_at(desc_table(descs), di);
    };
    // A chunk that lies wholly inside its tensor (all but a tensor's last) is loaded one iteration ahead, into
    // registers, so that a wave never waits for memory with nothing to compute; the others take the guarded path.
    auto whole_chunk = [&](const TensorDesc &d, uint64_t chunk) { return ((chunk - d.first_chunk) + 1) * kAxpyChunk <= d.numel; };
    auto load_chunk = [&](const TensorDesc &d, uint64_t chunk, uint4 (&v)[kIter]) {
        const W *__restrict__ src = (const W *)d.src + (chunk - d.first_chunk) * kAxpyChunk;
#pragma unroll
        for (int it = 0; it < kIter; ++it) v[it] = *(const uint4 *)(src + (size_t)(it * kStreamThreads + threadIdx.x) * VN);
    };
    uint32_t c = blockIdx.x;
    if (c >= total_chunks) return;
    TensorDesc d = desc_of((uint64_t)c + chunk_offset);
    bool whole = whole_chunk(d, (uint64_t)c + chunk_offset);
    uint4 cur[kIter], nxt[kIter];
    if (whole) load_chunk(d, (uint64_t)c + chunk_offset, cur);
    for (;;) {
        const uint64_t chunk = (uint64_t)c + chunk_offset;
        const uint32_t cn = c + gridDim.x;
        const bool has_next = cn < total_chunks;
        TensorDesc dn = d;
        bool whole_n = false;
        if (has_next) {
            dn = desc_of((uint64_t)cn + chunk_offset);
            whole_n = whole_chunk(dn, (uint64_t)cn + chunk_offset);
            if (whole_n) load_chunk(dn, (uint64_t)cn + chunk_offset, nxt);
        }
        const uint64_t base = (chunk - d.first_chunk) * kAxpyChunk;
        const W *__restrict__ src = (const W *)d.src;
        W *__restrict__ dst = (W *)d.dst;
        if (whole) {
#pragma unroll
            for (int it = 0; it < kIter; ++it) {
                const uint64_t i0 = base + (uint64_t)(it * kStreamThreads + threadIdx.x) * VN;
                float z[VN];
#pragma unroll
                for (int b = 0; b < VN / 4; ++b) normal4(philox_block(seed, d.tid, i0 / 4 + b), z + 4 * b, ln_tab);
                float th[VN];
                unpack16<DT>(cur[it], th);
#pragma unroll
                for (int e = 0; e < VN; ++e) th[e] = __builtin_fmaf(sc, z[e], th[e]);
                if constexpr (SR) {
                    uint32_t rw[VN];
#pragma unroll
                    for (int b = 0; b < VN / 4; ++b) {
                        const u32x4 r = philox_block(seed, d.tid, i0 / 4 + b, 3u);
                        rw[4 * b] = r.x; rw[4 * b + 1] = r.y; rw[4 * b + 2] = r.z; rw[4 * b + 3] = r.w;
                    }
                    *(uint4 *)(dst + i0) = pack16_sr<DT>(th, rw);
                } else {
                    *(uint4 *)(dst + i0) = pack16<DT>(th);
                }
            }
        } else {
#pragma unroll 1
            for (int it = 0; it < kIter; ++it) {
                const uint64_t i0 = base + (uint64_t)(it * kStreamThreads + threadIdx.x) * VN;
                if (i0 >= d.numel) break;
                float z[VN];
#pragma unroll
                for (int b = 0; b < VN / 4; ++b) normal4(philox_block(seed, d.tid, i0 / 4 + b), z + 4 * b, ln_tab);
                uint32_t rw[SR ? VN : 1];
                if constexpr (SR) {
#pragma unroll
                    for (int b = 0; b < VN / 4; ++b) {
                        const u32x4 r = philox_block(seed, d.tid, i0 / 4 + b, 3u);
                        rw[4 * b] = r.x; rw[4 * b + 1] = r.y; rw[4 * b + 2] = r.z; rw[4 * b + 3] = r.w;
                    }
                }
                if (i0 + VN <= d.numel) {
                    float th[VN];
                    unpack16<DT>(*(const uint4 *)(src + i0), th);
#pragma unroll
                    for (int e = 0; e < VN; ++e) th[e] = __builtin_fmaf(sc, z[e], th[e]);
                    if constexpr (SR) *(uint4 *)(dst + i0) = pack16_sr<DT>(th, rw);
                    else *(uint4 *)(dst + i0) = pack16<DT>(th);
                } else {
                    for (int e = 0; e < VN && i0 + e < d.numel; ++e) {
                        const float v = __builtin_fmaf(sc, z[e], Prec<DT>::w2f(src[i0 + e]));
                        if constexpr (SR) dst[i0 + e] = DT == kBF16 ? sr_to_bf16(v, rw[e]) : sr_to_f16(v, rw[e]);
                        else dst[i0 + e] = Prec<DT>::f2w(v);
                    }
                }
            }
        }
        if (!has_next) break;
        c = cn; d = dn; whole = whole_n;
#pragma unroll
        for (int it = 0; it < kIter; ++it) cur[it] = nxt[it];
    }
}

// Several updates of Eq. 2 in one pass (a streamed block that is several steps behind takes them all right
// after its upload): theta <- rn(fma(s_j, z_j, theta)) for j = 0 .. n-1 in this order, each rounded into the
// storage type before the next starts from it, exactly as n separate passes would leave it, with one read and
// one write of theta.  Same chunking and addressing as axpy_z_kernel; the scalars are dev_scale[0 .. n-1].
template <int DT, bool SR>
__global__ __launch_bounds__(kStreamThreads) void axpy_z_multi_kernel(const TensorDesc *__restrict__ descs, int n_desc,
                                                                      uint64_t chunk_offset, uint32_t total_chunks, UpdateSeeds upd,
                                                                      const float *__restrict__ dev_scale)
{
    using W = typename Prec<DT>::W;
    constexpr int VN = Vec16<DT>::N;
    __shared__ float4 ln_tab[kRayleighLast];
    load_rayleigh_cells(ln_tab);
    int di;
    {
        const uint64_t chunk = (uint64_t)blockIdx.x + chunk_offset;
        int lo = 0, hi = n_desc - 1;                      // last descriptor whose first_chunk <= chunk
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (desc_first_chunk(desc_table(descs), mid) <= chunk) lo = mid; else hi = mid - 1;
        }
        di = lo;
    }
    for (uint32_t c = blockIdx.x; c < total_chunks; c += gridDim.x) {
        const uint64_t chunk = (uint64_t)c + chunk_offset;
        while (di + 1 < n_desc && desc_first_chunk(desc_table(descs), di + 1) <= chunk) ++di;
        const TensorDesc d = desc_at(desc_table(descs), di);
        const uint64_t base = (chunk - d.first_chunk) * kAxpyChunk;
        const W *__restrict__ src = (const W *)d.src;
        W *__restrict__ dst = (W *)d.dst;
        constexpr int kIter = kAxpyChunk / (kStreamThreads * VN);
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            const uint64_t i0 = base + (uint64_t)(it * kStreamThreads + threadIdx.x) * VN;
            if (i0 >= d.numel) break;
            const bool whole = i0 + VN <= d.numel;
            float th[VN];
            if (whole) {
                unpack16<DT>(*(const uint4 *)(src + i0), th);
            } else {
                for (int e = 0; e < VN; ++e) th[e] = i0 + e < d.numel ? Prec<DT>::w2f(src[i0 + e]) : 0.0f;
            }
            uint4 packed = uint4{0u, 0u, 0u, 0u};
            for (int j = 0; j < upd.n; ++j) {
                const uint64_t seed = upd.seed[j];
                const float sc = dev_scale[j];
                float z[VN];
#pragma unroll
                for (int b = 0; b < VN / 4; ++b) normal4(philox_block(seed, d.tid, i0 / 4 + b), z + 4 * b, ln_tab);
#pragma unroll
                for (int e = 0; e < VN; ++e) th[e] = __builtin_fmaf(sc, z[e], th[e]);
                if constexpr (SR) {
                    uint32_t rw[VN];
#pragma unroll
                    for (int b = 0; b < VN / 4; ++b) {
                        const u32x4 r = philox_block(seed, d.tid, i0 / 4 + b, 3u);
                        rw[4 * b] = r.x; rw[4 * b + 1] = r.y; rw[4 * b + 2] = r.z; rw[4 * b + 3] = r.w;
                    }
                    packed = pack16_sr<DT>(th, rw);
                } else {
                    packed = pack16<DT>(th);
                }
                unpack16<DT>(packed, th);                 // the next update starts from the stored value
            }
            if (whole) {
                *(uint4 *)(dst + i0) = packed;
            } else {
                for (int e = 0; e < VN && i0 + e < d.numel; ++e) dst[i0 + e] = Prec<DT>::f2w(th[e]);   // exact: th holds stored values
            }
        }
    }
}

// ------------------------------------------------------------------ staging W+ / W-
// Transposing form (a caller that keeps a matrix [in, out] and wants the GEMMs' [out, in]): tiles move a 64 x 64
// patch of a [rows, cols] matrix through LDS so that both the read (along cols) and the write (along rows of the
// transposed result) are coalesced.  Tensors that keep their layout go through stage_flat_kernel below.
// UPD != 0: the pass first applies a pending update of Eq. 2 to theta itself, theta <- rn(fma(s, z', theta)) with z'
// drawn from `upd_seed` and s read from dev_scale (UPD 1: round to nearest, 2: stochastic rounding), writes theta
// back, and stages W+- from the updated value: Alg. 2's deferred update, in the pass that reads theta anyway.  The
// arithmetic per element is that of axpy_z_kernel followed by the plain staging.
#ifndef ZO_STAGE_THREADS
#define ZO_STAGE_THREADS 1024
#endif
#ifndef ZO_STAGE_PER_CU
#define ZO_STAGE_PER_CU 2
#endif
constexpr int kStageThreads = ZO_STAGE_THREADS;       // groups of 256 threads, one tile each
// A workgroup is kStageThreads / 256 groups of 256 threads that share the radius table; in every round of the
// persistent loop each group takes one tile (group g of workgroup w: tiles (w + i gridDim.x) G + g).  A transposing
// tile goes through the group's LDS buffer one sign at a time (W+ out, then W-), which halves the buffer and lets
// two 1024-thread workgroups, all 32 wave slots, share a CU next to the 24 KiB table.  The barriers of a round are
// the same for every group whether it has a tile or not.
template <int DT, bool SINGLE, int UPD>
__global__ __launch_bounds__(kStageThreads) __attribute__((amdgpu_waves_per_eu((DT != kFP32 && UPD != 2) ? 8 : 4))) void stage_kernel(StageBatch batch, uint64_t seed, float eps, uint64_t upd_seed,
                                                              const float *__restrict__ dev_scale)
{
    using W = typename Prec<DT>::W;
    constexpr int VN = Vec16<DT>::N;
    static_assert(!(SINGLE && UPD != 0) && !(DT == kFP32 && UPD == 2), "no such variant");
    constexpr int G = kStageThreads / 256;
    constexpr int T = (int)kStageTile;
    constexpr int LD = T + 4;                       // row stride: keeps 8-byte (16-byte for fp32) alignment, spreads banks
    constexpr int kTileF4 = G * T * LD * (int)sizeof(W) / 16;
    static_assert(kTileF4 >= kRayleighFirst, "the table's virtual base must not fall below the LDS allocation");
    // LDS: the groups' tile buffers first, the radius table behind them (its unused leading entries overlap the tile
    // area only virtually: load_rayleigh_cells and normal_pair touch entries >= kRayleighFirst alone)
    __shared__ float4 lds[kTileF4 + (SINGLE ? 0 : kRayleighLast - kRayleighFirst)];
    [[maybe_unused]] const float4 *const ln_tab = lds + kTileF4 - kRayleighFirst;
    if constexpr (!SINGLE) load_rayleigh_cells(lds + kTileF4 - kRayleighFirst);
    const int grp = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8));
    const uint32_t tix = threadIdx.x & 255u;
    W *const sbuf = (W *)lds + grp * T * LD;
    float us = 0.0f;
    if constexpr (UPD != 0) us = *dev_scale;
    for (uint32_t blk0 = blockIdx.x * G; blk0 < batch.total_tiles; blk0 += gridDim.x * G) {
        const uint32_t blk = blk0 + (uint32_t)grp;
        const bool active = blk < batch.total_tiles;
        int di = 0;
        for (int i = 1; i < batch.n; ++i)
            if (batch.d[i].first_tile <= blk) di = i;
        const StageDesc &d = batch.d[di];
        const uint32_t tile = blk - d.first_tile;
        W *const theta = (W *)const_cast<void *>(d.src);      // written only when UPD != 0
        const W *src = theta;
        W *__restrict__ dp = (W *)d.dst_plus;
        W *__restrict__ dm = (W *)d.dst_minus;
        const bool transposing = active;          // the launcher sends flat tensors to stage_flat_kernel

        // transposing tile: rows r0.., cols c0..  (cols % 4 == 0 is guaranteed by the caller)
        // A thread owns a 4 x 4 patch (4 adjacent rows, one Philox block each), so each of its 4 columns goes
        // into the transposed LDS tile as one packed store of 4 adjacent rows (no 2-byte scatter).
        const uint32_t tiles_c = transposing ? d.tiles_c : 1u;
        const uint32_t r0 = (tile / tiles_c) * T, c0 = (tile % tiles_c) * T;
        const uint32_t rb = tix / 16, cb = tix % 16;
        const uint32_t c = c0 + 4 * cb;
        // packed columns of the patch, per sign: col[e] = rows 0..3 of column e (2-byte types: two words; fp32: four)
        constexpr int CW = (int)sizeof(W) == 2 ? 2 : 4;
        uint32_t colp[4][CW], colm[SINGLE ? 1 : 4][CW];
        if (transposing) {
            // Rows or columns past the edge of the matrix are computed like the others, from element 0 (always there),
            // and never leave LDS: one straight-line body for the four rows lets the compiler share the generator's
            // constants between them instead of setting them up again behind every bounds branch.
            float fpv[4][4];
            [[maybe_unused]] float fmv[4][4];
            W rawv[4][4];
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const uint32_t r = r0 + 4 * rb + it;
                const bool valid = r < d.rows && c < d.cols;
                const uint64_t i0 = valid ? (uint64_t)r * d.cols + c : 0;
                W raw[4];
                if constexpr (sizeof(W) == 2) *(uint2 *)raw = *(const uint2 *)(src + i0);
                else *(uint4 *)raw = *(const uint4 *)(src + i0);
                if constexpr (SINGLE) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) rawv[it][e] = raw[e];
                } else {
                    float z[4];
                    normal4(philox_block(seed, d.tid, i0 / 4), z, ln_tab);
                    if constexpr (UPD != 0) {
                        float zu[4];
                        normal4(philox_block(upd_seed, d.tid, i0 / 4), zu, ln_tab);
                        u32x4 rr{};
                        if constexpr (UPD == 2) rr = philox_block(upd_seed, d.tid, i0 / 4, 3u);
                        const uint32_t rw[4] = {rr.x, rr.y, rr.z, rr.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float v = __builtin_fmaf(us, zu[e], Prec<DT>::w2f(raw[e]));
                            if constexpr (UPD == 2) raw[e] = DT == kBF16 ? sr_to_bf16(v, rw[e]) : sr_to_f16(v, rw[e]);
                            else raw[e] = Prec<DT>::f2w(v);
                        }
                        if (valid) {
                            if constexpr (sizeof(W) == 2) *(uint2 *)(theta + i0) = *(const uint2 *)raw;
                            else *(uint4 *)(theta + i0) = *(const uint4 *)raw;
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float th = Prec<DT>::w2f(raw[e]);
                        fpv[it][e] = __builtin_fmaf(eps, z[e], th);
                        fmv[it][e] = __builtin_fmaf(-eps, z[e], th);
                    }
                }
            }
            // round into the storage type, four rows of a column side by side
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (SINGLE) {
                    if constexpr (sizeof(W) == 2) {
                        colp[e][0] = (uint32_t)rawv[0][e] | ((uint32_t)rawv[1][e] << 16);
                        colp[e][1] = (uint32_t)rawv[2][e] | ((uint32_t)rawv[3][e] << 16);
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) colp[e][r] = __float_as_uint(rawv[r][e]);
                    }
                } else if constexpr (DT == kBF16) {
                    // one conversion instruction rounds two rows of the column (nearest even, as the scalar conversion does)
                    typedef float f32x2 __attribute__((ext_vector_type(2)));
                    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                    auto pk = [](float lo, float hi) { return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2)); };
                    colp[e][0] = pk(fpv[0][e], fpv[1][e]); colp[e][1] = pk(fpv[2][e], fpv[3][e]);
                    colm[e][0] = pk(fmv[0][e], fmv[1][e]); colm[e][1] = pk(fmv[2][e], fmv[3][e]);
                } else if constexpr (DT == kFP16) {
                    colp[e][0] = (uint32_t)Prec<DT>::f2w(fpv[0][e]) | ((uint32_t)Prec<DT>::f2w(fpv[1][e]) << 16);
                    colp[e][1] = (uint32_t)Prec<DT>::f2w(fpv[2][e]) | ((uint32_t)Prec<DT>::f2w(fpv[3][e]) << 16);
                    colm[e][0] = (uint32_t)Prec<DT>::f2w(fmv[0][e]) | ((uint32_t)Prec<DT>::f2w(fmv[1][e]) << 16);
                    colm[e][1] = (uint32_t)Prec<DT>::f2w(fmv[2][e]) | ((uint32_t)Prec<DT>::f2w(fmv[3][e]) << 16);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) { colp[e][r] = __float_as_uint(fpv[r][e]); colm[e][r] = __float_as_uint(fmv[r][e]); }
                }
            }
        }
        // one sign at a time through the group's tile: columns in, barrier, rows of the transposed result out
        auto tile_in = [&](const uint32_t (&col)[4][CW]) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                W *dst = sbuf + (4 * cb + e) * LD + 4 * rb;
                if constexpr (sizeof(W) == 2) *(uint2 *)dst = uint2{col[e][0], col[e][1]};
                else *(uint4 *)dst = uint4{col[e][0], col[e][1], col[e][2], col[e][3]};
            }
        };
        auto tile_out = [&](W *__restrict__ out) {
            // output row = source column c0 + tix/4, 16 consecutive source rows starting at r0 + 16*(tix%4)
            const uint32_t oc = tix / 4, seg = 16 * (tix % 4);
            if (c0 + oc >= d.cols) return;
            const uint64_t o0 = (uint64_t)(c0 + oc) * d.rows + r0 + seg;
            const bool full = (r0 + seg + 16 <= d.rows) && ((d.rows * sizeof(W)) % 16 == 0);
            if (full) {
                constexpr int NV = 16 * (int)sizeof(W) / 16;      // 16-byte pieces per 16 elements
                using LdsVec = typename std::conditional<sizeof(W) == 2, uint2, uint4>::type;
                constexpr int PER = 16 / (int)sizeof(LdsVec);     // LDS reads per 16-byte piece
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    LdsVec pp[PER];
#pragma unroll
                    for (int j = 0; j < PER; ++j) pp[j] = ((const LdsVec *)(sbuf + oc * LD + seg))[v * PER + j];
                    ((uint4 *)(out + o0))[v] = *(const uint4 *)pp;
                }
            } else {
                for (uint32_t e = 0; e < 16 && r0 + seg + e < d.rows; ++e) out[o0 + e] = sbuf[oc * LD + seg + e];
            }
        };
        if (transposing) tile_in(colp);
        __syncthreads();
        if (transposing) tile_out(dp);
        if constexpr (!SINGLE) {
            __syncthreads();
            if (transposing) tile_in(colm);
            __syncthreads();
            if (transposing) tile_out(dm);
        }
        __syncthreads();        // the tile is read out before the next round writes it
    }
}

// ------------------------------------------------------------------ staging W+ / W-, nothing to transpose
// The batch of a decoder block: every tensor keeps its layout (a linear weight is stored [out, in], the layout
// the GEMMs read), so the pass is a plain stream, theta in, W+ and W- out, built like axpy_z_kernel: four
// 512-thread workgroups per CU that fill the radius table once, chunks of kStageFlatTile consecutive elements of
// one tensor, the next chunk's theta fetched into registers while this one is computed.  Chunk numbering and
// arithmetic are those of stage_kernel's flat tiles.
template <int DT, bool SINGLE, int UPD>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu((DT != kFP32 && UPD == 0) ? 8 : 4)))
void stage_flat_kernel(StageBatch batch, uint64_t seed, float eps, uint64_t upd_seed,
                                                                    const float *__restrict__ dev_scale)
{
    using W = typename Prec<DT>::W;
    constexpr int VN = Vec16<DT>::N;
    constexpr int kIter = kStageFlatTile / (kStreamThreads * VN);
    static_assert(kIter >= 1 && kIter * kStreamThreads * VN == (int)kStageFlatTile, "a chunk is a whole number of 16-byte pieces per thread");
    static_assert(!(SINGLE && UPD != 0) && !(DT == kFP32 && UPD == 2), "no such variant");
    __shared__ float4 ln_tab[SINGLE ? 1 : kRayleighLast];
    if constexpr (!SINGLE) load_rayleigh_cells(ln_tab);
    float us = 0.0f;
    if constexpr (UPD != 0) us = *dev_scale;
    struct Piece {
        W *theta, *dp, *dm;      // theta is written only when UPD != 0
        uint64_t numel, base;    // base: first element of the chunk in its tensor
        uint32_t tid;
        bool whole;              // the chunk lies wholly inside the tensor
    };
    int di = 0;
    auto piece_of = [&](uint32_t tile) {
        while (di + 1 < batch.n && batch.d[di + 1].first_tile <= tile) ++di;
        const StageDesc &d = batch.d[di];
        Piece p;
        p.theta = (W *)const_cast<void *>(d.src); p.dp = (W *)d.dst_plus; p.dm = (W *)d.dst_minus;
        p.numel = (uint64_t)d.rows * d.cols;
        p.base = (uint64_t)(tile - d.first_tile) * kStageFlatTile;
        p.tid = d.tid;
        p.whole = p.base + kStageFlatTile <= p.numel;
        return p;
    };
    auto load_chunk = [&](const Piece &p, uint4 (&v)[kIter]) {
#pragma unroll
        for (int it = 0; it < kIter; ++it) v[it] = *(const uint4 *)(p.theta + p.base + (size_t)(it * kStreamThreads + threadIdx.x) * VN);
    };
    // 16 bytes of theta at element i0 (`raw` when `full`, else the tensor's ragged tail, read element-wise)
    auto piece16 = [&](const Piece &p, uint64_t i0, const uint4 &raw, bool full) {
        if constexpr (SINGLE) {
            if (full) *(uint4 *)(p.dp + i0) = raw;
            else for (int e = 0; e < VN && i0 + e < p.numel; ++e) p.dp[i0 + e] = p.theta[i0 + e];
        } else {
            float z[VN];
#pragma unroll
            for (int b = 0; b < VN / 4; ++b) normal4(philox_block(seed, p.tid, i0 / 4 + b), z + 4 * b, ln_tab);
            float th[VN], a[VN], b[VN];
            if (full) {
                unpack16<DT>(raw, th);
            } else {
                for (int e = 0; e < VN; ++e) th[e] = i0 + e < p.numel ? Prec<DT>::w2f(p.theta[i0 + e]) : 0.0f;
            }
            if constexpr (UPD != 0) {
                float zu[VN];
#pragma unroll
                for (int bk = 0; bk < VN / 4; ++bk) normal4(philox_block(upd_seed, p.tid, i0 / 4 + bk), zu + 4 * bk, ln_tab);
#pragma unroll
                for (int e = 0; e < VN; ++e) th[e] = __builtin_fmaf(us, zu[e], th[e]);
                uint4 stored;
                if constexpr (UPD == 2) {
                    uint32_t rw[VN];
#pragma unroll
                    for (int bk = 0; bk < VN / 4; ++bk) {
                        const u32x4 r = philox_block(upd_seed, p.tid, i0 / 4 + bk, 3u);
                        rw[4 * bk] = r.x; rw[4 * bk + 1] = r.y; rw[4 * bk + 2] = r.z; rw[4 * bk + 3] = r.w;
                    }
                    stored = pack16_sr<DT>(th, rw);
                } else {
                    stored = pack16<DT>(th);
                }
                unpack16<DT>(stored, th);          // staging starts from the stored value
                if (full) *(uint4 *)(p.theta + i0) = stored;
                else for (int e = 0; e < VN && i0 + e < p.numel; ++e) p.theta[i0 + e] = Prec<DT>::f2w(th[e]);   // exact
            }
#pragma unroll
            for (int e = 0; e < VN; ++e) {
                a[e] = __builtin_fmaf(eps, z[e], th[e]);
                b[e] = __builtin_fmaf(-eps, z[e], th[e]);
            }
            if (full) {
                *(uint4 *)(p.dp + i0) = pack16<DT>(a);
                *(uint4 *)(p.dm + i0) = pack16<DT>(b);
            } else {
                for (int e = 0; e < VN && i0 + e < p.numel; ++e) {
                    p.dp[i0 + e] = Prec<DT>::f2w(a[e]);
                    p.dm[i0 + e] = Prec<DT>::f2w(b[e]);
                }
            }
        }
    };
    uint32_t c = blockIdx.x;
    if (c >= batch.total_tiles) return;
    Piece p = piece_of(c);
    uint4 cur[kIter], nxt[kIter];
    if (p.whole) load_chunk(p, cur);
    for (;;) {
        const uint32_t cn = c + gridDim.x;
        const bool has_next = cn < batch.total_tiles;
        Piece pn = p;
        if (has_next) {
            pn = piece_of(cn);
            if (pn.whole) load_chunk(pn, nxt);
        }
        if (p.whole) {
#pragma unroll
            for (int it = 0; it < kIter; ++it) piece16(p, p.base + (uint64_t)(it * kStreamThreads + threadIdx.x) * VN, cur[it], true);
        } else {
#pragma unroll 1
            for (int it = 0; it < kIter; ++it) {
                const uint64_t i0 = p.base + (uint64_t)(it * kStreamThreads + threadIdx.x) * VN;
                if (i0 >= p.numel) break;
                const bool full = i0 + VN <= p.numel;
                uint4 raw = uint4{0u, 0u, 0u, 0u};
                if (full) raw = *(const uint4 *)(p.theta + i0);
                piece16(p, i0, raw, full);
            }
        }
        if (!has_next) break;
        c = cn; p = pn;
#pragma unroll
        for (int it = 0; it < kIter; ++it) cur[it] = nxt[it];
    }
}

// ------------------------------------------------------------------ launchers
hipError_t launch_z(float *out, uint64_t n, uint64_t seed, uint32_t tid, uint64_t first, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (first + n - 1) / 4 - first / 4 + 1;
    z_kernel<<<dim3((unsigned)((blocks + 255) / 256)), dim3(256), 0, s>>>(out, n, seed, tid, first);
    return hipGetLastError();
}

hipError_t launch_normal_pairs(const uint32_t *words, float *z, uint64_t n_pairs, hipStream_t s)
{
    if (n_pairs == 0) return hipSuccess;
    normal_pairs_kernel<<<dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, s>>>(words, z, n_pairs);
    return hipGetLastError();
}

// Persistent launches: `per_cu` workgroups per CU (what the kernel's LDS and wave slots allow), never more than
// there are chunks.
static hipError_t persistent_grid(uint64_t work, int per_cu, unsigned *grid)
{
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        n_cu = v > 0 ? v : 1;
    }
    const uint64_t cap = (uint64_t)n_cu * per_cu;
    *grid = (unsigned)(work < cap ? work : cap);
    return hipSuccess;
}

template <int DT>
static hipError_t axpy_launch_t(const TensorDesc *descs, int n_desc, const TensorDesc &single, uint64_t chunk_offset,
                                uint64_t chunks, uint64_t seed, float scale, const float *dev_scale, bool stochastic,
                                hipStream_t s)
{
    if (chunks == 0) return hipSuccess;
    if (chunks > 0x7fffffffull) return hipErrorInvalidValue;
    unsigned g = 0;
    if (hipError_t e = persistent_grid(chunks, ZO_AXPY_PER_CU, &g); e != hipSuccess) return e;
    const dim3 grid(g), block(kStreamThreads);
    if constexpr (DT != kFP32) {
        if (stochastic) {
            axpy_z_kernel<DT, true><<<grid, block, 0, s>>>(descs, n_desc, single, chunk_offset, (uint32_t)chunks, seed, scale, dev_scale);
            return hipGetLastError();
        }
    }
    if (stochastic) return hipErrorInvalidValue;          // fp32 storage has nothing to round stochastically
    axpy_z_kernel<DT, false><<<grid, block, 0, s>>>(descs, n_desc, single, chunk_offset, (uint32_t)chunks, seed, scale, dev_scale);
    return hipGetLastError();
}

hipError_t launch_axpy_multi(const TensorDesc *dev_descs, int n_desc, uint64_t chunk_offset, uint64_t total_chunks,
                             int dtype, uint64_t seed, float scale, const float *dev_scale, bool stochastic, hipStream_t s)
{
    TensorDesc none{};
    switch (dtype) {
    case kFP32: return axpy_launch_t<kFP32>(dev_descs, n_desc, none, chunk_offset, total_chunks, seed, scale, dev_scale, stochastic, s);
    case kBF16: return axpy_launch_t<kBF16>(dev_descs, n_desc, none, chunk_offset, total_chunks, seed, scale, dev_scale, stochastic, s);
    case kFP16: return axpy_launch_t<kFP16>(dev_descs, n_desc, none, chunk_offset, total_chunks, seed, scale, dev_scale, stochastic, s);
    }
    return hipErrorInvalidValue;
}

template <int DT>
static hipError_t axpy_multi_launch_t(const TensorDesc *descs, int n_desc, uint64_t chunk_offset, uint64_t chunks,
                                      const UpdateSeeds &upd, const float *dev_scales, bool stochastic, hipStream_t s)
{
    if (chunks == 0 || upd.n == 0) return hipSuccess;
    if (chunks > 0x7fffffffull || upd.n < 0 || upd.n > kMaxUpdates || !descs || !dev_scales) return hipErrorInvalidValue;
    unsigned g = 0;
    if (hipError_t e = persistent_grid(chunks, 4, &g); e != hipSuccess) return e;
    const dim3 grid(g), block(kStreamThreads);
    if constexpr (DT != kFP32) {
        if (stochastic) {
            axpy_z_multi_kernel<DT, true><<<grid, block, 0, s>>>(descs, n_desc, chunk_offset, (uint32_t)chunks, upd, dev_scales);
            return hipGetLastError();
        }
    }
    if (stochastic) return hipErrorInvalidValue;
    axpy_z_multi_kernel<DT, false><<<grid, block, 0, s>>>(descs, n_desc, chunk_offset, (uint32_t)chunks, upd, dev_scales);
    return hipGetLastError();
}

hipError_t launch_axpy_updates(const TensorDesc *dev_descs, int n_desc, uint64_t chunk_offset, uint64_t total_chunks, int dtype,
                               const UpdateSeeds &upd, const float *dev_scales, bool stochastic, hipStream_t s)
{
    switch (dtype) {
    case kFP32: return axpy_multi_launch_t<kFP32>(dev_descs, n_desc, chunk_offset, total_chunks, upd, dev_scales, stochastic, s);
    case kBF16: return axpy_multi_launch_t<kBF16>(dev_descs, n_desc, chunk_offset, total_chunks, upd, dev_scales, stochastic, s);
    case kFP16: return axpy_multi_launch_t<kFP16>(dev_descs, n_desc, chunk_offset, total_chunks, upd, dev_scales, stochastic, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_axpy_single(const TensorDesc &d, int dtype, uint64_t seed, float scale, const float *dev_scale,
                              bool stochastic, hipStream_t s)
{
    const uint64_t chunks = (d.numel + kAxpyChunk - 1) / kAxpyChunk;
    TensorDesc one = d;
    one.first_chunk = 0;
    switch (dtype) {
    case kFP32: return axpy_launch_t<kFP32>(nullptr, 0, one, 0, chunks, seed, scale, dev_scale, stochastic, s);
    case kBF16: return axpy_launch_t<kBF16>(nullptr, 0, one, 0, chunks, seed, scale, dev_scale, stochastic, s);
    case kFP16: return axpy_launch_t<kFP16>(nullptr, 0, one, 0, chunks, seed, scale, dev_scale, stochastic, s);
    }
    return hipErrorInvalidValue;
}

void stage_batch_add(StageBatch &b, const void *src, void *dp, void *dm, uint32_t rows, uint32_t cols, uint32_t tid,
                     bool transpose)
{
    StageDesc &d = b.d[b.n++];
    d.src = src; d.dst_plus = dp; d.dst_minus = dm; d.rows = rows; d.cols = cols; d.tid = tid;
    d.transpose = transpose ? 1u : 0u;
    d.first_tile = b.total_tiles;
    if (transpose) {
        d.tiles_c = (cols + kStageTile - 1) / kStageTile;
        b.total_tiles += d.tiles_c * ((rows + kStageTile - 1) / kStageTile);
    } else {
        d.tiles_c = 0;
        b.total_tiles += (uint32_t)(((uint64_t)rows * cols + kStageFlatTile - 1) / kStageFlatTile);
    }
}

hipError_t launch_stage(const StageBatch &b, int dtype, uint64_t seed, float eps, bool single_copy, hipStream_t s, int upd_mode,
                        uint64_t upd_seed, const float *dev_scale)
{
    if (b.total_tiles == 0) return hipSuccess;
    if (upd_mode < 0 || upd_mode > 2 || (upd_mode != 0 && (single_copy || !dev_scale)) || (upd_mode == 2 && dtype == kFP32))
        return hipErrorInvalidValue;
    // tensors that keep their layout and tensors to transpose take different kernels; no caller mixes them in a batch
    int n_tr = 0;
    for (int i = 0; i < b.n; ++i) n_tr += b.d[i].transpose != 0;
    if (n_tr != 0 && n_tr != b.n) return hipErrorInvalidValue;
    unsigned g = 0;
    if (n_tr == 0) {
        // registers allow four workgroups per CU for the plain 16-bit pass, three with the update folded in, two in fp32
        const int per_cu = dtype == kFP32 ? 2 : upd_mode != 0 ? 3 : ZO_AXPY_PER_CU;
        if (hipError_t e = persistent_grid(b.total_tiles, per_cu, &g); e != hipSuccess) return e;
        const dim3 grid(g), block(kStreamThreads);
#define ZO_STAGE(DT)                                                                                                   \
    if (single_copy) stage_flat_kernel<DT, true, 0><<<grid, block, 0, s>>>(b, seed, eps, 0, nullptr);                   \
    else if (upd_mode == 0) stage_flat_kernel<DT, false, 0><<<grid, block, 0, s>>>(b, seed, eps, 0, nullptr);           \
    else if (upd_mode == 1) stage_flat_kernel<DT, false, 1><<<grid, block, 0, s>>>(b, seed, eps, upd_seed, dev_scale);  \
    else if constexpr (DT != kFP32) stage_flat_kernel<DT, false, 2><<<grid, block, 0, s>>>(b, seed, eps, upd_seed, dev_scale); \
    return hipGetLastError();
        switch (dtype) {
        case kFP32: ZO_STAGE(kFP32)
        case kBF16: ZO_STAGE(kBF16)
        case kFP16: ZO_STAGE(kFP16)
        }
#undef ZO_STAGE
        return hipErrorInvalidValue;
    }
    // LDS per workgroup of four groups: 58 KiB (16-bit types), 92 KiB (fp32), 34 / 68 KiB for the plain copy
    constexpr int G = kStageThreads / 256;
    if (hipError_t e = persistent_grid((b.total_tiles + G - 1) / G, dtype == kFP32 ? 1 : ZO_STAGE_PER_CU, &g); e != hipSuccess) return e;
    const dim3 grid(g), block(kStageThreads);
#define ZO_STAGE(DT)                                                                                              \
    if (single_copy) stage_kernel<DT, true, 0><<<grid, block, 0, s>>>(b, seed, eps, 0, nullptr);                   \
    else if (upd_mode == 0) stage_kernel<DT, false, 0><<<grid, block, 0, s>>>(b, seed, eps, 0, nullptr);           \
    else if (upd_mode == 1) stage_kernel<DT, false, 1><<<grid, block, 0, s>>>(b, seed, eps, upd_seed, dev_scale);  \
    else if constexpr (DT != kFP32) stage_kernel<DT, false, 2><<<grid, block, 0, s>>>(b, seed, eps, upd_seed, dev_scale); \
    return hipGetLastError();
    switch (dtype) {
    case kFP32: ZO_STAGE(kFP32)
    case kBF16: ZO_STAGE(kBF16)
    case kFP16: ZO_STAGE(kFP16)
    }
#undef ZO_STAGE
    return hipErrorInvalidValue;
}

}  // namespace zo

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
// {0..3} for lane half h), which V^T is read with as well, so P never leaves registers.  V stays
// row-major in LDS; its transposed fragments come from the LDS transposing read of gfx950.
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

// Two probabilities into one register, round-to-nearest-even: one packed conversion instead of two
// single ones and a merge.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
template <int DT> __device__ __forceinline__ uint32_t pack2(float a, float b)
{
    const f32x2 v = {a, b};
    if constexpr (DT == kBF16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    else return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// The value that the lane 32 places away holds, taken with the register swap between the two halves of a
// wave (no trip through LDS as a shuffle would make): after the swap of two copies of x, one result holds
// x of lanes 0..31 in both halves and the other x of lanes 32..63, so one of the two is the lane's own value
// and the other its partner's; sum and maximum take both and do not care which is which.
__device__ __forceinline__ void swap_halves(float x, float &a, float &b)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers across the loop

template <int DT, int DH>
__global__ __launch_bounds__(256, (DH == 64 ? 3 : 2)) void attn_mfma_kernel(const uint16_t *__restrict__ qkv, uint16_t *__restrict__ out, int seq,
                                                        int n_heads, int n_seq)
{
    constexpr int CH = DH / 8;            // 16-byte chunks per K / V row
    // K and V tiles, both [key][channel] as they sit in memory, 16-byte chunks XOR-swizzled per key so that
    // the MFMA fragment reads of K (32 keys, one chunk) and the transposing reads of V (4 keys x 32 bytes
    // per 16 lanes) are free of conflicts on the 64-bank LDS.
    // Two buffers each: the tile after the current one arrives (global memory straight into LDS) while the
    // current one is multiplied.
    __shared__ u32x4 ks2[2][BKV * CH];
    __shared__ u32x4 vs2[2][BKV * CH];
    auto kswz = [](int r) { return DH == 128 ? (r & 15) : ((r >> 1) & 7); };
    auto vswz = [](int r) { return DH == 128 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); };

    // Workgroup -> (query tile, head, sequence).  The hardware deals consecutive workgroups round-robin to the 8
    // XCDs, so workgroup w runs on XCD w % 8 and is that XCD's (w / 8)-th.  Every (head, sequence) pair goes to one
    // XCD with all its query tiles, long rows first: the XCDs then hold equal shares of the causal triangle (dealing
    // the query tiles round-robin would give one XCD the two longest of every 16 and another the two shortest), and
    // the K and V of a pair are fetched into one L2 instead of eight.  The grid is padded to whole rounds of 8 pairs.
    const int n_qt = (seq + BQ - 1) / BQ;
    const int slot = (int)blockIdx.x >> 3;
    const int pair = (slot / n_qt) * 8 + ((int)blockIdx.x & 7);
    if (pair >= n_heads * n_seq) return;
    const int qt = n_qt - 1 - slot % n_qt;
    const int head = pair % n_heads, sq = pair / n_heads;
    const int d = n_heads * DH, ld = 3 * d;
    const uint16_t *base = qkv + (size_t)sq * seq * ld + head * DH;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, and known to be: it feeds scalar operands
    const int fr = lane & 31, fh = lane >> 5;
    const int q0 = qt * BQ + wave * 32;          // first query row of this wave
    const int qrow = q0 + fr;                    // this lane's query row
    const int qload = qrow < seq ? qrow : seq - 1;

    // Q fragments: B operand, lane = (row fr, k half fh), all DH/16 steps
    uint4 qf[DH / 16];
#pragma unroll
    for (int s = 0; s < DH / 16; ++s) qf[s] = *(const uint4 *)(base + (size_t)qload * ld + s * 16 + fh * 8);
    // The Q loads are made to land here, before the key loop.  Otherwise the compiler waits for them where the
    // loop first uses them, by counting outstanding memory operations, and inside the loop that count also
    // holds the next tile's global->LDS loads (issued from asm, unknown to the compiler): every tile would
    // wait for its successor's data.
#pragma unroll
    for (int s = 0; s < DH / 16; ++s) asm volatile("" ::"v"(qf[s].x), "v"(qf[s].y), "v"(qf[s].z), "v"(qf[s].w));

    f32x16 oacc[DH / 32];
#pragma unroll
    for (int c = 0; c < DH / 32; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[c][i] = 0.0f;
    // reference maximum of the raw scores (see the key loop), running normaliser; sc = log2(e)/sqrt(d_head)
    float m_run = -INFINITY, l_run = 0.0f;
    const float sc = 1.4426950408889634f / __builtin_sqrtf((float)DH);

    // global -> LDS for a K/V tile, without passing through registers: one wave instruction moves 64 x 16
    // bytes and lane L's piece lands at the instruction's LDS base + 16 L.  Piece p = 64 (NLD wave + i) + L of
    // a tile is slot p % CH of key row p / CH; the slot holds logical chunk slot ^ swizzle(row), so the
    // swizzle is applied on the global side (still whole 16-byte pieces of one row per lane).  The lane part
    // of the address does not change from tile to tile: the key advance goes into a scalar base.
    constexpr int NLD = BKV * CH / 256;   // instructions per wave and operand
    uint32_t kgo[NLD], vgo[NLD];          // byte offsets from the tile's first key row
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int pidx = 64 * (NLD * wave + i) + lane, r = pidx / CH, slot = pidx % CH;
        kgo[i] = (uint32_t)(r * ld + d + (slot ^ kswz(r)) * 8) * 2u;
        vgo[i] = (uint32_t)(r * ld + 2 * d + (slot ^ vswz(r)) * 8) * 2u;
    }
    const uint32_t ks_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)&ks2[0][0];
    const uint32_t vs_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)&vs2[0][0];
    auto dma16 = [](uint64_t gbase, uint32_t lane_off, uint32_t lds_off) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(gbase), "s"(lds_off) : "memory");
    };
    // (the halves go through unsigned 32-bit variables: readfirstlane returns a signed int, which would
    // sign-extend into the upper half)
    const uint32_t gb_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)base);
    const uint32_t gb_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)base >> 32));
    const uint64_t gbase0 = ((uint64_t)gb_hi << 32) | (uint64_t)gb_lo;
    auto issue_tile = [&](int k0, int buf) {
        const uint32_t kdst = ks_lds + (uint32_t)buf * (BKV * CH * 16) + (uint32_t)(NLD * wave) * 1024u;
        const uint32_t vdst = vs_lds + (uint32_t)buf * (BKV * CH * 16) + (uint32_t)(NLD * wave) * 1024u;
        if (k0 + BKV <= seq) {
            const uint64_t gb = gbase0 + (uint64_t)k0 * (uint64_t)ld * 2u;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                dma16(gb, kgo[i], kdst + i * 1024u);
                dma16(gb, vgo[i], vdst + i * 1024u);
            }
        } else {
            // last, ragged tile of the sequence: key rows past its end re-read the last row (masked as future keys)
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int pidx = 64 * (NLD * wave + i) + lane, r = pidx / CH, slot = pidx % CH;
                const int kr = k0 + r < seq ? k0 + r : seq - 1;
                dma16(gbase0, (uint32_t)(kr * ld + d + (slot ^ kswz(r)) * 8) * 2u, kdst + i * 1024u);
                dma16(gbase0, (uint32_t)(kr * ld + 2 * d + (slot ^ vswz(r)) * 8) * 2u, vdst + i * 1024u);
            }
        }
    };
    // Transposing LDS read (ds_read_b64_tr_b16): in every group of 16 lanes, lane j hands in the address of
    // four consecutive 16-bit elements ("row j") and lane i gets back element i%4 of rows i/4, i/4+4, i/4+8,
    // i/4+12.  With lane j pointing at key kb + j/4, channels cb + 4 (j%4) .. + 3, lane i receives channel
    // cb + i for the four keys kb .. kb+3: a V^T fragment straight from row-major V.
    const int tj = lane & 15;
    const int tr_key = tj >> 2;                                  // + key base
    const int tr_chan = 16 * ((lane >> 4) & 1) + 4 * (tj & 3);   // + 32 * channel tile
    // Everything of an LDS address that depends on the lane is worked out once, here: the key bases of the
    // loop are multiples of 4 (V) and 16 or 32 (K), which the swizzles do not see, so inside the loop an
    // address is one of these plus a compile-time constant.
    int voff[DH / 32];                                           // element offset of (key tr_key + 4 fh, channel tile c)
#pragma unroll
    for (int c = 0; c < DH / 32; ++c) {
        const int key = 4 * fh + tr_key, chan = c * 32 + tr_chan;
        voff[c] = (key * CH + ((chan >> 3) ^ vswz(key))) * 8 + (chan & 7);
    }
    auto vt_frag = [&](const u32x4 *vs, int kb16, int ctile) {   // keys kb16 + 4 fh + tr_key, kb16 a multiple of 8
        const uint16_t *p = (const uint16_t *)vs + voff[ctile] + kb16 * CH * 8;
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16 *)p);
    };
    int koff[DH / 16];                                           // u32x4 index of (key fr, k-step s)
#pragma unroll
    for (int s = 0; s < DH / 16; ++s) koff[s] = fr * CH + ((2 * s + fh) ^ kswz(fr));

    const int q_hi = qt * BQ + BQ - 1 < seq - 1 ? qt * BQ + BQ - 1 : seq - 1;   // last query row of the workgroup
    const int n_tiles = q_hi / BKV + 1;
    issue_tile(0, 0);
    for (int t = 0; t < n_tiles; ++t) {
        const int k0 = t * BKV;
        const u32x4 *ks = ks2[t & 1];
        const u32x4 *vs = vs2[t & 1];
        // this wave's pieces of tile t have landed; after the barrier everybody's have, and everybody is done
        // with tile t-1, whose buffer the next tile may now overwrite
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        const bool live = k0 <= q0 + 31;  // else: tile entirely in this wave's future (uniform per wave)
        // the first K fragments are asked for before the next tile's loads are issued: their LDS latency
        // passes while those instructions go out
        constexpr int KS = DH / 16, KRING = KS < 4 ? KS : 4;
        u32x4 kf[KRING][2];
        if (live) {
#pragma unroll
            for (int r = 0; r < KRING; ++r)
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) kf[r][kt] = ks[kt * 32 * CH + koff[r]];
        }
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < n_tiles) issue_tile(k0 + BKV, (t + 1) & 1);
        if (live) {

        // S^T tile: 64 keys x 32 queries = two 32 x 32 accumulators, advanced in turn so that consecutive
        // multiplies do not depend on each other.  K fragments run through a ring of four k-steps that is
        // refilled as it drains: an LDS read is always several multiplies ahead of its use (the
        // sched_barriers pin that order; left alone the compiler reads each fragment right before it).
        f32x16 sacc[2];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                if (s == 0) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.0f;
                }
                sacc[kt] = mfma32<DT>(__builtin_bit_cast(uint4, kf[s % KRING][kt]), qf[s], sacc[kt]);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (s + KRING < KS) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) kf[s % KRING][kt] = ks[kt * 32 * CH + koff[s + KRING]];
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the first V^T fragments are asked for now: they land while the softmax arithmetic runs
        constexpr int CT = DH / 32;
        v4i16 vf[2][CT][2];
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            vf[0][c][0] = vt_frag(vs, 0, c);
            vf[0][c][1] = vt_frag(vs, 8, c);
        }
        __builtin_amdgcn_sched_barrier(0);
        // mask (key > query) on the diagonal tiles, tile maximum of the raw scores
        if (k0 + BKV - 1 > q0) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = k0 + kt * 32 + 8 * (i >> 2) + 4 * fh + (i & 3);
                    if (key > qrow) sacc[kt][i] = -INFINITY;
                }
        }
        float tmax = sacc[0][0];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int i = 0; i < 16; i += 2) tmax = __builtin_fmaxf(__builtin_fmaxf(sacc[kt][i], sacc[kt][i + 1]), tmax);   // three-input maxima
        {
            float ha, hb;
            swap_halves(tmax, ha, hb);
            tmax = __builtin_fmaxf(ha, hb);
        }
        // m_run is the reference the exponentials are taken against, not the exact running maximum: it is
        // raised (and O and the normaliser rescaled) only when some row's scores pass it by more than 2^8 after
        // scaling, so after the first tiles almost no tile pays for the rescaling.  Probabilities then reach
        // 2^8 at most; the final division by the normaliser taken against the same reference cancels it.
        // First tile: m_run = -inf, every row moves (key k0 <= q0 <= qrow is never masked, so tmax is finite).
        if (__builtin_amdgcn_ballot_w64((tmax - m_run) * sc > 8.0f) != 0) {
            const float m_new = __builtin_fmaxf(tmax, m_run);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
            l_run *= alpha;
#pragma unroll
            for (int c = 0; c < DH / 32; ++c)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[c][i] *= alpha;
            m_run = m_new;
        }
        const float moff = -m_run * sc;
        float psum = 0.0f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kt][i], sc, moff));
                sacc[kt][i] = p;
                psum += p;
            }
        {
            float ha, hb;
            swap_halves(psum, ha, hb);
            l_run += ha + hb;
        }
        // O^T += V^T P^T : four contraction steps of 16 keys; lane half h contracts keys 16 s + 4 h + {0..3}
        // and 16 s + 8 + 4 h + {0..3}, the order in which the S^T accumulators hold them
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int kt = s >> 1, rb = (s & 1) * 8;
            uint4 pf;
            pf.x = pack2<DT>(sacc[kt][rb + 0], sacc[kt][rb + 1]);
            pf.y = pack2<DT>(sacc[kt][rb + 2], sacc[kt][rb + 3]);
            pf.z = pack2<DT>(sacc[kt][rb + 4], sacc[kt][rb + 5]);
            pf.w = pack2<DT>(sacc[kt][rb + 6], sacc[kt][rb + 7]);
            if (s + 1 < 4) {                                   // next step's V^T fragments, one step ahead
#pragma unroll
                for (int c = 0; c < CT; ++c) {
                    vf[(s + 1) & 1][c][0] = vt_frag(vs, 16 * (s + 1), c);
                    vf[(s + 1) & 1][c][1] = vt_frag(vs, 16 * (s + 1) + 8, c);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                const uint2 lo2 = __builtin_bit_cast(uint2, vf[s & 1][c][0]), hi2 = __builtin_bit_cast(uint2, vf[s & 1][c][1]);
                oacc[c] = mfma32<DT>(uint4{lo2.x, lo2.y, hi2.x, hi2.y}, pf, oacc[c]);
            }
            __builtin_amdgcn_sched_barrier(0);
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
    const long long pairs8 = ((long long)n_heads * n_seq + 7) / 8 * 8;
    const long long n_wg = pairs8 * ((seq + BQ - 1) / BQ);
    if (n_heads < 1 || n_seq < 1 || n_wg > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)n_wg), block(256);
    const uint16_t *q = (const uint16_t *)qkv;
    uint16_t *o = (uint16_t *)out;
    if (dtype == kBF16) {
        if (d_head == 64) attn_mfma_kernel<kBF16, 64><<<grid, block, 0, s>>>(q, o, seq, n_heads, n_seq);
        else attn_mfma_kernel<kBF16, 128><<<grid, block, 0, s>>>(q, o, seq, n_heads, n_seq);
    } else {
        if (d_head == 64) attn_mfma_kernel<kFP16, 64><<<grid, block, 0, s>>>(q, o, seq, n_heads, n_seq);
        else attn_mfma_kernel<kFP16, 128><<<grid, block, 0, s>>>(q, o, seq, n_heads, n_seq);
    }
    return hipGetLastError();
}

}  // namespace zo

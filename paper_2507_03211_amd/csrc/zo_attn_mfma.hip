// Causal multi-head attention on the matrix cores (bf16 / fp16 in, fp32 softmax statistics),
// part of the paired forward passes of Eq. 1 (DistZO2, Preliminaries).  Both signs are just
// more sequences: the kernel sees n_seq = 2 * batch independent sequences.
//
// One work item = (128 query rows, one head, one sequence); 4 waves x 32 query rows.  Persistent workgroups, as
// many as the chip holds at once, walk a per-XCD item list.  Key / value tiles of 64 keys stream through LDS.
// Everything is computed transposed so that a lane owns one query row:
//     S^T[key, q] = K Q^T        (MFMA A = K rows, B = Q rows; lane: column q, 16 keys)
//     O^T[c, q]  += V^T P^T      (MFMA A = V^T rows, B = P^T; lane: column q, 16 channels)
// so the online-softmax reference maximum, normaliser and the rescaling of O are per-lane scalars.  The contraction
// order of the P V product follows the accumulator layout of S^T (keys 16s + 4h + {0..3}, 16s + 8 + 4h + {0..3} for
// lane half h), which V^T is read with as well, so P never leaves registers.  V stays row-major in LDS; its
// transposed fragments come from the LDS transposing read of gfx950.  The key loop is software-pipelined in units of
// 32 keys: the vector arithmetic of one unit's softmax is issued between the matrix instructions of the next
// unit's scores and of its own P V product.
#include "zo_kernels.h"
#include "zo_types.hip.h"
#include <type_traits>

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
    constexpr int KS = DH / 16, CT = DH / 32;   // contraction steps of K Q^T, channel tiles of O^T
    constexpr int TILE = BKV * CH;        // 16-byte chunks per K / V tile
    // K and V tiles, both [key][channel] as they sit in memory, 16-byte chunks XOR-swizzled per key so that
    // the MFMA fragment reads of K (32 keys, one chunk) and the transposing reads of V (4 keys x 32 bytes
    // per 16 lanes) are free of conflicts on the 64-bank LDS.
    // Three K and two V buffers: tiles arrive (global memory straight into LDS) while earlier ones are multiplied.
    __shared__ u32x4 ks3[3][TILE];
    __shared__ u32x4 vs2[2][TILE];
    auto kswz = [](int r) { return DH == 128 ? (r & 15) : ((r >> 1) & 7); };
    auto vswz = [](int r) { return DH == 128 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); };

    const int d = n_heads * DH, ld = 3 * d;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, and known to be: it feeds scalar operands
    const int fr = lane & 31, fh = lane >> 5;
    // of the work item in hand (see the item loop at the end): its query tile, first query row of this wave, this
    // lane's query row, its first element in qkv as a pointer and as a wave-uniform address
    int q0 = 0, qrow = 0;
    const uint16_t *base = qkv;
    uint64_t gbase0 = 0;

    uint4 qf[KS];                                    // Q fragments: B operand, lane = (row fr, k half fh), all k-steps
    f32x16 oacc[CT];
    // reference maximum of the raw scores (see the key loop); l_lane: this lane's share of the normaliser (the keys
    // its half of the wave holds; the two halves are added once, at the end); sc = log2(e)/sqrt(d_head)
    const float sc = 1.4426950408889634f / __builtin_sqrtf((float)DH);
    const float lazy = 8.0f / sc;                    // the reference is raised when a raw score passes it by this
    float m_run = -INFINITY, l_lane = 0.0f, moff = 0.0f, thr = -INFINITY;   // (set per work item)

    // global -> LDS for a K/V tile, without passing through registers: one wave instruction moves 64 x 16
    // bytes and lane L's piece lands at the instruction's LDS base + 16 L.  Piece p = 64 (NLD wave + i) + L of
    // a tile is slot p % CH of key row p / CH; the slot holds logical chunk slot ^ swizzle(row), so the
    // swizzle is applied on the global side (still whole 16-byte pieces of one row per lane).  The lane part
    // of the address does not change from tile to tile: the key advance goes into a scalar base.
    constexpr int NLD = TILE / 256;       // instructions per wave and operand
    uint32_t kgo[NLD], vgo[NLD];          // byte offsets from the tile's first key row
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int pidx = 64 * (NLD * wave + i) + lane, r = pidx / CH, slot = pidx % CH;
        kgo[i] = (uint32_t)(r * ld + d + (slot ^ kswz(r)) * 8) * 2u;
        vgo[i] = (uint32_t)(r * ld + 2 * d + (slot ^ vswz(r)) * 8) * 2u;
    }
    const uint32_t ks_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)&ks3[0][0];
    const uint32_t vs_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)&vs2[0][0];
    auto dma16 = [](uint64_t gbase, uint32_t lane_off, uint32_t lds_off) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(gbase), "s"(lds_off) : "memory", "m0");
    };
    // this wave's pieces of K (which = 0) or V (which = 1) rows k0 .. k0 + 63, into buffer `buf` of that operand
    auto issue = [&](int which, int k0, int buf) {
        const uint32_t dst = (which ? vs_lds : ks_lds) + (uint32_t)buf * (TILE * 16) + (uint32_t)(NLD * wave) * 1024u;
        if (k0 + BKV <= seq) {
            const uint64_t gb = gbase0 + (uint64_t)k0 * (uint64_t)ld * 2u;
#pragma unroll
            for (int i = 0; i < NLD; ++i) dma16(gb, which ? vgo[i] : kgo[i], dst + i * 1024u);
        } else {
            // last, ragged tile of the sequence: key rows past its end re-read the last row (masked as future keys)
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int pidx = 64 * (NLD * wave + i) + lane, r = pidx / CH, slot = pidx % CH;
                const int kr = k0 + r < seq ? k0 + r : seq - 1;
                const int chunk = which ? (slot ^ vswz(r)) : (slot ^ kswz(r));
                dma16(gbase0, (uint32_t)(kr * ld + (which ? 2 * d : d) + chunk * 8) * 2u, dst + i * 1024u);
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
    int voff[CT];                                                // element offset of (key tr_key + 4 fh, channel tile c)
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        const int key = 4 * fh + tr_key, chan = c * 32 + tr_chan;
        voff[c] = (key * CH + ((chan >> 3) ^ vswz(key))) * 8 + (chan & 7);
    }
    auto vt_frag = [&](const u32x4 *vs, int kb16, int ctile) {   // keys kb16 + 4 fh + tr_key, kb16 a multiple of 8
        const uint16_t *p = (const uint16_t *)vs + voff[ctile] + kb16 * CH * 8;
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16 *)p);
    };
    int koff[KS];                                                // u32x4 index of (key fr, k-step s)
#pragma unroll
    for (int s = 0; s < KS; ++s) koff[s] = fr * CH + ((2 * s + fh) ^ kswz(fr));

    // The keys are worked in units of 32 (one 32 x 32 score block; a tile holds two), software-pipelined so that
    // the vector arithmetic of a unit's softmax is issued in the shadow of matrix instructions that do not depend
    // on it.  Step s of a wave:
    //     phase A   S(s+1) = K Q^T of the next unit          |  exponentials of the first 16 keys of unit s
    //     phase B   O^T += V^T P^T of unit s (first its 16   |  exponentials of its last 16 keys, then the
    //               keys done in phase A, then the rest)     |  maximum (and causal mask) of S(s+1)
    // A vector instruction issued right after a matrix instruction of the same wave runs beside it, so a step
    // costs about its 16 matrix instructions when the vector work (4 to 5 instructions per slot) fits under
    // them.  K fragments run through a ring of four that is refilled as it drains and runs on into the next unit;
    // V^T fragments are read one 16-key step ahead.  The sched_barriers pin the order written here.
    //
    // Tiles in LDS: K of tiles T, T+1 and the arriving T+2 (the pipeline reads K one unit ahead of V), V of tiles
    // T and the arriving T+1.  One barrier per tile: after it tile T+1's K and tile T's V have landed for
    // everybody (each wave waits for its own pieces first) and everybody is done with the buffers that the
    // loads issued next overwrite.  Those loads (K of tile T+2, V of tile T+1) go out together right after the
    // barrier: spread over the slots of a step they cost more, a wave that waits for the memory pipeline to accept
    // a load issues no multiplies either.
    int n_tiles = 0, u_last = 0;                     // of the work item: tiles of the workgroup, last unit of this wave
    int kb0 = 0, kb1 = 1, kb2 = 2;                   // K buffers of tiles T, T+1, T+2
    auto sync_tile = [&](int T) {                    // on entry to tile T
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (T + 2 < n_tiles) issue(0, (T + 2) * BKV, kb2);
        if (T + 1 < n_tiles) issue(1, (T + 1) * BKV, (T + 1) & 1);
    };

    f32x16 S[2];                                     // raw scores: S[s & 1] of unit s, the other of unit s + 1
    u32x4 kf[4];                                     // K fragment ring
    v4i16 vf[CT][2];                                 // V^T fragments of one 16-key step
    uint4 pf[2];                                     // probabilities of the unit's two 16-key steps, packed
    float tmax;                                      // this lane's maximum over S of the unit about to be exponentiated
    auto k_frag = [&](int buf, int half, int f) { return ks3[buf][half * 32 * CH + koff[f]]; };
    auto unit_max = [&](const f32x16 &x) {
        float t = __builtin_fmaxf(__builtin_fmaxf(x[0], x[1]), x[2]);
#pragma unroll
        for (int i = 3; i < 15; i += 2) t = __builtin_fmaxf(__builtin_fmaxf(x[i], x[i + 1]), t);
        return __builtin_fmaxf(t, x[15]);
    };
    auto causal_mask = [&](f32x16 &x, int key0) {    // key > query: a future key
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = key0 + 8 * (i >> 2) + 4 * fh + (i & 3);
            if (key > qrow) x[i] = -INFINITY;
        }
    };
    // scores of unit u from K buffer `buf`, half `half`, into dst; the ring then holds the first fragments of the
    // unit after it (buffer nbuf, half nhalf).  `between(i)`: what to issue after the i-th multiply.
    auto qk_unit = [&](f32x16 &dst, int buf, int half, int nbuf, int nhalf, auto &&between) {
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            if (i == 0) {
                const f32x16 zero = {};
                dst = mfma32<DT>(__builtin_bit_cast(uint4, kf[0]), qf[0], zero);
            } else {
                dst = mfma32<DT>(__builtin_bit_cast(uint4, kf[i % 4]), qf[i], dst);
            }
            __builtin_amdgcn_sched_barrier(0);       // the refill goes out after the multiply that frees its slot
            kf[i % 4] = i + 4 < KS ? k_frag(buf, half, i + 4) : k_frag(nbuf, nhalf, i + 4 - KS);
            between(i);
        }
    };
    // m_run is the reference the exponentials are taken against, not the exact running maximum: it is raised (and
    // O and the normaliser rescaled) only when some row's raw scores pass it by more than 2^8 after scaling, so
    // after the first units almost no step pays for the rescaling.  Probabilities then reach 2^8 at most; the
    // final division by the normaliser, taken against the same reference, cancels it.  A lane tests its own 16
    // keys; the two halves of the wave agree on the new reference only when one of them asks for it.
    // First unit: m_run = -inf and every row moves (key 0 is never masked, so the row maximum is finite).
    auto step = [&](auto hc, int s) {
        constexpr int H = decltype(hc)::value;       // s & 1: unit s is half H of tile T
        f32x16 &Sc = S[H], &Sn = S[H ^ 1];
        if (__builtin_amdgcn_ballot_w64(tmax > thr) != 0) {
            float ha, hb;
            swap_halves(tmax, ha, hb);
            const float m_new = __builtin_fmaxf(__builtin_fmaxf(ha, hb), m_run);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
            l_lane *= alpha;
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[c][i] *= alpha;
            m_run = m_new;
            moff = -m_new * sc;
            thr = m_new + lazy;
        }
        auto pre = [&](int e) { Sc[e] = __builtin_fmaf(Sc[e], sc, moff); };
        auto ex = [&](int e) {
            const float pe = __builtin_amdgcn_exp2f(Sc[e]);
            Sc[e] = pe;
            l_lane += pe;
            // (pinned here by the empty asm: left alone the compiler gathers the sixteen additions of a unit in one
            // place, a serial chain with no multiply to hide behind.  The addition itself stays the compiler's: it
            // has to keep the distance that a transcendental result needs before its first use.)
            asm volatile("" : "+v"(l_lane));
        };
        auto cvt = [&](int e) {                      // after elements e - 1 and e (e odd) are done
            const uint32_t w = pack2<DT>(Sc[e - 1], Sc[e]);
            uint4 &dst = pf[e >> 3];
            const int r = (e & 7) >> 1;
            if (r == 0) dst.x = w;
            else if (r == 1) dst.y = w;
            else if (r == 2) dst.z = w;
            else dst.w = w;
        };
        __builtin_amdgcn_sched_barrier(0);
        // phase A.  K of unit s + 1: H = 0: tile T, second half; H = 1: tile T + 1, first half.  Unit s + 2 is
        // tile T + 1 either way.
        qk_unit(Sn, H == 0 ? kb0 : kb1, H == 0 ? 1 : 0, kb1, H == 0 ? 0 : 1, [&](int i) {
            if (i < CT) {                            // V^T fragments of this unit's first 16 keys
                vf[i][0] = vt_frag(vs2[(s >> 1) & 1], 32 * H, i);
                vf[i][1] = vt_frag(vs2[(s >> 1) & 1], 32 * H + 8, i);
            }
            __builtin_amdgcn_sched_barrier(0);
            constexpr int PER = 8 / KS;              // elements of each 16-key step per slot
#pragma unroll
            for (int e = i * PER; e < (i + 1) * PER; ++e) {
                pre(e);
                ex(e);
                if (e & 1) cvt(e);
            }
#pragma unroll
            for (int e = 8 + i * PER; e < 8 + (i + 1) * PER; ++e) pre(e);
            __builtin_amdgcn_sched_barrier(0);
        });
        // phase B
#pragma unroll
        for (int j = 0; j < 2 * CT; ++j) {
            const int kstep = j / CT, c = j % CT;
            const uint2 lo2 = __builtin_bit_cast(uint2, vf[c][0]), hi2 = __builtin_bit_cast(uint2, vf[c][1]);
            oacc[c] = mfma32<DT>(uint4{lo2.x, lo2.y, hi2.x, hi2.y}, pf[kstep], oacc[c]);
            if (kstep == 0) {                        // the slot's fragments are in the matrix pipe: read the next step's
                vf[c][0] = vt_frag(vs2[(s >> 1) & 1], 32 * H + 16, c);
                vf[c][1] = vt_frag(vs2[(s >> 1) & 1], 32 * H + 24, c);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (kstep == 0) {
                constexpr int PER = 8 / CT;
#pragma unroll
                for (int e = 8 + c * PER; e < 8 + (c + 1) * PER; ++e) {
                    ex(e);
                    if (e & 1) cvt(e);
                }
            } else if (c == 0) {
                if (s + 1 == u_last) causal_mask(Sn, 32 * (s + 1));
            } else if (c == 1) {
                tmax = unit_max(Sn);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Work items: (query tile, head, sequence).  Persistent workgroups, as many as the chip holds at once: the
    // hardware deals consecutive workgroup ids round-robin to the 8 XCDs, so workgroup b sits on XCD b % 8 and is
    // that XCD's slot b / 8.  Every (head, sequence) pair goes to one XCD with all its query tiles, so the XCDs hold
    // equal shares of the causal triangle and the K and V of a pair are fetched into one L2 instead of eight.  The
    // XCD's items are listed in groups of as many pairs as fill its slots once, long rows first within a group, and
    // slot j takes entry j of the even rounds and entry slots - 1 - j of the odd ones: a long tile is followed by
    // a short one and every slot ends up with the same number of key tiles.
    const int n_qt = (seq + BQ - 1) / BQ;
    const int slots = (int)gridDim.x >> 3, slot = (int)blockIdx.x >> 3, xcd = (int)blockIdx.x & 7;
    const int n_pairs = n_heads * n_seq, pairs_xcd = (n_pairs + 7) / 8;
    const int group_pairs = slots / n_qt > 1 ? slots / n_qt : 1, group_items = group_pairs * n_qt;
    const int n_lin = (pairs_xcd + group_pairs - 1) / group_pairs * group_items;
    for (int round = 0; round * slots < n_lin; ++round) {
        const int lin = round * slots + ((round & 1) ? slots - 1 - slot : slot);
        if (lin >= n_lin) continue;
        const int grp = lin / group_items, r = lin % group_items;
        const int gp = pairs_xcd - grp * group_pairs < group_pairs ? pairs_xcd - grp * group_pairs : group_pairs;
        if (r >= gp * n_qt) continue;
        const int pair = (grp * group_pairs + r % gp) * 8 + xcd;
        if (pair >= n_pairs) continue;
        const int qt = n_qt - 1 - r / gp;
        const int head = pair % n_heads, sq = pair / n_heads;
        base = qkv + (size_t)sq * seq * ld + head * DH;
        // (the halves go through unsigned 32-bit variables: readfirstlane returns a signed int, which would
        // sign-extend into the upper half)
        const uint32_t gb_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)base);
        const uint32_t gb_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)base >> 32));
        gbase0 = ((uint64_t)gb_hi << 32) | (uint64_t)gb_lo;
        q0 = qt * BQ + wave * 32;
        qrow = q0 + fr;
        const int qload = qrow < seq ? qrow : seq - 1;
        const int q_hi = qt * BQ + BQ - 1 < seq - 1 ? qt * BQ + BQ - 1 : seq - 1;   // last query row of the workgroup
        n_tiles = q_hi / BKV + 1;
        // last unit this wave needs (the one on its diagonal); a wave whose rows all lie past a ragged end stops with
        // the last unit loaded, its results are not stored
        u_last = q0 / 32 < 2 * n_tiles - 1 ? q0 / 32 : 2 * n_tiles - 1;
        kb0 = 0, kb1 = 1, kb2 = 2;
        m_run = -INFINITY, l_lane = 0.0f, moff = 0.0f, thr = -INFINITY;
        // everybody is done with the LDS tiles of the previous item: the first tiles of this one go out, then Q is
        // read while they fly
        __syncthreads();
        issue(0, 0, 0);
        issue(1, 0, 0);
        if (n_tiles > 1) issue(0, BKV, 1);
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s] = *(const uint4 *)(base + (size_t)qload * ld + s * 16 + fh * 8);
        // The Q loads are made to land here, before the key loop.  Otherwise the compiler waits for them where the
        // loop first uses them, by counting outstanding memory operations, and inside the loop that count also
        // holds the next tile's global->LDS loads (issued from asm, unknown to the compiler): every tile would
        // wait for its successor's data.
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(qf[s].x), "v"(qf[s].y), "v"(qf[s].z), "v"(qf[s].w));
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[c][i] = 0.0f;
        sync_tile(0);

        // prologue: scores of unit 0, nothing to overlap them with
    #pragma unroll
        for (int r = 0; r < 4; ++r) kf[r] = k_frag(0, 0, r);
        qk_unit(S[0], 0, 0, 0, 1, [](int) { __builtin_amdgcn_sched_barrier(0); });
        if (u_last == 0) causal_mask(S[0], 0);
        tmax = unit_max(S[0]);


        for (int T = 0; T < n_tiles; ++T) {
            if (2 * T <= u_last) step(std::integral_constant<int, 0>{}, 2 * T);
            if (2 * T + 1 <= u_last) step(std::integral_constant<int, 1>{}, 2 * T + 1);
            if (T + 1 < n_tiles) {
                const int k = kb0;                       // tile T's K buffer takes tile T + 3
                kb0 = kb1;
                kb1 = kb2;
                kb2 = k;
                sync_tile(T + 1);
            }
        }
        float l_run;
        {
            float ha, hb;
            swap_halves(l_lane, ha, hb);
            l_run = ha + hb;
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
}

}  // namespace

bool mfma_attention_supported(int seq, int d_head) { return seq >= 1 && (d_head == 64 || d_head == 128); }

hipError_t launch_attention_mfma(const void *qkv, void *out, int dtype, int n_seq, int seq, int n_heads, int d_head,
                                 hipStream_t s)
{
    if (!mfma_attention_supported(seq, d_head) || (dtype != kBF16 && dtype != kFP16)) return hipErrorInvalidValue;
    if (n_heads < 1 || n_seq < 1) return hipErrorInvalidValue;
    // persistent workgroups: as many as are resident at once (2 per CU at d_head 128, 3 at 64; the CU count is
    // rounded down to whole XCDs' worth), fewer when there are fewer work items
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        n_cu = v >= 8 ? v / 8 * 8 : 8;
    }
    const long long pairs_xcd = ((long long)n_heads * n_seq + 7) / 8;
    const long long items_xcd = pairs_xcd * ((seq + BQ - 1) / BQ);
    const long long slots_max = (long long)(n_cu / 8) * (d_head == 64 ? 3 : 2);
    if (items_xcd > 0x7fffffffLL / 64) return hipErrorInvalidValue;      // the kernel's item indices are ints
    const dim3 grid((unsigned)(8 * (items_xcd < slots_max ? items_xcd : slots_max))), block(256);
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

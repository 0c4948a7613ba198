/*
 * CPU oracle, part 1: the random direction z and the in-place perturbation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP library is checked against.  Nothing in the product path may call it,
 * and it shares no code, header, table or constant generator with the HIP
 * sources: every constant below is typed in here by hand from the written
 * specification of the generator.
 *
 * What it follows (DistZO2, arXiv 2507.03211):
 *   - Preliminaries, Eq. 1-2: z ~ N(0, I), theta <- theta -/+ (scalar) * z.
 *   - Appendix A, Alg. 1 (MeZO): PerturbParameters / UpdateParameters visit
 *     every tensor, draw z_i of that tensor's shape and add (scalar * z_i);
 *     the generator is reset to the step's seed before each pass so that all
 *     passes of one step see the same z.
 *   - PertP workflow, Step 1: a shared seed must give the same z everywhere.
 * The paper names no generator.  The reading taken here: z is a pure function
 * of (seed, tensor id, element index) through the counter-based Philox4x32-10
 * generator (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
 * 1, 2, 3", SC'11) followed by a pair-wise Box-Muller transform whose fp32
 * arithmetic is fixed operation by operation, so that "reset the seed" becomes
 * "use the same counters" and the bits can be reproduced on any IEEE-754
 * machine.  The transform is laid out so that a GPU needs few instructions
 * for it (a table of piecewise cubics takes the place of logarithm and square
 * root, the angle's sign bits take the place of quadrant logic); what it
 * computes is the textbook Rayleigh radius times (cos, sin) of a uniform
 * angle, which is what the pins check it against.
 *
 * Precision: z is DEFINED in fp32 (this is part of the method's specification,
 * not an approximation of something else); the perturbation is one fp32 fused
 * multiply-add followed by round-to-nearest-even into the storage type.
 *
 * Pins (tests/test_oracle_rng.py): published Philox known-answer vectors, a
 * second implementation with Python integers, the closed form
 * (Rayleigh quantile) x (cos, sin)(angle) in fp64, moments and a KS test, numpy's
 * float16 cast for the half rounding, chunking invariance.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---------------------------------------------------------------- Philox */

/* One Philox4x32 block, 10 rounds.  The round, as the SC'11 paper defines it:
 *   (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0))
 * with the key bumped by the Weyl constants between rounds. */
void zo_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += W0; k1 += W1; }
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Counter layout: key = (seed low word, seed high word);
 * counter = (j low word, j high word, tensor id, stream tag), j = element/4.
 * Stream tag 0 is the perturbation direction z. */
static void block_for(uint64_t seed, uint32_t tensor_id, uint32_t stream_tag, uint64_t j, uint32_t out[4])
{
    uint32_t ctr[4] = { (uint32_t)j, (uint32_t)(j >> 32), tensor_id, stream_tag };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    zo_oracle_philox4x32_10(ctr, key, out);
}

/* ------------------------------------------------------ normal transform */

static float u32_as_f32(uint32_t x) { float f; memcpy(&f, &x, 4); return f; }
static uint32_t f32_as_u32(float f) { uint32_t x; memcpy(&x, &f, 4); return x; }

/* Two standard normals from two 32-bit words (pair-wise Box-Muller):
 *   rho   = a radius with the Rayleigh distribution, drawn by inverting its distribution function
 *           F(rho) = 1 - exp(-rho^2 / 2) at F uniform over (0,1)   [the textbook rho = sqrt(-2 ln U)]
 *   x     = (float)(int32_t)rb * 2^-31            in [-1, 1]: a quarter turn either way
 *   z1    = rho * sin(pi x / 2)
 *   z0    = +-rho * cos(pi x / 2), negative when bit 31 of ra is set
 * ((cos, sin) of an angle uniform over the right half circle with an independent fair sign on the
 * cosine is uniform over the circle.)  Every floating-point step is a single IEEE fp32 operation
 * (conversion, add, mul, fma), written out in the order the specification gives it.
 *
 * The radius.  q = (2 j + 1) 2^-25 with j = bits 30..8 of ra lies in (0, 1/2); bit 4 of ra says which
 * half of the distribution it measures:
 *   h = 0:  F = q,       rho = sqrt(-2 ln(1 - q))     (rho below the median)
 *   h = 1:  1 - F = q,   rho = sqrt(-2 ln q)          (rho above the median)
 * so that F is uniform over (0,1) and either end is resolved with the relative precision of a
 * floating-point q.  Both functions are smooth in the RELATIVE position of q inside a binade, so
 * each is tabulated piecewise: qf = (float)((2 j + 1) 2^7) is exact, its biased exponent E
 * (134..157) and top five fraction bits jj select one of 24 x 32 cells, the cell's pivot pf is its
 * midpoint (fraction bits jj, then a one, then zeros), and with d = qf - pf (exact)
 *   rho = a0 + d (a1 + d (a2 + d a3))
 * where a_k = fl32 of the k-th Taylor coefficient of rho_h at the pivot with respect to d
 * (|d| / pf <= 2^-6, the truncation error is below 0.05 ulp).  The coefficients are worked out below
 * from the derivatives of t = -2 ln g, g = 1 - q or q, and rho = sqrt(t), in double precision. */
static float rayleigh_cell[2][24 * 32][4];

__attribute__((constructor)) static void rayleigh_cells_init(void)
{
    for (int h = 0; h < 2; ++h)
        for (int E = 134; E < 158; ++E)
            for (int jj = 0; jj < 32; ++jj) {
                const double q = ldexp(1.0 + ((double)jj + 0.5) / 32.0, E - 127 - 32);   /* the pivot as a probability */
                const double g = h ? q : 1.0 - q, dg = h ? 1.0 : -1.0;                  /* g and dg/dq */
                const double t = h ? -2.0 * log(q) : -2.0 * log1p(-q);
                const double t1 = -2.0 * dg / g, t2 = 2.0 / (g * g), t3 = -4.0 * dg / (g * g * g);
                const double rho = sqrt(t);
                const double r1 = t1 / (2.0 * rho);
                const double r2 = t2 / (2.0 * rho) - t1 * t1 / (4.0 * rho * rho * rho);
                const double r3 = t3 / (2.0 * rho) - 3.0 * t1 * t2 / (4.0 * rho * rho * rho)
                                  + 3.0 * t1 * t1 * t1 / (8.0 * rho * rho * rho * rho * rho);
                float *a = rayleigh_cell[h][(E - 134) * 32 + jj];
                /* d counts in units of 2^-32 of q: each derivative order takes one factor 2^-32 */
                a[0] = (float)rho;
                a[1] = (float)ldexp(r1, -32);
                a[2] = (float)ldexp(r2 / 2.0, -64);
                a[3] = (float)ldexp(r3 / 6.0, -96);
            }
}

void zo_oracle_normal_pair(uint32_t ra, uint32_t rb, float *z0, float *z1)
{
    /* radius */
    const float qf = (float)((ra & 0x7FFFFF00u) | 0x80u);  /* (2 j + 1) 2^7, exact: 24 significant bits */
    const uint32_t b = f32_as_u32(qf);
    const float pf = u32_as_f32((b & 0xFFFC0000u) | 0x00020000u);
    const float d = qf - pf;                               /* exact */
    const float *a = rayleigh_cell[(ra >> 4) & 1u][(b >> 18) - 134u * 32u];
    float rho = fmaf(a[3], d, a[2]);
    rho = fmaf(rho, d, a[1]);
    rho = fmaf(rho, d, a[0]);

    /* angle: x in [-1, 1], w = x^2 */
    const float x = (float)(int32_t)rb * 0x1p-31f;        /* the conversion rounds to nearest even; the scaling is exact */
    const float w = x * x;
    float S = 0x1.3e17cap-13f;                            /* sin(pi x/2) = x * S(w) */
    S = fmaf(S, w, -0x1.32535ap-8f);
    S = fmaf(S, w, 0x1.4668f2p-4f);
    S = fmaf(S, w, -0x1.4abbc4p-1f);
    S = fmaf(S, w, 0x1.921fb6p+0f);
    const float sn = x * S;
    float Cc = -0x1.93c734p-16f;                          /* cos(pi x/2) = 1 + w * C(w) */
    Cc = fmaf(Cc, w, 0x1.e173cap-11f);
    Cc = fmaf(Cc, w, -0x1.55d268p-6f);
    Cc = fmaf(Cc, w, 0x1.03c1eep-2f);
    Cc = fmaf(Cc, w, -0x1.3bd3ccp+0f);
    const float cs = fmaf(w, Cc, 1.0f);
    /* z0 takes its sign from bit 31 of ra (the magnitude's own sign bit, which can be set by a rounding
     * error of cs at |x| = 1, is dropped) */
    const uint32_t mag = f32_as_u32(rho * cs) & 0x7FFFFFFFu;
    *z0 = u32_as_f32(mag | (ra & 0x80000000u));
    *z1 = rho * sn;
}

/* The transform alone over an array of word pairs: z[2i], z[2i+1] from words[2i], words[2i+1]. */
void zo_oracle_normal_pairs(const uint32_t *words, float *z, uint64_t n_pairs)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n_pairs; ++i)
        zo_oracle_normal_pair(words[2 * i], words[2 * i + 1], &z[2 * i], &z[2 * i + 1]);
}

/* z for the elements [first, first+n) of one tensor.  Words (r0,r1) of block j
 * give elements 4j and 4j+1, words (r2,r3) give 4j+2 and 4j+3. */
void zo_oracle_z(uint64_t seed, uint32_t tensor_id, uint32_t stream_tag, uint64_t first, uint64_t n, float *out)
{
    if (n == 0) return;
    #pragma omp parallel for schedule(static)
    for (int64_t jj = (int64_t)(first / 4); jj <= (int64_t)((first + n - 1) / 4); ++jj) {
        uint32_t w[4];
        float z[4];
        block_for(seed, tensor_id, stream_tag, (uint64_t)jj, w);
        zo_oracle_normal_pair(w[0], w[1], &z[0], &z[1]);
        zo_oracle_normal_pair(w[2], w[3], &z[2], &z[3]);
        for (int l = 0; l < 4; ++l) {
            uint64_t i = 4u * (uint64_t)jj + (uint64_t)l;
            if (i >= first && i < first + n) out[i - first] = z[l];
        }
    }
}

/* --------------------------------------------------- storage-type rounding */

/* dtype codes of the boundary: 0 fp32, 1 bf16, 2 fp16. */
uint16_t zo_oracle_f32_to_bf16(float f)
{
    uint32_t x = f32_as_u32(f);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x0040u); /* quiet NaN */
    uint32_t lsb = (x >> 16) & 1u;
    x += 0x7fffu + lsb;                                   /* round to nearest, ties to even */
    return (uint16_t)(x >> 16);
}
float zo_oracle_bf16_to_f32(uint16_t h) { return u32_as_f32((uint32_t)h << 16); }

uint16_t zo_oracle_f32_to_f16(float f)
{
    uint32_t x = f32_as_u32(f);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t a = x & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);           /* NaN */
    if (a >= 0x47800000u) {                                            /* >= 65536: Inf (or Inf in) */
        return (uint16_t)(sign | 0x7c00u);
    }
    if (a >= 0x38800000u) {                                            /* normal half range: >= 2^-14 */
        uint32_t mant = a & 0x007fffffu;
        uint32_t exp = (a >> 23) - 112u;                               /* rebias 127 -> 15 */
        uint32_t h = (exp << 10) | (mant >> 13);
        uint32_t rem = mant & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) h += 1u;    /* may carry into exponent / Inf: correct */
        return (uint16_t)(sign | h);
    }
    if (a < 0x33000000u) return sign;                                  /* < 2^-25: rounds to zero */
    /* subnormal half: value = mant24 * 2^(e-150), result unit 2^-24 */
    uint32_t mant = (a & 0x007fffffu) | 0x00800000u;
    uint32_t shift = 126u - (a >> 23);                                 /* 14..24 */
    uint32_t h = mant >> shift;
    uint32_t rem = mant & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1u);
    if (rem > half || (rem == half && (h & 1u))) h += 1u;
    return (uint16_t)(sign | h);
}
float zo_oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1fu, mant = h & 0x3ffu;
    if (exp == 0x1fu) return u32_as_f32(sign | 0x7f800000u | (mant << 13));
    if (exp != 0) return u32_as_f32(sign | ((exp + 112u) << 23) | (mant << 13));
    float v = (float)mant * 0x1p-24f;                                  /* subnormal or zero, exact */
    return sign ? -v : v;
}

static float load_as_f32(const void *p, int dtype, uint64_t i)
{
    if (dtype == 0) return ((const float *)p)[i];
    if (dtype == 1) return zo_oracle_bf16_to_f32(((const uint16_t *)p)[i]);
    return zo_oracle_f16_to_f32(((const uint16_t *)p)[i]);
}
static void store_from_f32(void *p, int dtype, uint64_t i, float v)
{
    if (dtype == 0) ((float *)p)[i] = v;
    else if (dtype == 1) ((uint16_t *)p)[i] = zo_oracle_f32_to_bf16(v);
    else ((uint16_t *)p)[i] = zo_oracle_f32_to_f16(v);
}

/* ---------------------------------------------------- perturb and update */

/* Alg. 1, PerturbParameters / UpdateParameters for one tensor (or a slice of
 * it): dst[i] <- rn(fma(scale, z_i, src[i])) for i in [first, first+n), where
 * the pointers address element `first`.  dst may equal src (in place).
 * scale = +eps, -2 eps, +eps for the three perturbations and -(lr*g) for the
 * update of Eq. 2. */
void zo_oracle_axpy_z(const void *src, void *dst, int dtype, uint64_t seed, uint32_t tensor_id,
                      uint64_t first, uint64_t n, float scale)
{
    if (n == 0) return;
    #pragma omp parallel for schedule(static)
    for (int64_t jj = (int64_t)(first / 4); jj <= (int64_t)((first + n - 1) / 4); ++jj) {
        uint32_t w[4];
        float z[4];
        block_for(seed, tensor_id, 0u, (uint64_t)jj, w);
        zo_oracle_normal_pair(w[0], w[1], &z[0], &z[1]);
        zo_oracle_normal_pair(w[2], w[3], &z[2], &z[3]);
        for (int l = 0; l < 4; ++l) {
            uint64_t i = 4u * (uint64_t)jj + (uint64_t)l;
            if (i < first || i >= first + n) continue;
            float th = load_as_f32(src, dtype, i - first);
            store_from_f32(dst, dtype, i - first, fmaf(scale, z[l], th));
        }
    }
}

/* ------------------------------------------- stochastic rounding (opt-in) */

/* An opt-in variant of the update of Eq. 2, not part of the paper's method:
 * the paper stores parameters in 16 bits ("FP16 mode", Sec. 7) and applies
 * theta <- theta - eta g z in that type; with round-to-nearest almost every
 * such update of a weight is lost (|eta g z| << ulp(theta) / 2, tested in
 * tests/test_oracle_step.py).  Stochastic rounding keeps the update unbiased:
 * the fp32 value v = fma(s, z, theta) goes to one of its two neighbours in
 * the storage type, the farther-from-zero one with probability equal to the
 * fraction of the way v lies from the nearer-to-zero one.
 *
 * Exact definition (integer arithmetic only, so the bits reproduce anywhere):
 * write |v| = (n + f) * u with u the spacing of the storage type at |v|,
 * n an integer and 0 <= f < 1.  F = floor(f * 2^24).  With r = word >> 8
 * (the top 24 bits of the element's random word) the magnitude becomes
 * (n + 1) * u if r < F and n * u otherwise; the sign is kept.  A value the
 * storage type represents has f = 0 and never moves.  Non-finite v passes
 * through as under round-to-nearest; a magnitude that rounds up past the
 * largest finite value becomes infinity.
 *
 * The random word of element i is word (i % 4) of the Philox block with
 * counter (i / 4, tensor id, tag 3) under the step's seed: independent of the
 * z of the same element (tag 0). */
uint16_t zo_oracle_sr_bf16(float v, uint32_t word)
{
    uint32_t bits;
    memcpy(&bits, &v, 4);
    const uint32_t sign = (bits >> 16) & 0x8000u, mag = bits & 0x7FFFFFFFu;
    if (mag >= 0x7F800000u) return zo_oracle_f32_to_bf16(v);
    /* bf16 keeps the top 16 bits of the fp32 pattern: n = those, f = the low 16 bits / 2^16 */
    const uint32_t n = mag >> 16, F = (mag & 0xFFFFu) << 8, r = word >> 8;
    return (uint16_t)(sign | (n + (r < F ? 1u : 0u)));
}

uint16_t zo_oracle_sr_f16(float v, uint32_t word)
{
    uint32_t bits;
    memcpy(&bits, &v, 4);
    const uint32_t sign = (bits >> 16) & 0x8000u, mag = bits & 0x7FFFFFFFu;
    if (mag >= 0x7F800000u) return zo_oracle_f32_to_f16(v);
    const uint32_t e = mag >> 23, m = mag & 0x7FFFFFu, r = word >> 8;
    uint32_t n, F;
    if (e >= 143u) return (uint16_t)(sign | 0x7C00u);          /* |v| >= 2^16: beyond the half range */
    if (e >= 113u) {
        /* normal half: exponent field e - 112, ten fraction bits kept, thirteen dropped */
        n = ((e - 112u) << 10) | (m >> 13);
        F = (m & 0x1FFFu) << 11;
    } else {
        /* below 2^-14 the spacing is 2^-24: |v| = sig * 2^(ee - 150), so n + f = sig / 2^s with s = 126 - ee */
        const uint32_t sig = e ? (m | 0x800000u) : m, ee = e ? e : 1u;
        const uint32_t s = 126u - ee;                           /* 14 .. 125 */
        if (s <= 24u) {
            n = sig >> s;
            F = (sig & ((1u << s) - 1u)) << (24u - s);
        } else {
            n = 0u;
            F = (s - 24u) < 32u ? sig >> (s - 24u) : 0u;
        }
    }
    return (uint16_t)(sign | (n + (r < F ? 1u : 0u)));
}

/* dst[i] = sr(fma(scale, z[i], src[i])): as zo_oracle_axpy_z with the rounding above.
 * dtype 1 (bf16) or 2 (fp16) only. */
void zo_oracle_axpy_z_sr(const void *src, void *dst, int dtype, uint64_t seed, uint32_t tensor_id,
                         uint64_t first, uint64_t n, float scale)
{
    if (n == 0) return;
    #pragma omp parallel for schedule(static)
    for (int64_t jj = (int64_t)(first / 4); jj <= (int64_t)((first + n - 1) / 4); ++jj) {
        uint32_t w[4], rw[4];
        float z[4];
        block_for(seed, tensor_id, 0u, (uint64_t)jj, w);
        block_for(seed, tensor_id, 3u, (uint64_t)jj, rw);
        zo_oracle_normal_pair(w[0], w[1], &z[0], &z[1]);
        zo_oracle_normal_pair(w[2], w[3], &z[2], &z[3]);
        for (int l = 0; l < 4; ++l) {
            uint64_t i = 4u * (uint64_t)jj + (uint64_t)l;
            if (i < first || i >= first + n) continue;
            const float v = fmaf(scale, z[l], load_as_f32(src, dtype, i - first));
            ((uint16_t *)dst)[i - first] = dtype == 1 ? zo_oracle_sr_bf16(v, rw[l]) : zo_oracle_sr_f16(v, rw[l]);
        }
    }
}

/* Element-wise stochastic rounding of n fp32 values with given random words (for the pins). */
void zo_oracle_sr_array(const float *v, const uint32_t *word, uint16_t *out, int dtype, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = dtype == 1 ? zo_oracle_sr_bf16(v[i], word[i]) : zo_oracle_sr_f16(v[i], word[i]);
}

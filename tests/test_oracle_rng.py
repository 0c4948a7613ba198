"""Pins for the oracle's random direction z and in-place perturbation
(oracle/zo_oracle_rng.c): things fixed by the published generator, by the
closed form of the Box-Muller transform, by library casts and by exact
rational arithmetic -- never by the oracle's own output."""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

from oracle import philox_ints
from oracle import zo_oracle as zo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat():
    rows = []
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[0:4], w[4:6], tuple(w[6:10])))
    return rows


def test_philox_known_answers_c_and_python():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert zo.philox(ctr, key) == want
        assert philox_ints.philox4x32(ctr, key) == want


def test_philox_two_implementations_agree_on_random_counters():
    rng = np.random.default_rng(7)
    for _ in range(300):
        ctr = [int(x) for x in rng.integers(0, 2**32, 4)]
        key = [int(x) for x in rng.integers(0, 2**32, 2)]
        assert zo.philox(ctr, key) == philox_ints.philox4x32(ctr, key)


def test_philox_fewer_rounds_differ():
    # a dropped round must not go unnoticed
    assert philox_ints.philox4x32((0, 0, 0, 0), (0, 0), rounds=9) != zo.philox((0, 0, 0, 0), (0, 0))


def _closed_form(ra, rb):
    """The transform's definition, in fp64.  Radius: q = (2 j + 1) 2^-25 with j = bits 30..8 of ra; bit 4 of ra clear:
    F = q, radius sqrt(-2 ln(1 - q)); set: 1 - F = q, radius sqrt(-2 ln q) (the Rayleigh quantile at F).  Angle: a quarter
    turn times x, x = the fp32 nearest to rb read as a signed integer, times 2^-31.  z1 = radius sin, z0 = -+radius cos
    with the sign in bit 31 of ra."""
    q = (2 * ((ra >> 8) & 0x7FFFFF) + 1) / 2.0**25
    rho = np.sqrt(-2.0 * np.log(q)) if (ra >> 4) & 1 else np.sqrt(-2.0 * np.log1p(-q))
    signed = rb - (1 << 32) if rb >= (1 << 31) else rb
    ang = float(np.float32(signed)) * 2.0**-31 * (np.pi / 2)
    return (-1.0 if ra >> 31 else 1.0) * rho * np.cos(ang), rho * np.sin(ang)


def _closed_form_arrays(ra, rb):
    """The same over uint32 arrays."""
    q = (2.0 * ((ra >> np.uint32(8)) & np.uint32(0x7FFFFF)).astype(np.float64) + 1.0) * 2.0**-25
    upper = ((ra >> np.uint32(4)) & np.uint32(1)) == 1
    rho = np.where(upper, np.sqrt(-2.0 * np.log(q)), np.sqrt(-2.0 * np.log1p(-q)))
    ang = rb.view(np.int32).astype(np.float32).astype(np.float64) * 2.0**-31 * (np.pi / 2)
    sign = np.where(ra >> np.uint32(31), -1.0, 1.0)
    return sign * rho * np.cos(ang), rho * np.sin(ang), rho


def test_counter_layout_words_to_elements():
    # element 4j+l of tensor t under seed s comes from Philox(counter=(j lo, j hi, t, 0), key=(s lo, s hi)):
    # words (0,1) -> elements 4j, 4j+1 ; words (2,3) -> elements 4j+2, 4j+3
    for seed, t, j in [(42, 0, 0), (42, 0, 1), (42, 1, 0), (2**40 + 5, 33, 2**31 + 3), (7, 66, 12345),
                       (9, 2, 2**33 + 5), (2**63 + 1, 1921, 2**35 + 2**32 - 1)]:      # block index beyond 32 bits: the counter's second word
        w = philox_ints.words_for(seed, t, j)
        z = zo.z_values(seed, t, 4 * j, 4)
        for pair in range(2):
            c0, c1 = _closed_form(w[2 * pair], w[2 * pair + 1])
            assert abs(z[2 * pair] - c0) < 2e-6 * max(1.0, abs(c0))
            assert abs(z[2 * pair + 1] - c1) < 2e-6 * max(1.0, abs(c1))


def test_normal_pair_matches_closed_form_everywhere():
    rng = np.random.default_rng(11)
    ras = list(rng.integers(0, 2**32, 20000)) + [0, 0x10, 0x100, 0x110, 0x7FFFFF00, 0x7FFFFF10, 0xFFFFFFFF, 0xFFFFFFEF, 0x80000000,
                                                 0x80000010, 0x40000000, 0x3FFFFF10, 0x00000FFF, 0x000080FF]
    rbs = list(rng.integers(0, 2**32, 20000)) + [0, 0x7FFFFFFF, 0x80000000, 0xFFFFFFFF, 0x40000000, 0xC0000000, 1, 0x7FFFFF80,
                                                 0x7FFFFFC0, 0x80000040, 0x01000001, 0xFEFFFFFF, 0x12345678, 0x9ABCDEF0]
    worst = 0.0
    for ra, rb in zip(ras, rbs):
        ra, rb = int(ra), int(rb)
        z0, z1 = zo.normal_pair(ra, rb)
        c0, c1 = _closed_form(ra, rb)
        rho = np.hypot(c0, c1)
        # error relative to the radius: a few fp32 ulps
        worst = max(worst, abs(z0 - c0) / rho, abs(z1 - c1) / rho)
    assert worst < 4 * 2.0**-23, worst


@pytest.mark.parametrize("upper", [0, 1])
def test_every_radius_code_matches_closed_form(upper):
    """All 2^23 values of q in either half of the distribution, the cosine's sign alternating: z0 = -+radius at angle
    0, within 2 ulp of the Rayleigh quantile, and monotone in q (a wrong cell, pivot or coefficient breaks the order)."""
    j = np.arange(2**23, dtype=np.uint32)
    ra = (j << np.uint32(8)) | np.uint32(upper << 4) | ((j & np.uint32(1)) << np.uint32(31))
    words = np.empty(2 * ra.size, dtype=np.uint32)
    words[0::2] = ra
    words[1::2] = 0
    z = zo.normal_pairs(words)
    c0, _, rho = _closed_form_arrays(ra, np.zeros_like(ra))
    assert np.all(z[1::2] == 0)
    assert np.all(np.signbit(z[0::2]) == (c0 < 0))
    err = np.abs(z[0::2].astype(np.float64) - c0) / np.spacing(rho.astype(np.float32)).astype(np.float64)
    assert err.max() < 2.0, (err.max(), int(err.argmax()))
    mag = np.abs(z[0::2]).astype(np.float64)
    if upper:
        assert np.all(mag[1:] <= mag[:-1]) and abs(mag[0] - np.sqrt(50 * np.log(2))) < 1e-6      # q = 2^-25
        assert abs(mag[-1] - np.sqrt(2 * np.log(2))) < 1e-6                                       # the median, from above
    else:
        assert np.all(mag[1:] >= mag[:-1]) and abs(mag[0] / np.sqrt(2.0**-24) - 1) < 1e-6         # sqrt(-2 ln(1 - 2^-25))
        assert abs(mag[-1] - np.sqrt(2 * np.log(2))) < 1e-6                                       # the median, from below


def test_every_angle_code_matches_closed_form():
    """All 2^24 angles rb = i << 8 (every value of the top 24 bits, both signs) at a fixed radius: absolute error of
    (cos, sin) within 3 fp32 ulps of 1, and cos^2 + sin^2 = 1."""
    rb = np.arange(2**24, dtype=np.uint64).astype(np.uint32) << np.uint32(8)
    ra = np.full(rb.size, 0x64E85C00, dtype=np.uint32)             # F = 0.394..., radius about 1
    words = np.empty(2 * rb.size, dtype=np.uint32)
    words[0::2] = ra
    words[1::2] = rb
    z = zo.normal_pairs(words).astype(np.float64)
    c0, c1, rho = _closed_form_arrays(ra, rb)
    assert 0.99 < rho[0] < 1.01
    assert np.max(np.abs(z[0::2] - c0)) < 3 * 2.0**-23 and np.max(np.abs(z[1::2] - c1)) < 3 * 2.0**-23
    assert np.max(np.abs((z[0::2]**2 + z[1::2]**2) / rho**2 - 1)) < 1e-6
    assert np.all(z[1::2][1:2**23] > 0) and np.all(z[1::2][2**23:] < 0) and z[1] == 0        # the sine carries the sign of rb


def test_normal_radius_identity_and_extremes():
    # z0^2 + z1^2 = radius^2 = -2 ln(1 - F); the largest radius at 1 - F = 2^-25, the smallest at F = 2^-25
    for ra, rb in [(0, 0x12345678), (0xFFFFFFFF, 0x9ABCDEF0), (0x40000010, 0), (0x12345678, 0x40000000)]:
        z0, z1 = zo.normal_pair(ra, rb)
        q = (2 * ((ra >> 8) & 0x7FFFFF) + 1) / 2.0**25
        f = 1 - q if (ra >> 4) & 1 else q
        assert abs((float(z0)**2 + float(z1)**2) / (-2 * np.log1p(-f)) - 1) < 1e-6
    s = float(np.sqrt(50 * np.log(2)))
    z0, z1 = zo.normal_pair(0x10, 0)
    assert abs(float(z0) - s) < 1e-5 and z1 == 0
    z0, z1 = zo.normal_pair(0, 0)
    assert abs(float(z0) / np.sqrt(-2 * np.log1p(-2.0**-25)) - 1) < 1e-6
    # the two halves meet at the median of the radius, sqrt(2 ln 2)
    lo, hi = float(zo.normal_pair(0x7FFFFF00, 0)[0]), float(zo.normal_pair(0x7FFFFF10, 0)[0])
    assert lo < np.sqrt(2 * np.log(2)) < hi and hi - lo < 1e-6
    # directions: angle 0 is the +-z0 axis (sign in bit 31 of ra), a quarter turn either way the +-z1 axis, and the
    # four sign combinations at an eighth of a turn land in the four quadrants
    assert [float(v) for v in zo.normal_pair(0x80000010, 0)] == [-float(np.float32(s)), 0.0]
    z0, z1 = zo.normal_pair(0x10, 0x7FFFFFFF)
    assert abs(float(z1) - s) < 1e-5 and abs(float(z0)) < 1e-6
    z0, z1 = zo.normal_pair(0x10, 0x80000000)
    assert abs(float(z1) + s) < 1e-5 and abs(float(z0)) < 1e-6
    quads = [np.sign(zo.normal_pair(ra, rb)).tolist() for ra in (0x10, 0x80000010) for rb in (0x40000000, 0xC0000000)]
    assert quads == [[1, 1], [1, -1], [-1, 1], [-1, -1]]
    z0, z1 = zo.normal_pair(0x10, 0x40000000)
    assert abs(float(z0) - s / np.sqrt(2)) < 1e-5 and abs(float(z1) - s / np.sqrt(2)) < 1e-5


def test_z_is_standard_normal():
    z = zo.z_values(123, 5, 0, 1 << 22).astype(np.float64)
    n = z.size
    assert abs(z.mean()) < 5 / np.sqrt(n)
    assert abs(z.var() - 1) < 5 * np.sqrt(2 / n)
    assert abs(stats.skew(z)) < 5 * np.sqrt(6 / n)
    assert abs(stats.kurtosis(z)) < 5 * np.sqrt(24 / n)
    assert stats.kstest(z[:200000], "norm").pvalue > 1e-3
    # neighbours (same pair, adjacent pairs, adjacent blocks) are uncorrelated
    for lag in (1, 2, 4):
        assert abs(np.mean(z[:-lag] * z[lag:])) < 5 / np.sqrt(n)


def test_same_seed_same_z_any_chunking():
    full = zo.z_values(42, 3, 0, 1003)
    again = zo.z_values(42, 3, 0, 1003)
    assert full.tobytes() == again.tobytes()
    pieces = [zo.z_values(42, 3, a, b - a) for a, b in [(0, 1), (1, 2), (2, 7), (7, 8), (8, 513), (513, 1003)]]
    assert np.concatenate(pieces).tobytes() == full.tobytes()
    assert zo.z_values(42, 3, 0, 0).size == 0
    assert zo.z_values(43, 3, 0, 64).tobytes() != full[:64].tobytes()
    assert zo.z_values(42, 4, 0, 64).tobytes() != full[:64].tobytes()
    assert zo.z_values(42, 3, 0, 64, stream_tag=1).tobytes() != full[:64].tobytes()
    # beyond 2^32 elements the high counter word takes over
    hi = zo.z_values(42, 3, 2**34, 8)
    w = philox_ints.words_for(42, 3, 2**32)
    assert abs(hi[0] - _closed_form(w[0], w[1])[0]) < 1e-5


def _bits_sample(rng, n):
    x = rng.integers(0, 2**32, n, dtype=np.uint64).astype(np.uint32).view(np.float32)
    near = rng.standard_normal(n).astype(np.float32) * np.float32(6e-5)   # half subnormals
    ties = (rng.integers(0, 2**16, n, dtype=np.uint64).astype(np.uint32) << 16 | 0x8000).view(np.float32)
    big = rng.standard_normal(n).astype(np.float32) * np.float32(65504)
    x = np.concatenate([x, near, ties, big, np.float32([0.0, -0.0, 65504, 65520, 65519.99, 2.0**-24, 2.0**-25,
                                                       1.5 * 2.0**-25, 2.0**-14, np.inf, -np.inf])])
    return x[np.isfinite(x) | np.isinf(x)]


def test_half_and_bfloat_rounding_match_library_casts():
    import torch
    rng = np.random.default_rng(3)
    x = _bits_sample(rng, 50000)
    x = x[~np.isnan(x)]
    lib = zo._clib()
    with np.errstate(over="ignore"):
        want16 = x.astype(np.float16).view(np.uint16)
    got16 = np.array([lib.zo_oracle_f32_to_f16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got16, want16)
    wantb = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    gotb = np.array([lib.zo_oracle_f32_to_bf16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(gotb, wantb)
    assert np.array_equal(zo.to_storage(x, zo.BF16), wantb)
    # widening is exact
    h = np.arange(0, 2**16, dtype=np.uint16)
    back = np.array([lib.zo_oracle_f16_to_f32(int(v)) for v in h], dtype=np.float32)
    ref = h.view(np.float16).astype(np.float32)
    ok = ~np.isnan(ref)
    assert np.array_equal(back[ok], ref[ok])


def _exact_fma_error_ok(scale, z, theta, result):
    """|result - (scale*z + theta)| <= half an ulp of result, in exact rationals."""
    exact = Fraction(float(scale)) * Fraction(float(z)) + Fraction(float(theta))
    r = float(result)
    ulp = Fraction(float(np.spacing(np.float32(abs(r)) if r != 0 else np.float32(0))))
    return abs(Fraction(r) - exact) <= ulp / 2


def test_axpy_fp32_is_a_correctly_rounded_fma():
    rng = np.random.default_rng(5)
    theta = (0.02 * rng.standard_normal(600)).astype(np.float32)
    z = zo.z_values(9, 17, 0, 600)
    for scale in (np.float32(1e-3), np.float32(-2e-3), np.float32(-3.3e-6)):
        out = zo.axpy_z(theta, zo.FP32, 9, 17, scale)
        assert all(_exact_fma_error_ok(scale, z[i], theta[i], out[i]) for i in range(600))
    # a separately rounded multiply then add differs somewhere: the fused form is what is specified
    unfused = (np.float32(1e-3) * z).astype(np.float32) + theta
    assert np.any(unfused != zo.axpy_z(theta, zo.FP32, 9, 17, np.float32(1e-3)))


@pytest.mark.parametrize("dtype", [zo.BF16, zo.FP16])
def test_axpy_low_precision_rounds_the_fp32_fma(dtype):
    rng = np.random.default_rng(6)
    x32 = (0.02 * rng.standard_normal(5000)).astype(np.float32)
    theta = zo.to_storage(x32, dtype)
    wide = zo.widen(theta, dtype).astype(np.float32)
    z = zo.z_values(1, 2, 0, 5000)
    scale = np.float32(1e-3)
    # fp64 product-sum of fp32 values rounded to fp32 equals the fp32 fma except on
    # double-rounding ties, which this sample is checked not to contain
    f32 = (np.float64(scale) * z.astype(np.float64) + wide.astype(np.float64)).astype(np.float32)
    want = zo.to_storage(f32, dtype)
    got = zo.axpy_z(theta, dtype, 1, 2, scale)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("dtype", [zo.FP32, zo.BF16, zo.FP16])
def test_zero_scale_and_slices(dtype):
    rng = np.random.default_rng(8)
    theta = zo.to_storage((0.02 * rng.standard_normal(1001)).astype(np.float32), dtype)
    assert zo.axpy_z(theta, dtype, 4, 4, 0.0).tobytes() == theta.tobytes()
    whole = zo.axpy_z(theta, dtype, 4, 4, 1e-3)
    parts = [zo.axpy_z(theta[a:b], dtype, 4, 4, 1e-3, first=a) for a, b in [(0, 3), (3, 3), (3, 510), (510, 1001)]]
    assert np.concatenate(parts).tobytes() == whole.tobytes()


def test_perturb_cycle_returns_within_one_ulp_fp32():
    rng = np.random.default_rng(9)
    theta = (0.02 * rng.standard_normal(20000)).astype(np.float32)
    t = theta.copy()
    eps = np.float32(1e-3)
    for s in (eps, -2 * eps, eps):
        zo.axpy_z(t, zo.FP32, 42, 0, s, out=t)
    # each of the three roundings is at most half an ulp at magnitude <= |theta| + 2 eps |z|
    bound = 1.5 * np.spacing(np.abs(theta) + 2 * eps * np.abs(zo.z_values(42, 0, 0, 20000)))
    assert np.all(np.abs(t - theta) <= bound)
    assert np.mean(t == theta) > 0.3

"""Pins for the oracle's opt-in stochastic rounding of the update (oracle/zo_oracle_rng.c,
zo_oracle_sr_*): exact rational arithmetic on the neighbours that numpy's casts give, exact
counts over all 2^24 random values, and the unbiasedness that is the point of it."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import philox_ints
from oracle import zo_oracle as zo


def _f16_neighbours(v):
    """(lo, hi): the float16 magnitudes that bracket |v| (equal when representable), as Fractions."""
    a = abs(float(v))
    with np.errstate(over="ignore"):
        c = np.float16(a)
    if np.isinf(c):
        c = np.float16(65504.0)
    cf = float(c)
    if cf == a:
        return Fraction(cf), Fraction(cf)
    if cf < a:
        with np.errstate(over="ignore"):
            up = np.nextafter(c, np.float16(np.inf))
        return Fraction(cf), (Fraction(float(up)) if np.isfinite(up) else Fraction(65536))
    return Fraction(float(np.nextafter(c, np.float16(0.0)))), Fraction(cf)


def _bf16_value(pattern):
    return float(np.array([pattern << 16], dtype=np.uint32).view(np.float32)[0])


def _bf16_neighbours(v):
    a = abs(float(v))
    p = int(zo.to_storage(np.array([a], dtype=np.float32), zo.BF16)[0])       # nearest-even pattern (library-pinned elsewhere)
    for cand in (p - 1, p, p + 1):
        if cand < 0:
            continue
        lo, hi = _bf16_value(cand), _bf16_value(cand + 1)
        if lo == a:
            return Fraction(lo), Fraction(lo)
        if lo < a < hi:
            return Fraction(lo), Fraction(hi) if np.isfinite(hi) else Fraction(2) ** 128
    raise AssertionError(a)


def _expected(v, word, dtype):
    lo, hi = (_f16_neighbours if dtype == zo.FP16 else _bf16_neighbours)(v)
    if lo == hi:
        mag = lo
    else:
        f = (Fraction(abs(float(v))) - lo) / (hi - lo)
        F = (f * 2**24).__floor__()
        mag = hi if (word >> 8) < F else lo
    return -mag if np.signbit(np.float32(v)) else mag


def _as_fraction(out, dtype):
    if dtype == zo.FP16:
        x = float(out)
    else:
        x = _bf16_value(int(out))
    if np.isinf(x):
        return Fraction(65536 if dtype == zo.FP16 else 2**128) * (1 if x > 0 else -1)
    return Fraction(x)


@pytest.mark.parametrize("dtype", [zo.BF16, zo.FP16])
def test_stochastic_rounding_against_exact_rationals(dtype):
    rng = np.random.default_rng(11 + dtype)
    # every exponent the type sees, including the half's subnormal range, the last binade, tiny and zero
    exps = rng.integers(-45 if dtype == zo.FP16 else -130, 16 if dtype == zo.FP16 else 127, 3000)
    v = (rng.uniform(1.0, 2.0, exps.size) * np.exp2(exps.astype(np.float64)) * rng.choice([-1.0, 1.0], exps.size)).astype(np.float32)
    edge = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.0, 65535.0, 2.0**-24, 2.0**-25, 1.5 * 2.0**-24, 2.0**-14, 2.0**-14 * (1 - 2.0**-12),
            6.1e-5, 3e-8, 1e-10, 1e-38, 1e-40]
    v = np.concatenate([v, np.array(edge, dtype=np.float32)])
    words = rng.integers(0, 2**32, v.size, dtype=np.uint64).astype(np.uint32)
    words[::7] = 0
    words[3::7] = 0xFFFFFFFF
    got = zo.sr_round(v, words, dtype)
    for i in range(v.size):
        want = _expected(v[i], int(words[i]), dtype)
        assert _as_fraction(got[i], dtype) == want, (i, float(v[i]), hex(int(words[i])))


@pytest.mark.parametrize("dtype", [zo.BF16, zo.FP16])
def test_probability_of_rounding_up_is_the_fraction_counted_over_all_random_values(dtype):
    r = np.arange(2**24, dtype=np.uint32) << 8            # every value of the 24 bits that decide
    for v in (np.float32(0.02) * np.float32(1.0003), np.float32(-3.14159), np.float32(2.0**-20 * 1.37)):
        lo, hi = (_f16_neighbours if dtype == zo.FP16 else _bf16_neighbours)(v)
        F = ((Fraction(abs(float(v))) - lo) / (hi - lo) * 2**24).__floor__()
        out = zo.sr_round(np.full(r.shape, v, np.float32), r, dtype)
        mags = np.abs(zo.widen(out, dtype)) if dtype == zo.BF16 else np.abs(out.astype(np.float64))
        assert set(np.unique(mags)) <= {float(lo), float(hi)}
        assert int((mags == float(hi)).sum()) == F
        # the low 8 bits of the word play no part
        assert np.array_equal(zo.sr_round(np.full(1000, v, np.float32), r[:1000] | 0xFF, dtype).view(np.uint16),
                              out[:1000].view(np.uint16))


@pytest.mark.parametrize("dtype", [zo.BF16, zo.FP16])
def test_representable_values_never_move(dtype):
    pats = np.arange(65536, dtype=np.uint16)
    with np.errstate(invalid="ignore"):
        vals = zo.widen(pats if dtype == zo.BF16 else pats.view(np.float16), dtype)
    finite = np.isfinite(vals)
    v32 = vals[finite].astype(np.float32)
    for w in (0, 0x7FFFFFFF, 0xFFFFFFFF):
        out = zo.sr_round(v32, np.full(v32.shape, w, np.uint32), dtype)
        assert np.array_equal(out.view(np.uint16), pats[finite])


def test_axpy_with_stochastic_rounding_uses_tag_three_words_and_any_chunking():
    rng = np.random.default_rng(5)
    n, seed, tid, scale = 1003, 77, 9, np.float32(3e-4)
    for dtype in (zo.BF16, zo.FP16):
        th = zo.to_storage(0.02 * rng.standard_normal(n), dtype)
        whole = zo.axpy_z(th, dtype, seed, tid, scale, stochastic=True)
        # rebuilt from parts: the fp32 fma of the plain path (pinned by exact rationals in test_oracle_rng.py),
        # the words of tag 3 from the Python-integer generator
        v = zo.axpy_z(zo.widen(th, dtype).astype(np.float32), zo.FP32, seed, tid, scale)
        words = np.array([philox_ints.words_for(seed, tid, i // 4, 3)[i % 4] for i in range(n)], dtype=np.uint32)
        assert np.array_equal(whole.view(np.uint16), zo.sr_round(v, words, dtype).view(np.uint16))
        for first, cnt in ((0, 1), (1, 6), (5, 498), (503, 500)):
            part = zo.axpy_z(th[first:first + cnt], dtype, seed, tid, scale, first=first, stochastic=True)
            assert np.array_equal(part.view(np.uint16), whole[first:first + cnt].view(np.uint16))
        # and it is not the nearest rounding
        assert not np.array_equal(whole.view(np.uint16), zo.axpy_z(th, dtype, seed, tid, scale).view(np.uint16))


def test_stochastically_rounded_update_is_unbiased_where_nearest_loses_it():
    rng = np.random.default_rng(3)
    n, scale = 1 << 20, np.float32(1e-6)
    th = zo.to_storage(0.02 * rng.standard_normal(n), zo.BF16)
    z = zo.z_values(123, 4, 0, n).astype(np.float64)
    before = zo.widen(th, zo.BF16)
    near = zo.widen(zo.axpy_z(th, zo.BF16, 123, 4, scale), zo.BF16) - before
    stoch = zo.widen(zo.axpy_z(th, zo.BF16, 123, 4, scale, stochastic=True), zo.BF16) - before
    want = np.float64(scale) * z
    big = np.abs(before) > 0.01                     # spacing >= 2^-14 = 6e-5 >> |scale z|
    assert (near[big] != 0).mean() < 1e-3           # round-to-nearest: the update is lost
    slope = float((stoch[big] * want[big]).sum() / (want[big] ** 2).sum())
    assert abs(slope - 1.0) < 0.06, slope           # stochastic: the expected step is the asked one
    moved = stoch[big] != 0
    assert 1e-3 < moved.mean() < 0.1                # a few elements take a whole spacing each
    assert np.all(np.sign(stoch[big][moved]) == np.sign(want[big][moved]))


def test_step_with_stochastic_update_moves_theta_along_minus_g_z():
    import zo_inputs as zi
    c = zi.CONFIGS["tiny"]
    cfg = zo.Config(c["n_layers"], c["d_model"], c["n_heads"], c["d_ffn"], c["vocab"], c["max_pos"], zo.BF16)
    theta = zi.make_weights(cfg.shapes(), zo.BF16, seed=0)
    tok = zi.make_tokens(c["batch"], c["seq"], c["vocab"])
    th_n = [t.copy() for t in theta]
    th_s = [t.copy() for t in theta]
    lp, lm, g = zo.zo_step_fused(cfg, th_n, tok, 42, 1e-3, 1e-6)
    lp2, lm2, g2 = zo.zo_step_fused(cfg, th_s, tok, 42, 1e-3, 1e-6, stochastic_update=True)
    assert (lp, lm, g) == (lp2, lm2, g2)            # the forward passes do not change
    num = den = 0.0
    for i, t0 in enumerate(theta):
        d = zo.widen(th_s[i], zo.BF16) - zo.widen(t0, zo.BF16)
        want = float(zo.step_scalar(1e-6, g)) * zo.z_values(42, i, 0, t0.size).reshape(t0.shape).astype(np.float64)
        num += float((d * want).sum())
        den += float((want ** 2).sum())
    assert 0.5 < num / den < 1.5, num / den         # 135k parameters: unbiased within the sampling noise

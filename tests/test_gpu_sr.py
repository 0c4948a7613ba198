"""GPU parity for the opt-in stochastic rounding of the update: the kernel must reproduce the oracle's
bits; at model level the forward is untouched, theta' lands on the oracle's two neighbours, the step is
unbiased, and the streamed schedule gives the resident one's bits."""
import numpy as np
import pytest
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from oracle import zo_oracle as zo
from gpu_util import DEV, Model, to_dev, to_host

pytestmark = pytest.mark.gpu


def _theta_all_ranges(rng, n, dtype):
    """Weights of the usual size plus every exponent range the rounding treats differently."""
    x = (0.02 * rng.standard_normal(n)).astype(np.float32)
    k = min(n, 4096) // 4
    if k:
        x[:k] = (rng.uniform(1.0, 2.0, k) * np.exp2(rng.integers(-30, 15, k).astype(np.float64)) * rng.choice([-1.0, 1.0], k)).astype(np.float32)
    edge = [0.0, -0.0, 1e-40, -1e-40, 6e-8, 65504.0, -65504.0, 60000.0, 2.0**-14, 2.0**-24, 1.0, -1.0, 3.0e38 if dtype == zi.BF16 else 4.0e4]
    m = min(n, len(edge))
    x[:m] = edge[:m]
    return zi.round_to_storage(x, dtype)


@pytest.mark.parametrize("dtype", [zi.BF16, zi.FP16])
@pytest.mark.parametrize("n", [1, 7, 8, 4096, 4097, 3 * 4096 + 13, 1 << 20])
def test_axpy_stochastic_bits_exact(dtype, n):
    rng = np.random.Generator(np.random.PCG64(1000 + n))
    theta = _theta_all_ranges(rng, max(n, 16), dtype)[:n]
    for scale in (1e-3, -3.17e-6, 1e-7, 37.5, 0.0):
        src = to_dev(theta, dtype)
        dst = torch.empty_like(src)
        zo_amd.zo_kernel_axpy_z_sr(src, dst, dtype, n, 42, 5, scale)
        got = to_host(dst, dtype)
        want = zo.axpy_z(theta, dtype, 42, 5, scale, stochastic=True)
        assert got.view(np.uint16).tobytes() == want.view(np.uint16).tobytes(), (dtype, n, scale)
    # in place, scalar read from device memory (the form the update inside zo_step uses), another seed / tensor
    src = to_dev(theta, dtype)
    dev_scale = torch.tensor([-1.25e-6], dtype=torch.float32, device=DEV)
    zo_amd.zo_kernel_axpy_z_sr(src, src, dtype, n, 2**40 + 3, 66, 123.0, dev_scale)
    want = zo.axpy_z(theta, dtype, 2**40 + 3, 66, np.float32(-1.25e-6), stochastic=True)
    assert to_host(src, dtype).view(np.uint16).tobytes() == want.view(np.uint16).tobytes()


def test_rounding_mode_argument_checks():
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_kernel_axpy_z_sr(torch.zeros(8, device=DEV), torch.zeros(8, device=DEV), zi.FP32, 8, 1, 1, 1e-3)
    f32 = Model(1, 64, 2, 128, 100, 16, zi.FP32, 1, 8)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_update_rounding(f32.handle, zo_amd.ZO_ROUND_STOCHASTIC)
    zo_amd.zo_set_update_rounding(f32.handle, zo_amd.ZO_ROUND_NEAREST)
    f32.close()
    b16 = Model(1, 64, 2, 128, 100, 16, zi.BF16, 1, 8)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_update_rounding(b16.handle, 7)
    b16.close()


SHAPE = dict(n_layers=2, d_model=128, n_heads=4, d_ffn=512, vocab=1000, max_pos=64)


@pytest.mark.parametrize("dtype", [zi.BF16, zi.FP16])
def test_step_with_stochastic_update_against_oracle(dtype):
    # learning rates at which |s z| stays below the spacing of a weight of size 0.01 and more (the paper's
    # regime): such a weight either stays or takes one whole spacing in the direction of s z, whatever
    # the exact size of s, so the oracle's two neighbours do not depend on the few percent by which the
    # GPU's g (16-bit activations) differs from the oracle's
    lr = 1e-6 if dtype == zi.BF16 else 1e-7
    near = Model(**SHAPE, dtype=dtype, batch=2, seq=40, seed=3, plain_small=False, std=0.05)
    stoch = Model(**SHAPE, dtype=dtype, batch=2, seq=40, seed=3, plain_small=False, std=0.05)
    zo_amd.zo_set_update_rounding(stoch.handle, zo_amd.ZO_ROUND_STOCHASTIC)
    tok, tok_dev = near.tokens()
    a = zo_amd.zo_step(near.handle, tok_dev, 2, 40, 9, 1e-3, lr)
    b = zo_amd.zo_step(stoch.handle, tok_dev, 2, 40, 9, 1e-3, lr)
    assert a == b                                         # the rounding mode touches the update only
    # the oracle's own step (its g differs from the GPU's by the 16-bit activation noise)
    theta = [t.copy() for t in stoch.theta0]
    olp, olm, og = zo.zo_step_fused(stoch.ocfg, theta, tok, 9, 1e-3, lr, stochastic_update=True)
    assert abs(b[2] / og - 1) < 0.2, (b[2], og)
    s_o = zo.step_scalar(lr, og)
    got, got_near = stoch.theta(), near.theta()
    inside = total = 0
    num = den = 0.0
    moved_s = moved_n = 0
    for i, t0 in enumerate(stoch.theta0):
        v = zo.axpy_z(zo.widen(t0, dtype).astype(np.float32), zi.FP32, 9, i, s_o)          # fma(s, z, theta) in fp32
        down = zo.sr_round(v, np.full(v.shape, 0xFFFFFFFF, np.uint32), dtype).view(np.uint16)
        up = zo.sr_round(v, np.zeros(v.shape, np.uint32), dtype).view(np.uint16)
        g16 = got[i].view(np.uint16)
        big = np.abs(zo.widen(t0, dtype)) > 0.01
        assert float(np.abs(v[big] - zo.widen(t0, dtype)[big].astype(np.float32)).max(initial=0.0)) < 2.0 ** (-14 if dtype == zi.BF16 else -17)
        inside += int(((g16 == down) | (g16 == up))[big].sum())
        total += int(big.sum())
        want = float(s_o) * zo.z_values(9, i, 0, t0.size).reshape(t0.shape).astype(np.float64)
        d = zo.widen(got[i], dtype) - zo.widen(t0, dtype)
        num += float((d * want).sum())
        den += float((want ** 2).sum())
        moved_s += int((got[i].view(np.uint16) != t0.view(np.uint16))[big].sum())
        moved_n += int((got_near[i].view(np.uint16) != t0.view(np.uint16))[big].sum())
    assert total > 100000 and inside == total, (inside, total)   # theta' sits on the oracle's two neighbours
    assert 0.7 < num / den < 1.3, num / den               # the step taken is the step asked for, on average
    assert moved_s > 1000 and moved_n < moved_s // 20     # weights of that size moved; under round-to-nearest (almost) none did
    near.close(); stoch.close()


@pytest.mark.parametrize("dtype", [zi.BF16, zi.FP16])
def test_streamed_equals_resident_with_stochastic_update(dtype):
    kw = dict(dtype=dtype, batch=2, seq=40, seed=3, plain_small=False, std=0.05)
    res, stm = Model(**SHAPE, **kw), Model(**SHAPE, streamed=True, **kw)
    for mdl in (res, stm):
        zo_amd.zo_set_update_rounding(mdl.handle, zo_amd.ZO_ROUND_STOCHASTIC)
    tok, tok_dev = res.tokens()
    for seed in (0, 1, 2):
        assert zo_amd.zo_step(res.handle, tok_dev, 2, 40, seed, 1e-3, 1e-4) == zo_amd.zo_step(stm.handle, tok_dev, 2, 40, seed, 1e-3, 1e-4)
    zo_amd.zo_flush_pending(stm.handle)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(res.theta(), stm.theta()))
    assert any(x.tobytes() != y.tobytes() for x, y in zip(res.theta(), res.theta0))
    res.close(); stm.close()

"""GPU parity, part 5: the deferred update on a resident model (Alg. 2's order: the update of step j-1 is applied
when step j next reads the parameters, here inside the staging pass) must leave exactly the bits that the
immediate update leaves, and the staging pass with the update folded in must match the oracle's update followed
by the oracle's perturbation bit for bit."""
import numpy as np
import pytest
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from oracle import zo_oracle as zo
from gpu_util import DEV, Model, to_dev, to_host

pytestmark = pytest.mark.gpu

SHAPE = dict(n_layers=3, d_model=128, n_heads=2, d_ffn=256, vocab=512, max_pos=64)


@pytest.mark.parametrize("dtype,stochastic", [(zi.FP32, False), (zi.BF16, False), (zi.FP16, False), (zi.BF16, True), (zi.FP16, True)])
@pytest.mark.parametrize("rows,cols,transpose", [(64, 64, True), (100, 72, True), (200, 264, True), (130, 8, True),
                                                 (1, 4099, False), (37, 100, False), (300, 768, False)])
def test_stage_with_update_bits_exact(dtype, stochastic, rows, cols, transpose):
    rng = np.random.Generator(np.random.PCG64(rows * 1000 + cols + 7))
    theta = zi.round_to_storage((0.02 * rng.standard_normal((rows, cols))).astype(np.float32), dtype)
    s = np.float32(-3.7e-3)
    src = to_dev(theta, dtype)
    wp, wm = torch.zeros_like(src).reshape(-1), torch.zeros_like(src).reshape(-1)
    dev_scale = torch.tensor([float(s)], dtype=torch.float32, device=DEV)
    eps = 1e-3
    zo_amd.zo_kernel_stage_update_pm(src, wp, wm, dtype, rows, cols, transpose, 77, 9, eps, 55, dev_scale, stochastic)
    updated = zo.axpy_z(theta, dtype, 55, 9, s, stochastic=stochastic)          # Eq. 2 with the step's z
    assert to_host(src, dtype).tobytes() == updated.tobytes()
    assert updated.tobytes() != theta.tobytes()
    want_p = zo.axpy_z(updated, dtype, 77, 9, eps)
    want_m = zo.axpy_z(updated, dtype, 77, 9, -np.float32(eps))
    if transpose:
        want_p, want_m = np.ascontiguousarray(want_p.T), np.ascontiguousarray(want_m.T)
    assert to_host(wp, dtype).tobytes() == want_p.tobytes()
    assert to_host(wm, dtype).tobytes() == want_m.tobytes()


@pytest.mark.parametrize("dtype,lr,stochastic", [(zi.BF16, 3e-2, False), (zi.FP16, 3e-3, False), (zi.FP32, 1e-3, False),
                                                 (zi.BF16, 1e-3, True), (zi.FP16, 1e-4, True)])
def test_deferred_equals_immediate_bit_for_bit(dtype, lr, stochastic):
    kw = dict(dtype=dtype, batch=2, seq=40, seed=3, plain_small=False, std=0.05)
    now, later = Model(**SHAPE, **kw), Model(**SHAPE, **kw)
    if stochastic:
        for mdl in (now, later):
            zo_amd.zo_set_update_rounding(mdl.handle, zo_amd.ZO_ROUND_STOCHASTIC)
    zo_amd.zo_set_deferred_update(later.handle, 1)
    tok, tok_dev = now.tokens()
    for seed in (0, 1, 2, 3):
        a = zo_amd.zo_step(now.handle, tok_dev, 2, 40, seed, 1e-3, lr)
        b = zo_amd.zo_step(later.handle, tok_dev, 2, 40, seed, 1e-3, lr)
        assert a == b, (seed, a, b)                          # the same arithmetic per element in the same order
    th = now.theta()
    assert any(x.tobytes() != y.tobytes() for x, y in zip(th, later.theta()))      # the last update is still pending
    assert any(x.tobytes() != y.tobytes() for x, y in zip(later.theta0, later.theta()))   # the earlier ones are in
    zo_amd.zo_flush_pending(later.handle)
    zo_amd.zo_flush_pending(later.handle)                    # nothing left: a no-op
    assert all(x.tobytes() == y.tobytes() for x, y in zip(th, later.theta()))
    now.close(); later.close()


def test_pending_update_is_applied_before_anything_else_touches_theta():
    kw = dict(dtype=zi.BF16, batch=2, seq=40, seed=5, plain_small=False, std=0.05)
    now, later = Model(**SHAPE, **kw), Model(**SHAPE, **kw)
    zo_amd.zo_set_deferred_update(later.handle, 1)
    tok, tok_dev = now.tokens()
    lr = 3e-2
    # a fused dual forward takes the pending update on its way
    assert zo_amd.zo_step(now.handle, tok_dev, 2, 40, 1, 1e-3, lr) == zo_amd.zo_step(later.handle, tok_dev, 2, 40, 1, 1e-3, lr)
    assert zo_amd.zo_dual_forward(now.handle, tok_dev, 2, 40, 2, 1e-3) == zo_amd.zo_dual_forward(later.handle, tok_dev, 2, 40, 2, 1e-3)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(now.theta(), later.theta()))
    # a literal-mode step: pending update first, its own update at once
    assert zo_amd.zo_step(now.handle, tok_dev, 2, 40, 3, 1e-3, lr) == zo_amd.zo_step(later.handle, tok_dev, 2, 40, 3, 1e-3, lr)
    a = zo_amd.zo_step(now.handle, tok_dev, 2, 40, 4, 1e-3, lr, zo_amd.ZO_MODE_LITERAL)
    b = zo_amd.zo_step(later.handle, tok_dev, 2, 40, 4, 1e-3, lr, zo_amd.ZO_MODE_LITERAL)
    assert a == b
    assert all(x.tobytes() == y.tobytes() for x, y in zip(now.theta(), later.theta()))
    # zo_perturb, and switching the mode off
    assert zo_amd.zo_step(now.handle, tok_dev, 2, 40, 5, 1e-3, lr) == zo_amd.zo_step(later.handle, tok_dev, 2, 40, 5, 1e-3, lr)
    zo_amd.zo_perturb(now.handle, 9, 1e-3, 0, 4)
    zo_amd.zo_perturb(later.handle, 9, 1e-3, 0, 4)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(now.theta(), later.theta()))
    assert zo_amd.zo_step(now.handle, tok_dev, 2, 40, 6, 1e-3, lr) == zo_amd.zo_step(later.handle, tok_dev, 2, 40, 6, 1e-3, lr)
    zo_amd.zo_set_deferred_update(later.handle, 0)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(now.theta(), later.theta()))
    assert zo_amd.zo_step(now.handle, tok_dev, 2, 40, 7, 1e-3, lr) == zo_amd.zo_step(later.handle, tok_dev, 2, 40, 7, 1e-3, lr)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(now.theta(), later.theta()))
    # a streamed model has no such switch
    stm = Model(**SHAPE, streamed=True, **kw)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_deferred_update(stm.handle, 1)
    now.close(); later.close(); stm.close()

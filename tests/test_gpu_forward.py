"""GPU parity, part 2: each forward kernel and the whole dual forward / step against the
oracle on the same seeded inputs.

Tolerances.  fp32 parameters run with fp64 activations and accumulation, so only summation
order differs from the oracle: 1e-9 relative on activations; g (a difference of two nearly
equal losses, magnified by 1/(2 eps) = 500) within 1e-6 relative here, 100x inside the 1e-4 the
configuration asks for.  2-byte types round activations to 8 (bf16) or 11 (fp16) significand
bits between kernels and accumulate in fp32: per-kernel bounds are a few units of that
rounding on the result's scale (stated per test); losses within 2e-2 relative.
"""
import numpy as np
import pytest
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from oracle import zo_oracle as zo
from gpu_util import DEV, Model, act_dtype, act_to_dev, resid_dtype, to_dev, to_host

pytestmark = pytest.mark.gpu

ULP = {zi.FP32: 1e-12, zi.BF16: 2.0**-8, zi.FP16: 2.0**-11}


def _rounded_act(x64, dtype):
    """What the kernel really receives: activations rounded to the activation type, back in fp64."""
    return act_to_dev(x64, dtype).double().cpu().numpy()


def _weights(rng, shape, dtype, std=0.05):
    return zi.round_to_storage((std * rng.standard_normal(shape)).astype(np.float32), dtype)


@pytest.mark.parametrize("dtype", [zi.FP32, zi.BF16, zi.FP16])
@pytest.mark.parametrize("m_half,d", [(5, 64), (33, 768), (64, 200), (7, 2048), (6, 2052), (4, 5120), (3, 12288), (9, 6000), (5, 12292)])
def test_layernorm(dtype, m_half, d):
    rng = np.random.Generator(np.random.PCG64(d))
    h = rng.standard_normal((2 * m_half, d)) * 3 + 0.5
    resid = torch.from_numpy(h).to(resid_dtype(dtype)).to(DEV)
    h_seen = resid.double().cpu().numpy()
    g = [_weights(rng, d, dtype, 0.3) for _ in range(2)]
    b = [_weights(rng, d, dtype, 0.3) for _ in range(2)]
    y = torch.empty((2 * m_half, d), dtype=act_dtype(dtype), device=DEV)
    zo_amd.zo_kernel_layernorm_pm(resid, to_dev(g[0], dtype), to_dev(g[1], dtype), to_dev(b[0], dtype), to_dev(b[1], dtype), y,
                                  dtype, m_half, d, 1e-5)
    want = np.concatenate([zo.layer_norm(h_seen[s * m_half:(s + 1) * m_half], zo.widen(g[s], dtype), zo.widen(b[s], dtype), 1e-5)
                           for s in range(2)])
    got = y.double().cpu().numpy()
    tol = 1e-10 if dtype == zi.FP32 else 1.5 * ULP[dtype]
    assert np.max(np.abs(got - want) / (np.abs(want) + 1.0)) < tol


@pytest.mark.parametrize("dtype", [zi.FP32, zi.BF16, zi.FP16])
@pytest.mark.parametrize("m_half,n,k", [(64, 128, 64), (130, 200, 192), (37, 72, 128), (256, 384, 320), (3, 8, 24),
                                        (2100, 2600, 128), (1024, 8200, 64),
                                        (2100, 2600, 192), (1024, 8200, 256), (1280, 3328, 192), (2100, 4104, 320)])
@pytest.mark.parametrize("epi", [0, 1, 2, 3])
def test_linear_pm(dtype, m_half, n, k, epi):
    """Shapes span several 128-wide tiles with ragged tails; (3, 8, 24) is below the MFMA tile depth.  The last
    four take the persistent 256 x 256 kernel (at least 128 tiles, k >= 192), ragged in both directions: 198 tiles
    on 200 workgroups (two find no tile), 264 tiles on 256 workgroups (some walk two tiles), 130 whole tiles, and
    306 tiles with five slabs each."""
    rng = np.random.Generator(np.random.PCG64(m_half * 7 + n + k + epi))
    x = rng.standard_normal((2 * m_half, k))
    xd = act_to_dev(x, dtype)
    x_seen = xd.double().cpu().numpy()
    w = [_weights(rng, (n, k), dtype) for _ in range(2)]          # already transposed: wt[n, k]
    bias = [_weights(rng, n, dtype, 0.5) for _ in range(2)]
    acc = np.concatenate([x_seen[s * m_half:(s + 1) * m_half] @ zo.widen(w[s], dtype).T for s in range(2)])
    with_bias = acc + np.concatenate([np.broadcast_to(zo.widen(bias[s], dtype), (m_half, n)) for s in range(2)])
    if epi in (0, 1):
        y = torch.zeros((2 * m_half, n), dtype=act_dtype(dtype), device=DEV)
        want = with_bias if epi == 0 else np.maximum(with_bias, 0)
    elif epi == 2:
        r0 = rng.standard_normal((2 * m_half, n))
        y = torch.from_numpy(r0).to(resid_dtype(dtype)).to(DEV)
        want = y.double().cpu().numpy() + with_bias
    else:
        y = torch.zeros((2 * m_half, n), dtype=resid_dtype(dtype), device=DEV)
        want = acc
    zo_amd.zo_kernel_linear_pm(xd, to_dev(w[0], dtype), to_dev(w[1], dtype), to_dev(bias[0], dtype), to_dev(bias[1], dtype), y,
                               dtype, m_half, n, k, epi)
    got = y.double().cpu().numpy()
    scale = np.sqrt(k) * 0.05 + 1.0           # size of a dot product of k such terms (+ bias / residual)
    if dtype == zi.FP32:
        bound = 4e-12 * scale
    elif epi in (0, 1):
        # one rounding of the output, half a unit in its own last place, + fp32 accumulation over k terms in tile order
        bound = ULP[dtype] * np.abs(want) + 2e-5 * scale
    else:
        bound = 4e-5 * scale                          # fp32 accumulation order only
    assert np.max(np.abs(got - want) / bound) < 1.0


@pytest.mark.parametrize("dtype", [zi.FP32, zi.BF16, zi.FP16])
@pytest.mark.parametrize("n_seq,seq,heads,dh", [(2, 32, 4, 16), (3, 70, 2, 64), (1, 200, 1, 128), (2, 130, 3, 32),
                                                (2, 300, 2, 64), (1, 257, 2, 128), (2, 512, 3, 64), (1, 1, 1, 64)])
def test_attention(dtype, n_seq, seq, heads, dh):
    rng = np.random.Generator(np.random.PCG64(seq * 3 + dh))
    d = heads * dh
    qkv = rng.standard_normal((n_seq, seq, 3 * d))
    qd = act_to_dev(qkv, dtype)
    seen = qd.double().cpu().numpy()
    out = torch.zeros((n_seq, seq, d), dtype=act_dtype(dtype), device=DEV)
    zo_amd.zo_kernel_attention(qd, out, dtype, n_seq, seq, heads, dh)
    want = zo.causal_attention(seen[..., :d], seen[..., d:2 * d], seen[..., 2 * d:], heads)
    got = out.double().cpu().numpy()
    tol = 1e-11 if dtype == zi.FP32 else 3 * ULP[dtype]      # probabilities and the output are each rounded once
    assert np.max(np.abs(got - want)) < tol * (1 + np.abs(want).max())


@pytest.mark.parametrize("dtype", [zi.FP32, zi.BF16, zi.FP16])
@pytest.mark.parametrize("m_half,d,vocab", [(6, 64, 512), (70, 128, 1000), (20, 64, 50272),
                                            (2100, 192, 4104), (1024, 768, 50272)])
def test_lmhead_ce(dtype, m_half, d, vocab):
    """The last two shapes take the persistent 256-wide kernel in the 2-byte types (at least 128 tiles, d >= 192): its
    per-row (max, sum-exp) slots, target-logit store, ragged vocabulary tail (4104 = 16 x 256 + 8, 50272 = 196 x 256 + 96)
    and ragged row tail (2100 = 8 x 256 + 52)."""
    rng = np.random.Generator(np.random.PCG64(vocab + d))
    x = rng.standard_normal((2 * m_half, d))
    xd = act_to_dev(x, dtype)
    seen = xd.double().cpu().numpy()
    e = [_weights(rng, (vocab, d), dtype, 0.1) for _ in range(2)]
    target = rng.integers(0, vocab, size=2 * m_half).astype(np.int32)
    target[::5] = -1
    target[1], target[2], target[m_half + 1] = vocab - 1, vocab - vocab % 256 if vocab % 256 else vocab - 256, (vocab - 1) // 256 * 256 - 1
    row_loss = torch.full((2 * m_half,), 7.0, dtype=torch.float64, device=DEV)
    scratch = torch.empty(zo_amd.zo_kernel_lmhead_scratch_bytes(dtype, m_half, vocab), dtype=torch.uint8, device=DEV)
    zo_amd.zo_kernel_lmhead_ce(xd, to_dev(e[0], dtype), to_dev(e[1], dtype), torch.from_numpy(target).to(DEV), row_loss, scratch,
                               dtype, m_half, d, vocab)
    got = row_loss.cpu().numpy()
    for s in range(2):
        logits = seen[s * m_half:(s + 1) * m_half] @ zo.widen(e[s], dtype).T
        mx = logits.max(-1)
        lse = np.log(np.exp(logits - mx[:, None]).sum(-1)) + mx
        tg = target[s * m_half:(s + 1) * m_half]
        want = np.where(tg >= 0, lse - logits[np.arange(m_half), np.maximum(tg, 0)], 0.0)
        tol = 1e-10 if dtype == zi.FP32 else 2e-4      # logits stay in fp32 (values up to ~10): accumulation order only
        assert np.max(np.abs(got[s * m_half:(s + 1) * m_half] - want)) < tol


def _tiny_model(**kw):
    c = zi.CONFIGS["tiny"]
    return Model(c["n_layers"], c["d_model"], c["n_heads"], c["d_ffn"], c["vocab"], c["max_pos"], c["dtype"], c["batch"], c["seq"],
                 **kw), c


def test_config1_fused_step_matches_oracle():
    """Config 1 as specified: weights N(0, 0.02) seed 0, LN gain 1 / bias 0, biases 0, 2 x 32 tokens,
    seed 42, eps 1e-3, lr 1e-5.  z bits exact; g and theta' within 1e-4 relative (measured: ~1e-9)."""
    mdl, c = _tiny_model(plain_small=True)
    tok, tok_dev = mdl.tokens()
    theta = [t.copy() for t in mdl.theta0]
    lp, lm, g = zo_amd.zo_step(mdl.handle, tok_dev, c["batch"], c["seq"], 42, c["eps"], c["lr"], zo_amd.ZO_MODE_FUSED)
    olp, olm, og = zo.zo_step_fused(mdl.ocfg, theta, tok, 42, c["eps"], c["lr"])
    assert abs(lp / olp - 1) < 1e-12 and abs(lm / olm - 1) < 1e-12
    assert abs(g / og - 1) < 1e-6, (g, og)
    got = mdl.theta()
    # theta' : the update scalar differs by |g - og| only; compare the applied deltas norm-wise and the values element-wise
    num = sum(float(np.sum((a.astype(np.float64) - b) ** 2)) for a, b in zip(got, theta))
    den = sum(float(np.sum((b.astype(np.float64) - t0) ** 2)) for b, t0 in zip(theta, mdl.theta0))
    assert den > 0 and np.sqrt(num / den) < 1e-4
    for a, b in zip(got, theta):
        assert np.all(np.abs(a.astype(np.float64) - b) <= 1e-4 * np.abs(b) + 1e-12)
    assert zo_amd.zo_device_flags(mdl.handle) == 0
    mdl.close()


def test_config1_update_bits_exact_given_the_oracles_scalar():
    mdl, c = _tiny_model(plain_small=False)
    s = zo.step_scalar(c["lr"], 3.1794912934978368)
    zo_amd.zo_perturb(mdl.handle, 42, float(s), 0, mdl.ocfg.n_tensors)
    want = [zo.axpy_z(t, mdl.dtype, 42, i, s) for i, t in enumerate(mdl.theta0)]
    assert all(a.tobytes() == b.tobytes() for a, b in zip(mdl.theta(), want))
    # a sub-range touches only its tensors
    zo_amd.zo_perturb(mdl.handle, 7, 1e-3, 3, 5)
    want = [zo.axpy_z(t, mdl.dtype, 7, i, 1e-3) if 3 <= i < 8 else t for i, t in enumerate(want)]
    assert all(a.tobytes() == b.tobytes() for a, b in zip(mdl.theta(), want))
    mdl.close()


def test_config1_literal_mode_matches_oracle_and_restores_theta():
    mdl, c = _tiny_model(plain_small=False)
    tok, tok_dev = mdl.tokens()
    theta = [t.copy() for t in mdl.theta0]
    lp, lm = zo_amd.zo_dual_forward(mdl.handle, tok_dev, c["batch"], c["seq"], 42, c["eps"], zo_amd.ZO_MODE_LITERAL)
    zo.perturb_all(mdl.ocfg, theta, 42, c["eps"])
    olp = zo.loss_of_storage(mdl.ocfg, theta, tok)
    zo.perturb_all(mdl.ocfg, theta, 42, -2.0 * np.float32(c["eps"]))
    olm = zo.loss_of_storage(mdl.ocfg, theta, tok)
    zo.perturb_all(mdl.ocfg, theta, 42, c["eps"])
    assert abs(lp / olp - 1) < 1e-12 and abs(lm / olm - 1) < 1e-12
    assert abs(((lp - lm) / (olp - olm)) - 1) < 1e-6
    assert all(a.tobytes() == b.tobytes() for a, b in zip(mdl.theta(), theta))       # same three roundings
    # and the whole literal step
    lp, lm, g = zo_amd.zo_step(mdl.handle, tok_dev, c["batch"], c["seq"], 43, c["eps"], c["lr"], zo_amd.ZO_MODE_LITERAL)
    olp, olm, og = zo.zo_step_literal(mdl.ocfg, theta, tok, 43, c["eps"], c["lr"])
    assert abs(g / og - 1) < 1e-6
    mdl.close()


def test_lr_zero_leaves_theta_bit_identical_and_seed_changes_g():
    mdl, c = _tiny_model(plain_small=True)
    tok, tok_dev = mdl.tokens()
    r1 = zo_amd.zo_step(mdl.handle, tok_dev, c["batch"], c["seq"], 42, c["eps"], 0.0)
    assert all(a.tobytes() == b.tobytes() for a, b in zip(mdl.theta(), mdl.theta0))
    r2 = zo_amd.zo_step(mdl.handle, tok_dev, c["batch"], c["seq"], 42, c["eps"], 0.0)
    assert r1 == r2                                             # same seed: same z, same losses, bit for bit
    r3 = zo_amd.zo_step(mdl.handle, tok_dev, c["batch"], c["seq"], 43, c["eps"], 0.0)
    assert r3[2] != r1[2]
    mdl.close()


def test_bad_token_poisons_the_loss_and_skips_the_update():
    mdl, c = _tiny_model(plain_small=True)
    tok, _ = mdl.tokens()
    tok[1, 5] = c["vocab"]
    lp, lm, g = zo_amd.zo_step(mdl.handle, torch.from_numpy(tok).to(DEV), c["batch"], c["seq"], 42, c["eps"], c["lr"])
    assert np.isnan(lp) and np.isnan(g)
    assert zo_amd.zo_device_flags(mdl.handle) == 3
    assert all(a.tobytes() == b.tobytes() for a, b in zip(mdl.theta(), mdl.theta0))
    mdl.close()


@pytest.mark.parametrize("dtype", [zi.BF16, zi.FP16])
def test_small_low_precision_model_matches_oracle(dtype):
    """A 2-layer, d = 128 model (MFMA tiles with ragged tails: 2 x 70 tokens, vocab 1000) in both 2-byte
    types.  The oracle reads the same rounded W+-; only activation rounding and summation order differ."""
    mdl = Model(2, 128, 4, 512, 1000, 128, dtype, 2, 70, plain_small=False, std=0.05)
    tok, tok_dev = mdl.tokens()
    lp, lm = zo_amd.zo_dual_forward(mdl.handle, tok_dev, 2, 70, 5, 1e-3)
    olp, olm = zo.dual_loss_fused(mdl.ocfg, mdl.theta0, tok, 5, 1e-3)
    tol = 2e-2 if dtype == zi.BF16 else 3e-3
    assert abs(lp / olp - 1) < tol and abs(lm / olm - 1) < tol
    assert all(a.tobytes() == b.tobytes() for a, b in zip(mdl.theta(), mdl.theta0))      # fused mode never writes theta
    mdl.close()


@pytest.mark.parametrize("dtype", [zi.FP32, zi.BF16])
def test_degenerate_shapes_match_oracle(dtype):
    """The smallest step there is: one block, one head, one sequence of two tokens (a single predicted token),
    then a call with fewer tokens than the model was set up for (batch 1 x seq 2 inside 3 x 9)."""
    for alloc, call in (((1, 2), (1, 2)), ((3, 9), (1, 2)), ((3, 9), (3, 9))):
        mdl = Model(1, 64, 1, 128, 96, 16, dtype, alloc[0], alloc[1], plain_small=False, std=0.05)
        tok, tok_dev = mdl.tokens(batch=call[0], seq=call[1])
        theta = [t.copy() for t in mdl.theta0]
        lp, lm, g = zo_amd.zo_step(mdl.handle, tok_dev, call[0], call[1], 11, 1e-3, 1e-4)
        olp, olm, og = zo.zo_step_fused(mdl.ocfg, theta, tok, 11, 1e-3, 1e-4)
        tol = 1e-10 if dtype == zi.FP32 else 2e-2
        assert abs(lp / olp - 1) < tol and abs(lm / olm - 1) < tol, (alloc, call, lp, olp)
        if dtype == zi.FP32:
            assert abs(g / og - 1) < 1e-5, (alloc, call, g, og)
        # the update is the kernel's own g times the oracle's z: bit-exact given that scalar
        want = [zo.axpy_z(t, mdl.dtype, 11, i, zo.step_scalar(1e-4, g)) for i, t in enumerate(mdl.theta0)]
        assert all(a.tobytes() == b.tobytes() for a, b in zip(mdl.theta(), want)), (alloc, call)
        assert zo_amd.zo_device_flags(mdl.handle) == 0
        mdl.close()

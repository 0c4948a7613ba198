"""Pins for the oracle's ZO-SGD step (oracle/zo_oracle.py): what Eq. 1-2 and
Alg. 1-2 of the paper fix -- same z in every pass, lr = 0 leaves theta alone,
g tends to the directional derivative z . grad L, g is even in eps, the
deferred order of Alg. 2 gives the same parameters as the immediate one."""
import numpy as np
import pytest

import zo_inputs as zi
from oracle import zo_oracle as zo


def _tiny():
    c = zi.CONFIGS["tiny"]
    cfg = zo.Config(c["n_layers"], c["d_model"], c["n_heads"], c["d_ffn"], c["vocab"], c["max_pos"], c["dtype"])
    theta = zi.make_weights(cfg.shapes(), cfg.dtype, seed=0)
    tokens = zi.make_tokens(c["batch"], c["seq"], c["vocab"], seed=1)
    return cfg, theta, tokens, c


def _micro(dtype=zo.FP32, seed=2):
    cfg = zo.Config(1, 16, 2, 32, 32, 8, dtype)
    theta = zi.make_weights(cfg.shapes(), dtype, seed=seed, std=0.3, plain_small=False)
    tokens = zi.make_tokens(2, 8, cfg.vocab, seed=3)
    return cfg, theta, tokens


def _flat_z(cfg, theta, seed):
    return np.concatenate([zo.z_values(seed, i, 0, t.size).astype(np.float64) for i, t in enumerate(theta)])


def test_lr_zero_leaves_theta_bit_identical():
    cfg, theta, tokens, c = _tiny()
    before = [t.copy() for t in theta]
    zo.zo_step_fused(cfg, theta, tokens, 42, c["eps"], 0.0)
    assert all(a.tobytes() == b.tobytes() for a, b in zip(theta, before))


def test_literal_and_fused_agree_and_use_one_z():
    cfg, theta, tokens, c = _tiny()
    a = [t.copy() for t in theta]
    b = [t.copy() for t in theta]
    lp1, lm1, g1 = zo.zo_step_literal(cfg, a, tokens, 42, c["eps"], c["lr"])
    lp2, lm2, g2 = zo.zo_step_fused(cfg, b, tokens, 42, c["eps"], c["lr"])
    assert abs(lp1 - lp2) < 1e-12 and abs(lm1 - lm2) < 1e-7      # second pass sees re-rounded weights
    assert abs(g1 / g2 - 1) < 1e-5
    # the update moved theta along the very z that perturbed it
    z = _flat_z(cfg, theta, 42)
    delta = np.concatenate([(y.astype(np.float64) - x.astype(np.float64)).ravel() for x, y in zip(theta, b)])
    s = float(zo.step_scalar(c["lr"], g2))
    mag = np.concatenate([np.maximum(np.abs(x), np.abs(y)).ravel() for x, y in zip(theta, b)])
    assert np.all(np.abs(delta - s * z) <= 0.51 * np.spacing(mag.astype(np.float32)))
    cos = delta @ z / np.linalg.norm(delta) / np.linalg.norm(z)
    assert abs(abs(cos) - 1) < 1e-4 and np.sign(delta @ z) == -np.sign(g2)


def test_g_is_the_directional_derivative_brute_force():
    """On a micro model, grad L by per-coordinate central differences in fp64;
    g(eps) -> z . grad L to 1e-3 relative as eps -> 0.  (At eps = 1e-3 this
    deliberately rough micro model, weights of size 0.3 and ReLU kinks within
    reach of eps |z|, is only within a few percent.)"""
    cfg, theta, tokens = _micro()
    w = [t.astype(np.float64) for t in theta]
    grad = []
    hstep = 1e-5
    for t in w:
        gt = np.zeros(t.size)
        flat = t.reshape(-1)
        for i in range(flat.size):
            keep = flat[i]
            flat[i] = keep + hstep; up = zo.loss(cfg, w, tokens)
            flat[i] = keep - hstep; dn = zo.loss(cfg, w, tokens)
            flat[i] = keep
            gt[i] = (up - dn) / (2 * hstep)
        grad.append(gt)
    grad = np.concatenate(grad)
    z = _flat_z(cfg, theta, 77)
    want = float(grad @ z)
    for eps, tol in ((1e-3, 5e-2), (1e-4, 1e-3), (3e-5, 1e-3)):
        lp, lm = zo.dual_loss_fused(cfg, theta, tokens, 77, eps)
        g = zo.projected_gradient(lp, lm, eps)
        assert abs(g / want - 1) < tol, (eps, g, want)


def test_g_against_autograd_on_the_tiny_config():
    torch = pytest.importorskip("torch")
    cfg, theta, tokens, c = _tiny()
    ws = [torch.tensor(t.astype(np.float64), requires_grad=True) for t in theta]
    F = torch.nn.functional
    tok = torch.from_numpy(tokens.astype(np.int64))
    S, d, H = tokens.shape[1], cfg.d_model, cfg.n_heads
    h = ws[0][tok] + ws[1][:S]
    for l in range(cfg.n_layers):
        p = dict(zip(zo.BLOCK_TENSORS, [ws[i] for i in cfg.block_ids(l)]))
        a = F.layer_norm(h, (d,), p["ln1_g"], p["ln1_b"], cfg.ln_eps)
        split = lambda x: x.view(-1, S, H, d // H).transpose(1, 2)
        q, k, v = split(a @ p["wq"].T + p["bq"]), split(a @ p["wk"].T + p["bk"]), split(a @ p["wv"].T + p["bv"])
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(-1, S, d)
        h = h + o @ p["wo"].T + p["bo"]
        f = F.layer_norm(h, (d,), p["ln2_g"], p["ln2_b"], cfg.ln_eps)
        h = h + torch.relu(f @ p["w1"].T + p["b1"]) @ p["w2"].T + p["b2"]
    g_id, b_id = cfg.head_ids()
    logits = F.layer_norm(h, (d,), ws[g_id], ws[b_id], cfg.ln_eps) @ ws[0].T
    loss = F.cross_entropy(logits[:, :-1].reshape(-1, cfg.vocab), tok[:, 1:].reshape(-1))
    assert abs(float(loss.detach()) - zo.loss_of_storage(cfg, theta, tokens)) < 1e-12
    loss.backward()
    grad = np.concatenate([w.grad.numpy().ravel() for w in ws])
    want = float(grad @ _flat_z(cfg, theta, 42))
    # (i) Eq. 1 in exact (fp64, unrounded) arithmetic tends to z . grad L
    w = [t.astype(np.float64) for t in theta]
    z = [zo.z_values(42, i, 0, t.size).astype(np.float64).reshape(t.shape) for i, t in enumerate(theta)]
    def g_exact(eps):
        lp = zo.loss(cfg, [a + eps * b for a, b in zip(w, z)], tokens)
        lm = zo.loss(cfg, [a - eps * b for a, b in zip(w, z)], tokens)
        return (lp - lm) / (2 * eps)
    # (the ReLU kinks of 32768 hidden units are dense around theta: the limit is only clean well below 1e-6)
    assert abs(g_exact(1e-8) / want - 1) < 1e-6
    # (ii) the oracle's step, which rounds theta +- eps z into fp32 storage, computes that same Eq. 1
    #      at the configured eps.  There the loss is far from linear along z (eps |z| reaches 0.37 against weights
    #      of size 0.02 and 32768 ReLU kinks lie in between: g(eps) for this z runs 0.26, 0.49, 0.69, 0.65, 0.56 at
    #      eps = 1e-3, 5e-4, 2.5e-4, 1e-4, 1e-5 towards the derivative 0.53), a property of the workload, not of
    #      the code: only sign and order of magnitude are asked of it
    lp, lm = zo.dual_loss_fused(cfg, theta, tokens, 42, c["eps"])
    g = zo.projected_gradient(lp, lm, c["eps"])
    assert abs(g / g_exact(float(np.float32(c["eps"]))) - 1) < 1e-5, (g, want)
    assert 1 / 3 < g / want < 3


def test_g_is_even_in_eps_and_converges_quadratically():
    cfg, theta, tokens = _micro()
    w = [t.astype(np.float64) for t in theta]
    shapes = [t.shape for t in theta]
    z = [zo.z_values(5, i, 0, t.size).astype(np.float64).reshape(s) for i, (t, s) in enumerate(zip(theta, shapes))]
    def g_of(eps):     # exact-arithmetic (fp64, no storage rounding) version of Eq. 1
        lp = zo.loss(cfg, [a + eps * b for a, b in zip(w, z)], tokens)
        lm = zo.loss(cfg, [a - eps * b for a, b in zip(w, z)], tokens)
        return (lp - lm) / (2 * eps)
    assert g_of(1e-3) == pytest.approx(g_of(-1e-3), rel=1e-13)
    # below the reach of the ReLU kinks the error is c eps^2: a tenfold smaller eps, a hundredfold smaller error
    g2, g3, g4 = g_of(1e-4), g_of(1e-5), g_of(1e-6)
    ratio = (g2 - g3) / (g3 - g4)
    assert 80 < ratio < 125, ratio
    # and the storage-rounded oracle step agrees with this exact-arithmetic g
    lp, lm = zo.dual_loss_fused(cfg, theta, tokens, 5, 1e-3)
    assert abs(zo.projected_gradient(lp, lm, 1e-3) / g_of(float(np.float32(1e-3))) - 1) < 1e-4


@pytest.mark.parametrize("dtype", [zo.FP32, zo.BF16])
@pytest.mark.parametrize("literal", [False, True])
def test_alg2_deferred_update_equals_immediate(dtype, literal):
    cfg, theta, tokens = _micro(dtype)
    eps, lr = 1e-3, (1e-2 if dtype == zo.FP32 else 1e-1)
    imm = [t.copy() for t in theta]
    dfr = [t.copy() for t in theta]
    runner = zo.Alg2Runner(cfg, dfr, eps, lr, literal=literal)
    step = zo.zo_step_literal if literal else zo.zo_step_fused
    # Fused: nothing but the update ever writes theta, so the two orders are the same operations per
    # element and must agree bit for bit.  Literal: Alg. 2 restores the tied embedding through a
    # +eps/-2eps/+eps cycle before the LM head perturbs it again, Alg. 1 does not, so the two differ
    # by the few ulps those roundings leave (and g, a difference of near-equal losses, by more).
    tol = dict(rel=1e-12, abs=0) if not literal else dict(rel=(1e-6 if dtype == zo.FP32 else 5e-2), abs=0)
    for seed in (0, 1, 2):
        a = step(cfg, imm, tokens, seed, eps, lr)
        b = runner.step(tokens, seed)
        assert a[:2] == pytest.approx(b[:2], **tol)
        if not literal:
            assert a[2] == pytest.approx(b[2], **tol)
    assert any(x.tobytes() != y.tobytes() for x, y in zip(imm, dfr))     # last update still pending
    runner.flush()
    if not literal:
        assert all(x.tobytes() == y.tobytes() for x, y in zip(imm, dfr))
    elif dtype == zo.FP32:
        for x, y in zip(imm, dfr):
            assert np.all(np.abs(x.astype(np.float64) - y) <= 1e-4 * (np.abs(x) + 1e-2))
    assert any(x.tobytes() != y.tobytes() for x, y in zip(imm, theta))   # and the steps did move theta


def test_bf16_updates_mostly_vanish_at_paper_learning_rates():
    """lr |g z| is far below half an ulp of a bf16 weight of size 0.02: with plain
    nearest-even rounding and no master copy almost every element is unchanged."""
    cfg = zo.Config(1, 32, 2, 64, 64, 8, zo.BF16)
    theta = zi.make_weights(cfg.shapes(), zo.BF16, seed=0)
    tokens = zi.make_tokens(2, 8, cfg.vocab)
    before = [t.copy() for t in theta]
    zo.zo_step_fused(cfg, theta, tokens, 0, 1e-3, 1e-6)
    # (zero-initialised biases do move: any s*z is representable next to 0)
    big = [np.abs(zo.widen(b, zo.BF16)) > 0.01 for b in before]
    changed = sum(int(((a != b) & m).sum()) for a, b, m in zip(theta, before, big) if a.ndim == 2)
    total = sum(int(m.sum()) for t, m in zip(theta, big) if t.ndim == 2)
    assert total > 1000 and changed / total < 1e-3

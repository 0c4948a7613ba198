"""GPU parity at the full sizes bench.py times (OPT-13B shapes, batch 4 x seq 2048, bf16), in the same
launch configuration, on sampled outputs the oracle computes one by one.  Inputs are drawn on the device
by torch's generator (a seeded library generator, not the HIP path) and the sampled rows / columns are
copied back for the oracle."""
import numpy as np
import pytest
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from oracle import zo_oracle as zo
from gpu_util import DEV, to_host

pytestmark = pytest.mark.gpu

D, F, H, DH, V = 5120, 20480, 40, 128, 50272
M_HALF = 4 * 2048
BF = zi.BF16


def _gen(seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return g


def _wide(t):
    """bf16 device tensor (any shape) -> fp64 numpy."""
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("n,k,epi", [(3 * D, D, 0), (F, D, 1), (D, F, 2), (D, D, 2)])
def test_linear_at_13b_shapes_sampled(n, k, epi):
    g = _gen(n + k + epi)
    x = torch.randn(2 * M_HALF, k, device=DEV, generator=g).to(torch.bfloat16)
    w = [(0.02 * torch.randn(n, k, device=DEV, generator=g)).to(torch.bfloat16) for _ in range(2)]
    b = [(0.1 * torch.randn(n, device=DEV, generator=g)).to(torch.bfloat16) for _ in range(2)]
    if epi == 2:
        y = torch.randn(2 * M_HALF, n, device=DEV, generator=g)
        y0 = y.clone()
    else:
        y = torch.zeros(2 * M_HALF, n, device=DEV, dtype=torch.bfloat16)
    zo_amd.zo_kernel_linear_pm(x, w[0], w[1], b[0], b[1], y, BF, M_HALF, n, k, epi)
    rng = np.random.Generator(np.random.PCG64(5))
    rows = np.concatenate([rng.integers(0, 2 * M_HALF, 24), [0, M_HALF - 1, M_HALF, 2 * M_HALF - 1]])
    cols = np.concatenate([rng.integers(0, n, 24), [0, n - 1, 255, 256]])
    for r in rows:
        s = int(r >= M_HALF)
        xr = _wide(x[int(r)])
        want = _wide(w[s][cols]) @ xr + _wide(b[s][cols])
        if epi == 1:
            want = np.maximum(want, 0)
        if epi == 2:
            want = want + y0[int(r)][cols].double().cpu().numpy()
        got = y[int(r)][cols].double().cpu().numpy()
        scale = np.sqrt(k) * 0.02 + 1.0
        # bf16 outputs: one rounding (half a unit in the output's own last place) + fp32 accumulation order; fp32 outputs: the latter
        bound = (2.0**-8 * np.abs(want) if epi != 2 else 0.0) + 4e-5 * scale
        assert np.max(np.abs(got - want) / bound) < 1.0, (r, np.max(np.abs(got - want) / bound))


def test_attention_at_13b_shape_sampled_heads():
    n_seq, seq = 8, 2048
    g = _gen(11)
    qkv = torch.randn(n_seq * seq, 3 * D, device=DEV, generator=g).to(torch.bfloat16)
    out = torch.zeros(n_seq * seq, D, device=DEV, dtype=torch.bfloat16)
    zo_amd.zo_kernel_attention(qkv, out, BF, n_seq, seq, H, DH)
    for sq, head in [(0, 0), (3, 17), (7, 39)]:
        blk = qkv[sq * seq:(sq + 1) * seq]
        q, k, v = (_wide(blk[:, o * D + head * DH:o * D + (head + 1) * DH])[None] for o in range(3))
        want = zo.causal_attention(q, k, v, 1)[0]
        got = _wide(out[sq * seq:(sq + 1) * seq, head * DH:(head + 1) * DH])
        assert np.max(np.abs(got - want)) < 3 * 2.0**-8 * (1 + np.abs(want).max())


@pytest.mark.parametrize("seq", [8192, 4100])
def test_attention_long_context_sampled_heads(seq):
    """The longer-context variants (8192 tokens; 4100 leaves a ragged last key tile and query block): whole heads
    against the oracle, which costs it O(S^2 d) per head only."""
    n_seq, heads = 2, 4
    d = heads * DH
    g = _gen(13 + seq)
    qkv = torch.randn(n_seq * seq, 3 * d, device=DEV, generator=g).to(torch.bfloat16)
    out = torch.zeros(n_seq * seq, d, device=DEV, dtype=torch.bfloat16)
    zo_amd.zo_kernel_attention(qkv, out, BF, n_seq, seq, heads, DH)
    for sq, head in [(0, 0), (1, 3)]:
        blk = qkv[sq * seq:(sq + 1) * seq]
        q, k, v = (_wide(blk[:, o * d + head * DH:o * d + (head + 1) * DH])[None] for o in range(3))
        want = zo.causal_attention(q, k, v, 1)[0]
        got = _wide(out[sq * seq:(sq + 1) * seq, head * DH:(head + 1) * DH])
        assert np.max(np.abs(got - want)) < 3 * 2.0**-8 * (1 + np.abs(want).max())


@pytest.mark.parametrize("n_seq,seq,heads,dh", [(2, 1024, 40, 128), (2, 1100, 48, 64), (3, 300, 5, 128)])
def test_attention_work_list_covers_every_item(n_seq, seq, heads, dh):
    """More (query tile, head, sequence) items than resident workgroups: several rounds over the per-XCD item list,
    a last group of fewer pairs, and a pair count that does not fill the 8 XCDs evenly.  Every output row must have
    been written (they start as NaN), the first row of every head is v[0] itself (one key, probability 1), and
    sampled heads, the last pair among them, are compared with the oracle."""
    d = heads * dh
    g = _gen(17 + seq)
    qkv = torch.randn(n_seq * seq, 3 * d, device=DEV, generator=g).to(torch.bfloat16)
    out = torch.full((n_seq * seq, d), float("nan"), device=DEV, dtype=torch.bfloat16)
    zo_amd.zo_kernel_attention(qkv, out, BF, n_seq, seq, heads, dh)
    assert not bool(torch.isnan(out).any())
    first = out.view(n_seq, seq, d)[:, 0]
    assert bool((first == qkv.view(n_seq, seq, 3 * d)[:, 0, 2 * d:]).all())
    for sq, head in [(0, 0), (n_seq // 2, heads // 2), (n_seq - 1, heads - 1)]:
        blk = qkv[sq * seq:(sq + 1) * seq]
        q, k, v = (_wide(blk[:, o * d + head * dh:o * d + (head + 1) * dh])[None] for o in range(3))
        want = zo.causal_attention(q, k, v, 1)[0]
        got = _wide(out[sq * seq:(sq + 1) * seq, head * dh:(head + 1) * dh])
        assert np.max(np.abs(got - want)) < 3 * 2.0**-8 * (1 + np.abs(want).max())


def test_layernorm_and_update_streams_at_13b_sizes_sampled():
    g = _gen(12)
    h = torch.randn(2 * M_HALF, D, device=DEV, generator=g) * 2 + 0.3
    gam = [(1 + 0.1 * torch.randn(D, device=DEV, generator=g)).to(torch.bfloat16) for _ in range(2)]
    bet = [(0.1 * torch.randn(D, device=DEV, generator=g)).to(torch.bfloat16) for _ in range(2)]
    y = torch.empty(2 * M_HALF, D, device=DEV, dtype=torch.bfloat16)
    zo_amd.zo_kernel_layernorm_pm(h, gam[0], gam[1], bet[0], bet[1], y, BF, M_HALF, D, 1e-5)
    for r in (0, 4097, M_HALF - 1, M_HALF, 2 * M_HALF - 1):
        s = int(r >= M_HALF)
        want = zo.layer_norm(h[r].double().cpu().numpy(), _wide(gam[s]), _wide(bet[s]), 1e-5)
        assert np.max(np.abs(_wide(y[r]) - want) / (np.abs(want) + 1)) < 1.5 * 2.0**-8
    # one FFN matrix of a 13B block through the in-place stream and through staging: sampled elements, bit-exact
    n = D * F
    theta = (0.02 * torch.randn(n, device=DEV, generator=g)).to(torch.bfloat16)
    keep = theta.clone()
    zo_amd.zo_kernel_axpy_z(theta, theta, BF, n, 2**40 + 3, 654, -2e-3)
    wp, wm = torch.empty_like(theta), torch.empty_like(theta)
    zo_amd.zo_kernel_stage_pm(keep, wp, wm, BF, D, F, 1, 99, 654, 1e-3)
    rng = np.random.Generator(np.random.PCG64(6))
    idx = np.unique(np.concatenate([rng.integers(0, n, 4000), [0, 1, 2, 3, n - 4, n - 1, 4095, 4096]]))
    src = to_host(keep[torch.from_numpy(idx).to(DEV)], BF)
    got = to_host(theta[torch.from_numpy(idx).to(DEV)], BF)
    tr = (idx % F) * D + idx // F                               # where element (r, c) lands after transposition
    got_p = to_host(wp[torch.from_numpy(tr).to(DEV)], BF)
    got_m = to_host(wm[torch.from_numpy(tr).to(DEV)], BF)
    for j, i in enumerate(idx):
        one = src[j:j + 1]
        assert zo.axpy_z(one, BF, 2**40 + 3, 654, -2e-3, first=int(i))[0] == got[j]
        assert zo.axpy_z(one, BF, 99, 654, 1e-3, first=int(i))[0] == got_p[j]
        assert zo.axpy_z(one, BF, 99, 654, -np.float32(1e-3), first=int(i))[0] == got_m[j]


def test_step_invariants_at_opt_1_3b_size():
    """A whole OPT-1.3B-shaped model (the oracle cannot run it): the step is a deterministic function of
    (theta, tokens, seed); lr = 0 leaves every parameter bit for bit; a step with lr > 0 moves theta and changes
    the next step's losses; losses sit near ln V for the synthetic initialisation."""
    c = dict(zi.CONFIGS["opt-1.3b"])
    shapes = zi.tensor_shapes(c["n_layers"], c["d_model"], c["d_ffn"], c["vocab"], c["max_pos"])
    g = _gen(21)
    tensors = []
    for name, shape in shapes:
        leaf = name.split(".")[-1]
        if len(shape) == 2:
            tensors.append((0.02 * torch.randn(shape, device=DEV, generator=g)).to(torch.bfloat16))
        elif leaf.endswith("_g"):
            tensors.append(torch.ones(shape, device=DEV, dtype=torch.bfloat16))
        else:
            tensors.append(torch.zeros(shape, device=DEV, dtype=torch.bfloat16))
    batch, seq = 2, 1024
    tokens = torch.randint(0, c["vocab"], (batch, seq), dtype=torch.int32, device=DEV, generator=g)
    cfg = zo_amd.make_config(c["n_layers"], c["d_model"], c["n_heads"], c["d_ffn"], c["vocab"], c["max_pos"], BF)
    nbytes = zo_amd.zo_workspace_bytes(cfg, batch, seq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    stream = torch.cuda.Stream(device=DEV)
    torch.cuda.synchronize()
    h = zo_amd.zo_init_model(cfg, tensors, ws, nbytes, batch, seq, stream, None)
    before = [t.clone() for t in tensors]
    a = zo_amd.zo_step(h, tokens, batch, seq, 5, 1e-3, 0.0)
    b = zo_amd.zo_step(h, tokens, batch, seq, 5, 1e-3, 0.0)
    assert a == b                                                       # same seed, same theta: same bits
    assert all(torch.equal(x.view(torch.int16), y.view(torch.int16)) for x, y in zip(tensors, before))   # lr = 0
    assert abs(a[0] / np.log(c["vocab"]) - 1) < 0.1 and abs(a[1] / np.log(c["vocab"]) - 1) < 0.1
    other = zo_amd.zo_step(h, tokens, batch, seq, 6, 1e-3, 0.0)
    assert other[2] != a[2]                                             # another direction, another g
    zo_amd.zo_step(h, tokens, batch, seq, 5, 1e-3, 1e-2)                # a large step so that bf16 weights do move
    assert any(not torch.equal(x.view(torch.int16), y.view(torch.int16)) for x, y in zip(tensors, before))
    after = zo_amd.zo_step(h, tokens, batch, seq, 5, 1e-3, 0.0)
    assert after != a
    assert zo_amd.zo_device_flags(h) == 0
    zo_amd.zo_free(h)

"""GPU parity at the real shapes of the configurations that the oracle cannot run whole: one OPT-175B block
(fp16, d 12288, 96 heads of 128, FFN 49152, 2 x 2048 rows) and the OPT-1.3B shapes (bf16, d 2048, 32 heads of 64,
FFN 8192, 8 sequences of 1024), plus the LM head with the cross entropy fused at d 12288 / 5120 / 2048 and vocab 50272.
Every kernel runs in the launch configuration the step uses at that shape; outputs are compared with the oracle on
sampled rows and columns (or whole heads), which it computes one by one from the same inputs.  Inputs are drawn on
the device by torch's generator (a seeded library generator, not the HIP path)."""
import numpy as np
import pytest
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from oracle import zo_oracle as zo
from gpu_util import DEV, to_host

pytestmark = pytest.mark.gpu

V = 50272
TDT = {zi.BF16: torch.bfloat16, zi.FP16: torch.float16}
ULP = {zi.BF16: 2.0**-8, zi.FP16: 2.0**-11}

# name: (dtype, d, heads, d_head, ffn, m_half = batch x seq of the configuration, n_seq per sign, seq)
SHAPES = {"opt-175b": (zi.FP16, 12288, 96, 128, 49152, 2048, 1, 2048),
          "opt-1.3b": (zi.BF16, 2048, 32, 64, 8192, 8192, 8, 1024)}


def _gen(seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return g


def _wide(t):
    return t.float().cpu().numpy().astype(np.float64)


def _linear_cases():
    out = []
    for name, (dt, d, h, dh, f, m_half, _, _) in SHAPES.items():
        out += [(name, 3 * d, d, 0), (name, d, d, 2), (name, f, d, 1), (name, d, f, 2)]
    return out


@pytest.mark.parametrize("name,n,k,epi", _linear_cases())
def test_linear_at_real_shapes_sampled(name, n, k, epi):
    dt, _, _, _, _, m_half, _, _ = SHAPES[name]
    tdt = TDT[dt]
    g = _gen(n + k + epi)
    x = torch.randn(2 * m_half, k, device=DEV, generator=g).to(tdt)
    w = [(0.02 * torch.randn(n, k, device=DEV, generator=g)).to(tdt) for _ in range(2)]
    b = [(0.1 * torch.randn(n, device=DEV, generator=g)).to(tdt) for _ in range(2)]
    if epi == 2:
        y = torch.randn(2 * m_half, n, device=DEV, generator=g)
        y0 = y.clone()
    else:
        y = torch.zeros(2 * m_half, n, device=DEV, dtype=tdt)
    zo_amd.zo_kernel_linear_pm(x, w[0], w[1], b[0], b[1], y, dt, m_half, n, k, epi)
    rng = np.random.Generator(np.random.PCG64(5))
    rows = np.concatenate([rng.integers(0, 2 * m_half, 20), [0, m_half - 1, m_half, 2 * m_half - 1, 255, 256]])
    cols = np.concatenate([rng.integers(0, n, 24), [0, n - 1, 255, 256, n - 256, n - 257]])
    scale = np.sqrt(k) * 0.02 + 1.0                  # size of a dot product of k such terms (+ bias / residual)
    # 2-byte outputs: one rounding of the result (half a unit in its own last place) on top of the fp32 accumulation
    # over k terms in tile order; fp32 outputs (the residual stream): the accumulation order alone
    worst = 0.0
    for r in rows:
        s = int(r >= m_half)
        want = _wide(w[s][cols]) @ _wide(x[int(r)]) + _wide(b[s][cols])
        if epi == 1:
            want = np.maximum(want, 0)
        if epi == 2:
            want = want + y0[int(r)][cols].double().cpu().numpy()
        got = y[int(r)][cols].double().cpu().numpy()
        bound = (ULP[dt] * np.abs(want) if epi != 2 else 0.0) + 4e-5 * scale
        worst = max(worst, float(np.max(np.abs(got - want) / bound)))
    assert worst < 1.0, (name, n, k, epi, worst)


@pytest.mark.parametrize("name", list(SHAPES))
def test_attention_at_real_shapes_sampled_heads(name):
    dt, d, heads, dh, _, _, n_seq_half, seq = SHAPES[name]
    n_seq = 2 * n_seq_half
    g = _gen(31 + d)
    qkv = torch.randn(n_seq * seq, 3 * d, device=DEV, generator=g).to(TDT[dt])
    out = torch.full((n_seq * seq, d), float("nan"), device=DEV, dtype=TDT[dt])
    zo_amd.zo_kernel_attention(qkv, out, dt, n_seq, seq, heads, dh)
    assert not bool(torch.isnan(out).any())
    for sq, head in [(0, 0), (n_seq // 2, heads // 3), (n_seq - 1, heads - 1)]:
        blk = qkv[sq * seq:(sq + 1) * seq]
        q, k, v = (_wide(blk[:, o * d + head * dh:o * d + (head + 1) * dh])[None] for o in range(3))
        want = zo.causal_attention(q, k, v, 1)[0]
        got = _wide(out[sq * seq:(sq + 1) * seq, head * dh:(head + 1) * dh])
        assert np.max(np.abs(got - want)) < 3 * ULP[dt] * (1 + np.abs(want).max()), (name, sq, head)


@pytest.mark.parametrize("dtype", [zi.BF16, zi.FP16, zi.FP32])
@pytest.mark.parametrize("n_seq,seq,heads,dh", [(2, 2048, 3, 128), (2, 1100, 4, 64), (1, 4100, 2, 128), (3, 257, 2, 64), (1, 70, 2, 32)])
def test_attention_weighs_every_key_once(dtype, n_seq, seq, heads, dh):
    """With q = 0 every causal probability of query t is 1 / (t + 1), and with unit-vector values, v[key] = e_(key mod
    d_head), output element j of query t is (number of keys <= t with key mod d_head = j) / (t + 1): each key's weight
    can be read off one output element, so a key that is dropped, doubled or given to the wrong query fails at any row
    length (a random-data comparison at 3 ulp of bf16 would let a single key among hundreds pass)."""
    d = heads * dh
    tdt = {zi.BF16: torch.bfloat16, zi.FP16: torch.float16, zi.FP32: torch.float64}[dtype]
    g = _gen(7 + seq)
    qkv = torch.zeros(n_seq, seq, 3 * d, device=DEV, dtype=tdt)
    qkv[..., d:2 * d] = torch.randn(n_seq, seq, d, device=DEV, generator=g).to(tdt)       # keys: anything
    key = torch.arange(seq, device=DEV)
    onehot = torch.nn.functional.one_hot(key % dh, dh).to(tdt)                             # [seq, dh]
    qkv[..., 2 * d:] = onehot.repeat(1, heads)[None]
    out = torch.full((n_seq, seq, d), float("nan"), device=DEV, dtype=tdt)
    zo_amd.zo_kernel_attention(qkv, out, dtype, n_seq, seq, heads, dh)
    t = np.arange(seq)[:, None]
    j = np.arange(dh)[None, :]
    count = (t >= j) * ((t - j) // dh + 1)                                                 # keys j, j + dh, ... <= t
    want = count / (t + 1.0)
    got = out.double().cpu().numpy().reshape(n_seq, seq, heads, dh)
    # one rounding of the output (the probabilities 1 and the counts are exact in every type)
    tol = 1e-12 if dtype == zi.FP32 else ULP[dtype]
    err = np.abs(got - want[None, :, None, :])
    assert np.all(err <= tol * want[None, :, None, :] + 1e-30), (np.unravel_index(err.argmax(), err.shape), err.max())
    # what a single lost or doubled key would change is 1 / (t + 1) of one element; the tolerance there is
    # tol * count / (t + 1), a small fraction of it at every length
    assert tol * count.max() < 0.5


@pytest.mark.parametrize("name,d,m_half,dtype", [("opt-175b", 12288, 2048, zi.FP16), ("opt-13b", 5120, 8192, zi.BF16),
                                                 ("opt-1.3b", 2048, 8192, zi.BF16)])
def test_lmhead_ce_at_real_shapes_sampled_rows(name, d, m_half, dtype):
    """The persistent 256-wide kernel's fused cross-entropy epilogue at the real head shapes: ragged vocabulary tail
    (50272 = 196 x 256 + 96), targets in the last partial tile, rows that do not count."""
    tdt = TDT[dtype]
    g = _gen(3 + d)
    x = torch.randn(2 * m_half, d, device=DEV, generator=g).to(tdt)
    e = [(0.02 * torch.randn(V, d, device=DEV, generator=g)).to(tdt) for _ in range(2)]
    target = torch.randint(0, V, (2 * m_half,), device=DEV, generator=g, dtype=torch.int32)
    target[::9] = -1
    target[1] = V - 1
    target[2] = V - 96                      # first column of the last, partial tile
    target[m_half + 3] = 196 * 256 - 1      # last column of the last whole tile
    row_loss = torch.full((2 * m_half,), 7.0, dtype=torch.float64, device=DEV)
    scratch = torch.empty(zo_amd.zo_kernel_lmhead_scratch_bytes(dtype, m_half, V), dtype=torch.uint8, device=DEV)
    zo_amd.zo_kernel_lmhead_ce(x, e[0], e[1], target, row_loss, scratch, dtype, m_half, d, V)
    got = row_loss.cpu().numpy()
    tg = target.cpu().numpy()
    assert np.all(got[tg < 0] == 0.0) and np.all(np.isfinite(got))
    rng = np.random.Generator(np.random.PCG64(8))
    rows = np.unique(np.concatenate([rng.integers(0, 2 * m_half, 24), [0, 1, 2, m_half - 1, m_half, m_half + 3, 2 * m_half - 1]]))
    for r in rows:
        s = int(r >= m_half)
        logits = (e[s].double() @ x[int(r)].double()).cpu().numpy()         # torch fp64 matmul on the same values: a library routine
        mx = logits.max()
        want = 0.0 if tg[r] < 0 else float(np.log(np.exp(logits - mx).sum()) + mx - logits[tg[r]])     # logsumexp - target logit
        assert abs(got[r] - want) < 2e-4, (name, r, got[r], want)


@pytest.mark.parametrize("name", list(SHAPES))
def test_stage_and_update_streams_at_real_block_shapes_sampled(name):
    """The FFN matrices of a block through the transposing staging pass (both orientations: d x F and F x d) and the
    in-place stream: sampled elements, bit-exact against the oracle's rn(fma(c, z, theta))."""
    dt, d, _, _, f, _, _, _ = SHAPES[name]
    tdt = TDT[dt]
    g = _gen(12 + d)
    n = d * f
    theta = (0.02 * torch.randn(n, device=DEV, generator=g)).to(tdt)
    keep = theta.clone()
    zo_amd.zo_kernel_axpy_z(theta, theta, dt, n, 2**41 + 5, 1203, -2e-3)
    rng = np.random.Generator(np.random.PCG64(6))
    idx = np.unique(np.concatenate([rng.integers(0, n, 3000), [0, 1, 2, 3, n - 4, n - 1, 8191, 8192, 8193]]))
    sel = torch.from_numpy(idx).to(DEV)
    src = to_host(keep[sel], dt)
    got = to_host(theta[sel], dt)
    for j, i in enumerate(idx):
        assert zo.axpy_z(src[j:j + 1], dt, 2**41 + 5, 1203, -2e-3, first=int(i))[0] == got[j], (name, i)
    for rows, cols in ((d, f), (f, d)):
        wp, wm = torch.empty_like(keep), torch.empty_like(keep)
        zo_amd.zo_kernel_stage_pm(keep, wp, wm, dt, rows, cols, 1, 99, 1207, 1e-3)
        tr = (idx % cols) * rows + idx // cols                  # where element (r, c) lands after transposition
        trs = torch.from_numpy(tr).to(DEV)
        got_p, got_m = to_host(wp[trs], dt), to_host(wm[trs], dt)
        for j, i in enumerate(idx):
            one = src[j:j + 1]
            assert zo.axpy_z(one, dt, 99, 1207, 1e-3, first=int(i))[0] == got_p[j], (name, rows, cols, i)
            assert zo.axpy_z(one, dt, 99, 1207, -np.float32(1e-3), first=int(i))[0] == got_m[j], (name, rows, cols, i)


@pytest.mark.parametrize("name", list(SHAPES))
def test_layernorm_at_real_shapes_sampled(name):
    dt, d, _, _, _, m_half, _, _ = SHAPES[name]
    tdt = TDT[dt]
    g = _gen(40 + d)
    h = torch.randn(2 * m_half, d, device=DEV, generator=g) * 2 + 0.3
    gam = [(1 + 0.1 * torch.randn(d, device=DEV, generator=g)).to(tdt) for _ in range(2)]
    bet = [(0.1 * torch.randn(d, device=DEV, generator=g)).to(tdt) for _ in range(2)]
    y = torch.empty(2 * m_half, d, device=DEV, dtype=tdt)
    zo_amd.zo_kernel_layernorm_pm(h, gam[0], gam[1], bet[0], bet[1], y, dt, m_half, d, 1e-5)
    for r in (0, m_half // 2 + 1, m_half - 1, m_half, 2 * m_half - 1):
        s = int(r >= m_half)
        want = zo.layer_norm(h[r].double().cpu().numpy(), _wide(gam[s]), _wide(bet[s]), 1e-5)
        assert np.max(np.abs(_wide(y[r]) - want) / (np.abs(want) + 1)) < 1.5 * ULP[dt]

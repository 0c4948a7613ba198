"""The LM-head entry point that allocates nothing (its partial results live in a buffer inside the library)
against the entry point that takes the caller's scratch buffer: same kernels, so the same bits, on two calls in a
row, the second one smaller (the shared buffer still holds the first call's partials), in the tilings the head uses
(128-wide tiles, the persistent 256-wide kernel, the fp32 configuration's logits chunk) and against the oracle."""
import numpy as np
import pytest
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from oracle import zo_oracle as zo
from gpu_util import DEV, act_to_dev, to_dev

pytestmark = pytest.mark.gpu


def _case(dtype, m_half, d, vocab, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    x = act_to_dev(rng.standard_normal((2 * m_half, d)), dtype)
    e = [zi.round_to_storage((0.1 * rng.standard_normal((vocab, d))).astype(np.float32), dtype) for _ in range(2)]
    target = rng.integers(0, vocab, size=2 * m_half).astype(np.int32)
    target[::7] = -1
    return x, e, target


def _both(dtype, m_half, d, vocab, seed):
    x, e, target = _case(dtype, m_half, d, vocab, seed)
    ed = [to_dev(w, dtype) for w in e]
    td = torch.from_numpy(target).to(DEV)
    want = torch.full((2 * m_half,), 7.0, dtype=torch.float64, device=DEV)
    scratch = torch.empty(zo_amd.zo_kernel_lmhead_scratch_bytes(dtype, m_half, vocab), dtype=torch.uint8, device=DEV)
    zo_amd.zo_kernel_lmhead_ce(x, ed[0], ed[1], td, want, scratch, dtype, m_half, d, vocab)
    got = torch.full((2 * m_half,), -3.0, dtype=torch.float64, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    zo_amd.zo_kernel_lmhead_ce_noalloc(x, ed[0], ed[1], td, got, dtype, m_half, d, vocab)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return x, e, target, want.cpu().numpy(), got.cpu().numpy()


def _oracle_rows(x, e, target, dtype, m_half, rows):
    seen = x.double().cpu().numpy()
    out = {}
    for r in rows:
        s = int(r >= m_half)
        logits = zo.widen(e[s], dtype) @ seen[r]
        mx = logits.max()
        out[r] = 0.0 if target[r] < 0 else float(np.log(np.exp(logits - mx).sum()) + mx - logits[target[r]])
    return out


@pytest.mark.parametrize("dtype,first,second", [
    (zi.BF16, (70, 128, 1000), (20, 64, 512)),               # 128-wide tiles
    (zi.FP16, (1100, 192, 4104), (600, 256, 4104)),           # persistent 256-wide kernel, ragged vocabulary tail; then the small tiling
    (zi.FP32, (100, 64, 50272), (6, 64, 512)),                # fp64 logits in row chunks cut to the buffer (83 + 17 rows)
])
def test_no_alloc_lmhead_matches_the_scratch_argument_form_twice_in_a_row(dtype, first, second):
    for i, (m_half, d, vocab) in enumerate((first, second)):
        x, e, target, want, got = _both(dtype, m_half, d, vocab, seed=31 + i)
        assert got.tobytes() == want.tobytes(), (dtype, m_half, d, vocab)       # the same kernels on the same inputs
        rows = [0, 1, m_half - 1, m_half, 2 * m_half - 1, 7, 2 * m_half - 7]
        ref = _oracle_rows(x, e, target, dtype, m_half, rows)
        tol = 1e-10 if dtype == zi.FP32 else 2e-4
        for r in rows:
            assert abs(got[r] - ref[r]) < tol, (r, got[r], ref[r])


def test_no_alloc_lmhead_rejects_sizes_beyond_its_buffer():
    m_half, d, vocab = 2700, 64, 50272
    assert 2 * m_half * (2 * ((vocab + 127) // 128) * 8 + 4) > zo_amd.ZO_NOALLOC_SCRATCH_BYTES
    x = torch.zeros((2 * m_half, d), dtype=torch.bfloat16, device=DEV)
    e = torch.zeros((vocab, d), dtype=torch.bfloat16, device=DEV)
    t = torch.zeros(2 * m_half, dtype=torch.int32, device=DEV)
    out = torch.full((2 * m_half,), 5.0, dtype=torch.float64, device=DEV)
    with pytest.raises(zo_amd.ZoError) as err:
        zo_amd.zo_kernel_lmhead_ce_noalloc(x, e, e, t, out, zi.BF16, m_half, d, vocab)
    assert err.value.status == zo_amd.ZO_ENOMEM and "zo_kernel_lmhead_ce" in str(err.value)
    torch.cuda.synchronize()
    assert bool((out == 5.0).all())                                               # nothing was enqueued

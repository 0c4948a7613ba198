"""GPU parity, part 3: the block-streamed model (Alg. 2's deferred update under Alg. 3's upload /
compute / offload overlap) must give exactly what the resident model gives, and what the oracle's
Alg. 2 runner gives."""
import numpy as np
import pytest
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from oracle import zo_oracle as zo
from gpu_util import DEV, Model

pytestmark = pytest.mark.gpu

SHAPE = dict(n_layers=3, d_model=128, n_heads=2, d_ffn=256, vocab=512, max_pos=64)


def _pair(dtype, lr_std=0.05):
    kw = dict(dtype=dtype, batch=2, seq=40, seed=3, plain_small=False, std=lr_std)
    return Model(**SHAPE, **kw), Model(**SHAPE, streamed=True, **kw)


@pytest.mark.parametrize("dtype,lr", [(zi.BF16, 3e-2), (zi.FP16, 3e-3), (zi.FP32, 1e-3)])
def test_streamed_equals_resident_bit_for_bit(dtype, lr):
    res, stm = _pair(dtype)
    tok, tok_dev = res.tokens()
    for seed in (0, 1, 2, 3):
        a = zo_amd.zo_step(res.handle, tok_dev, 2, 40, seed, 1e-3, lr)
        b = zo_amd.zo_step(stm.handle, tok_dev, 2, 40, seed, 1e-3, lr)
        assert a == b, (seed, a, b)                         # same kernels, same order per element: same bits
    th_res = res.theta()
    before_flush = stm.theta()
    assert any(x.tobytes() != y.tobytes() for x, y in zip(th_res, before_flush))      # last update still pending
    zo_amd.zo_flush_pending(stm.handle)
    zo_amd.zo_flush_pending(stm.handle)                     # second flush is a no-op
    assert all(x.tobytes() == y.tobytes() for x, y in zip(th_res, stm.theta()))
    assert any(x.tobytes() != y.tobytes() for x, y in zip(th_res, res.theta0))        # and the steps did move theta
    res.close(); stm.close()


def test_streamed_matches_the_oracles_alg2_runner():
    stm = Model(**SHAPE, dtype=zi.FP32, batch=2, seq=40, seed=4, plain_small=False, std=0.05, streamed=True)
    tok, tok_dev = stm.tokens()
    theta = [t.copy() for t in stm.theta0]
    runner = zo.Alg2Runner(stm.ocfg, theta, 1e-3, 1e-3, literal=False)
    for seed in (5, 6, 7):
        lp, lm, g = zo_amd.zo_step(stm.handle, tok_dev, 2, 40, seed, 1e-3, 1e-3)
        olp, olm, og = runner.step(tok, seed)
        assert abs(lp / olp - 1) < 1e-10 and abs(lm / olm - 1) < 1e-10
        assert abs(g / og - 1) < 1e-5
    zo_amd.zo_flush_pending(stm.handle)
    runner.flush()
    for a, b in zip(stm.theta(), theta):
        assert np.all(np.abs(a.astype(np.float64) - b) <= 1e-5 * np.abs(b) + 1e-10)
    stm.close()


def test_manual_schedule_equals_zo_step_and_state_errors():
    a = Model(**SHAPE, dtype=zi.BF16, batch=2, seq=40, seed=3, plain_small=False, std=0.05, streamed=True)
    b = Model(**SHAPE, dtype=zi.BF16, batch=2, seq=40, seed=3, plain_small=False, std=0.05, streamed=True)
    tok, tok_dev = a.tokens()
    P, C, W = zo_amd.ZO_PHASE_PREFETCH, zo_amd.ZO_PHASE_COMPUTE, zo_amd.ZO_PHASE_WRITEBACK
    L = SHAPE["n_layers"]
    for seed in (0, 1):
        want = zo_amd.zo_step(a.handle, tok_dev, 2, 40, seed, 1e-3, 3e-2)
        zo_amd.zo_stream_begin(b.handle, tok_dev, 2, 40, seed, 1e-3)
        zo_amd.zo_stream_block(b.handle, 0, P)
        for l in range(L):                                   # Alg. 3: U(W_{l+1}) with C(W_l), then O(W_l)
            if l + 1 < L:
                zo_amd.zo_stream_block(b.handle, l + 1, P)
            zo_amd.zo_stream_block(b.handle, l, C | W)
        got = zo_amd.zo_stream_end(b.handle, 3e-2)
        assert got == want
    zo_amd.zo_flush_pending(a.handle); zo_amd.zo_flush_pending(b.handle)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(a.theta(), b.theta()))

    def status(fn, *args):
        with pytest.raises(zo_amd.ZoError) as e:
            fn(*args)
        return e.value.status

    zo_amd.zo_step(b.handle, tok_dev, 2, 40, 8, 1e-3, 3e-2)                                # leaves an update pending
    assert status(zo_amd.zo_stream_block, b.handle, 0, C) == zo_amd.ZO_ESTATE              # no step open
    assert status(zo_amd.zo_dual_forward, b.handle, tok_dev, 2, 40, 0, 1e-3) == zo_amd.ZO_ESTATE
    assert status(zo_amd.zo_perturb, b.handle, 0, 1e-3, 2, 1) == zo_amd.ZO_ESTATE          # a host-resident tensor
    zo_amd.zo_perturb(b.handle, 0, 0.0, 0, 2)                                              # device-resident ones are fine
    zo_amd.zo_stream_begin(b.handle, tok_dev, 2, 40, 9, 1e-3)
    assert status(zo_amd.zo_stream_begin, b.handle, tok_dev, 2, 40, 9, 1e-3) == zo_amd.ZO_ESTATE   # already open
    assert status(zo_amd.zo_stream_block, b.handle, 0, C) == zo_amd.ZO_ESTATE              # not prefetched
    zo_amd.zo_stream_block(b.handle, 0, P)
    assert status(zo_amd.zo_stream_block, b.handle, 2, P) == zo_amd.ZO_ESTATE              # slot 0 still awaits COMPUTE
    zo_amd.zo_stream_block(b.handle, 1, P)
    assert status(zo_amd.zo_stream_block, b.handle, 1, C) == zo_amd.ZO_ESTATE              # out of order
    assert status(zo_amd.zo_stream_end, b.handle, 1e-3) == zo_amd.ZO_ESTATE                # blocks missing
    assert status(zo_amd.zo_stream_block, b.handle, 7, P) == zo_amd.ZO_EINVAL
    zo_amd.zo_stream_block(b.handle, 0, C)
    assert status(zo_amd.zo_stream_block, b.handle, 2, P) == zo_amd.ZO_ESTATE              # block 0 updated, not written back
    zo_amd.zo_stream_block(b.handle, 0, W)
    zo_amd.zo_stream_block(b.handle, 2, P)
    zo_amd.zo_stream_block(b.handle, 1, C | W)
    zo_amd.zo_stream_block(b.handle, 2, C | W)
    lp, lm, g = zo_amd.zo_stream_end(b.handle, 1e-3)
    assert np.isfinite(g)
    a.close(); b.close()


@pytest.mark.parametrize("dtype,interval", [(zi.BF16, 3), (zi.FP16, 2), (zi.FP32, 4)])
def test_writeback_interval_leaves_results_bit_identical(dtype, interval):
    """Blocks written back only every `interval` steps: losses, g and (after a flush) theta are bit for bit those
    of the resident model; between write-backs the host copies lag; the setting can only change with nothing
    pending."""
    lr = {zi.BF16: 1e-2, zi.FP16: 3e-3, zi.FP32: 1e-3}[dtype]
    res, stm = _pair(dtype)
    zo_amd.zo_set_writeback_interval(stm.handle, interval)
    if dtype == zi.FP16:            # the one-pass multi-update kernel with the stochastic rounding as well
        for mdl in (res, stm):
            zo_amd.zo_set_update_rounding(mdl.handle, zo_amd.ZO_ROUND_STOCHASTIC)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_writeback_interval(res.handle, 2)            # not a streamed model
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_writeback_interval(stm.handle, 17)
    tok, tok_dev = res.tokens()
    block_ids = range(2, 2 + 16 * SHAPE["n_layers"])
    stale_seen = False
    for seed in range(2 * interval + 2):
        a = zo_amd.zo_step(res.handle, tok_dev, 2, 40, seed, 1e-3, lr)
        b = zo_amd.zo_step(stm.handle, tok_dev, 2, 40, seed, 1e-3, lr)
        assert a == b, (seed, a, b)
        host = stm.theta()
        if seed == 0:
            assert all(host[i].tobytes() == stm.theta0[i].tobytes() for i in block_ids)     # nothing written back yet
        if seed == interval:        # the step that found `interval` pending updates wrote the blocks back
            assert any(host[i].tobytes() != stm.theta0[i].tobytes() for i in block_ids)
            stale_seen = True
    assert stale_seen
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_writeback_interval(stm.handle, 1)            # updates pending
    zo_amd.zo_flush_pending(stm.handle)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(res.theta(), stm.theta()))
    zo_amd.zo_set_writeback_interval(stm.handle, 1)                # allowed again after the flush
    a = zo_amd.zo_step(res.handle, tok_dev, 2, 40, 99, 1e-3, lr)
    b = zo_amd.zo_step(stm.handle, tok_dev, 2, 40, 99, 1e-3, lr)
    assert a == b
    zo_amd.zo_flush_pending(stm.handle)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(res.theta(), stm.theta()))
    res.close(); stm.close()


@pytest.mark.parametrize("dtype,device_blocks,interval", [(zi.BF16, (0,), 1), (zi.BF16, (1,), 1), (zi.BF16, (0, 2), 3),
                                                         (zi.FP16, (1, 2), 2), (zi.FP32, (0, 1, 2), 1), (zi.BF16, (2,), 2)])
def test_blocks_kept_in_hbm_leave_results_bit_identical(dtype, device_blocks, interval):
    """A streamed model keeps each block where its pointers say: some in pinned host memory (uploaded per visit),
    some in device memory (no transfer).  Losses, g and, after a flush, theta are those of the resident model bit
    for bit, for any placement, with the write-back interval and the stochastic rounding as well."""
    lr = {zi.BF16: 1e-2, zi.FP16: 3e-3, zi.FP32: 1e-3}[dtype]
    kw = dict(dtype=dtype, batch=2, seq=40, seed=3, plain_small=False, std=0.05)
    res = Model(**SHAPE, **kw)
    mix = Model(**SHAPE, streamed=True, device_blocks=device_blocks, **kw)
    if interval > 1:
        zo_amd.zo_set_writeback_interval(mix.handle, interval)
    if dtype == zi.FP16:
        for mdl in (res, mix):
            zo_amd.zo_set_update_rounding(mdl.handle, zo_amd.ZO_ROUND_STOCHASTIC)
    tok, tok_dev = res.tokens()
    for seed in range(2 * interval + 1):
        a = zo_amd.zo_step(res.handle, tok_dev, 2, 40, seed, 1e-3, lr)
        b = zo_amd.zo_step(mix.handle, tok_dev, 2, 40, seed, 1e-3, lr)
        assert a == b, (seed, a, b)
    assert any(x.tobytes() != y.tobytes() for x, y in zip(res.theta(), mix.theta()))      # the last update is pending
    zo_amd.zo_flush_pending(mix.handle)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(res.theta(), mix.theta()))
    # and on after the flush, through the manual schedule (uploads and write-backs of HBM blocks are no-ops)
    zo_amd.zo_stream_begin(mix.handle, tok_dev, 2, 40, 77, 1e-3)
    P, C, W = zo_amd.ZO_PHASE_PREFETCH, zo_amd.ZO_PHASE_COMPUTE, zo_amd.ZO_PHASE_WRITEBACK
    for l in range(SHAPE["n_layers"]):
        zo_amd.zo_stream_block(mix.handle, l, P | C | W)
    b = zo_amd.zo_stream_end(mix.handle, lr)
    a = zo_amd.zo_step(res.handle, tok_dev, 2, 40, 77, 1e-3, lr)
    assert a == b
    zo_amd.zo_flush_pending(mix.handle)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(res.theta(), mix.theta()))
    # a perturbation may touch a block in HBM, not one in host memory
    zo_amd.zo_perturb(mix.handle, 5, 1e-3, 2 + 16 * device_blocks[0], 16)
    host_blocks = [l for l in range(SHAPE["n_layers"]) if l not in device_blocks]
    if host_blocks:
        with pytest.raises(zo_amd.ZoError):
            zo_amd.zo_perturb(mix.handle, 5, 1e-3, 2 + 16 * host_blocks[0], 16)
    res.close(); mix.close()


@pytest.mark.parametrize("lookahead", [0, 1])
def test_steps_queued_without_host_waits_leave_the_same_bits(lookahead):
    """zo_step without host out-pointers: the host runs up to one step ahead of the device (or none with look-ahead 0).
    Six steps queued that way, with a write-back interval of 2 and one block kept in HBM, end in the theta of the
    resident model bit for bit, and the last step's losses are the resident model's."""
    kw = dict(dtype=zi.BF16, batch=2, seq=40, seed=3, plain_small=False, std=0.05)
    res = Model(**SHAPE, **kw)
    stm = Model(**SHAPE, streamed=True, device_blocks=(1,), **kw)
    zo_amd.zo_set_stream_lookahead(stm.handle, lookahead)
    zo_amd.zo_set_writeback_interval(stm.handle, 2)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_stream_lookahead(res.handle, 1)              # not a streamed model
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_stream_lookahead(stm.handle, 2)
    tok, tok_dev = res.tokens()
    for seed in range(6):
        zo_amd.zo_step(res.handle, tok_dev, 2, 40, seed, 1e-3, 1e-2, want_host=False)
        zo_amd.zo_step(stm.handle, tok_dev, 2, 40, seed, 1e-3, 1e-2, want_host=False)
    a = zo_amd.zo_step(res.handle, tok_dev, 2, 40, 6, 1e-3, 1e-2)
    b = zo_amd.zo_step(stm.handle, tok_dev, 2, 40, 6, 1e-3, 1e-2)
    assert a == b and np.isfinite(a[2])
    zo_amd.zo_flush_pending(stm.handle)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(res.theta(), stm.theta()))
    res.close(); stm.close()


def test_profile_classes_and_alg3_spans_of_a_streamed_step():
    """zo_profile_*: per-class kernel times and work, and the (upload, kernels, write-back) records of Alg. 3's
    schedule: one of each per streamed block and step, every block's kernels after its upload, its write-back after
    its kernels, block i + 1's upload not waiting for block i's kernels to end; profiling changes no result."""
    L = SHAPE["n_layers"]
    ref = Model(**SHAPE, dtype=zi.BF16, batch=2, seq=40, seed=3, plain_small=False, std=0.05, streamed=True)
    stm = Model(**SHAPE, dtype=zi.BF16, batch=2, seq=40, seed=3, plain_small=False, std=0.05, streamed=True, device_blocks=(1,))
    tok, tok_dev = stm.tokens()
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_profile_end(stm.handle)                               # not begun
    zo_amd.zo_profile_begin(stm.handle, 4096)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_profile_spans(stm.handle)                             # still on
    got = [zo_amd.zo_step(stm.handle, tok_dev, 2, 40, seed, 1e-3, 1e-2) for seed in (0, 1)]
    classes = zo_amd.zo_profile_end(stm.handle)
    spans = zo_amd.zo_profile_spans(stm.handle)
    want = [zo_amd.zo_step(ref.handle, tok_dev, 2, 40, seed, 1e-3, 1e-2) for seed in (0, 1)]
    assert got == want
    # classes: 2 steps x (4 GEMMs per block + the LM head, one launch or one per sign and row chunk), attention and
    # LayerNorm per block, staging per block + globals
    assert classes["linear"][1] >= 2 * (4 * L + 1) and classes["attention"][1] == 2 * L
    assert classes["norm"][1] == 2 * (2 * L + 1) and classes["stage"][1] >= 2 * (L + 1)
    for name in ("linear", "attention", "stage", "norm"):
        ms, launches, work = classes[name]
        assert ms > 0 and work > 0, name
    M, d, F = 2 * 2 * 40, SHAPE["d_model"], SHAPE["d_ffn"]
    flop = 2.0 * M * (L * (4 * d * d + 2 * d * F) + d * SHAPE["vocab"])
    assert abs(classes["linear"][2] / (2 * flop) - 1) < 1e-12          # 2 m n k over every GEMM of the two steps
    # spans: blocks 0 and 2 stream (upload, kernels, write-back each step), block 1 lives in HBM (kernels only)
    by = {}
    for kind, block, t0, t1 in spans:
        assert 0 <= block < L and t0 >= 0 and t1 >= t0
        by.setdefault((kind, block), []).append((t0, t1))
    U, C, O = zo_amd.ZO_SPAN_UPLOAD, zo_amd.ZO_SPAN_COMPUTE, zo_amd.ZO_SPAN_WRITEBACK
    assert all(len(by[(C, b)]) == 2 for b in range(L))
    assert (U, 1) not in by and (O, 1) not in by
    for b in (0, 2):
        assert len(by[(U, b)]) == 2
        assert len(by[(O, b)]) >= 1                                     # step 1 has no update to write back yet
        for (u0, u1), (c0, c1) in zip(by[(U, b)], by[(C, b)]):
            assert c0 >= u1 - 1e-3                                      # kernels start once the block has landed
        last_c, last_o = by[(C, b)][-1], by[(O, b)][-1]
        assert last_o[0] >= last_c[0]                                   # written back after its update was enqueued
    assert min(t0 for _, _, t0, _ in spans) == 0.0
    ref.close(); stm.close()

"""GPU parity on configuration 2 as specified: OPT-125m shape, bf16 storage with fp32 accumulation,
batch 16 x seq 512, ten ZO-SGD steps with eps 1e-3, lr 1e-6 and seeds 0..9.  Expected values were
written by tests/golden/make_config2_golden.py, which calls only the oracle (fp64 forward over the same
bf16-rounded W+-).  Tolerances of the configuration: losses within 2e-2 relative, g sign-consistent."""
import json
import os

import numpy as np
import pytest
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from gpu_util import Model

pytestmark = pytest.mark.gpu


def test_config2_ten_steps_against_the_oracle():
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "config2_opt125m_steps.json")))
    c = zi.CONFIGS["opt-125m"]
    mdl = Model(c["n_layers"], c["d_model"], c["n_heads"], c["d_ffn"], c["vocab"], c["max_pos"], c["dtype"], c["batch"], c["seq"],
                seed=gold["weights_seed"], plain_small=True, std=0.02)
    _, tok_dev = mdl.tokens(seed=gold["tokens_seed"])
    got = [zo_amd.zo_step(mdl.handle, tok_dev, c["batch"], c["seq"], st["seed"], c["eps"], c["lr"]) for st in gold["steps"]]
    noise = 0.0
    for (lp, lm, g), st in zip(got, gold["steps"]):
        assert abs(lp / st["l_plus"] - 1) < 2e-2 and abs(lm / st["l_minus"] - 1) < 2e-2, (st, lp, lm)
        noise = max(noise, abs(lp - st["l_plus"]), abs(lm - st["l_minus"]))
    # The configuration asks for 2e-2 on the losses; what bf16 activations really cost at this size is two orders
    # below that (measured 1e-4 .. 2e-4 absolute on losses of 10.97), and the sign test below depends on it: bound it.
    assert noise < 2.9e-4, noise
    # sign of g wherever the oracle's loss difference stands clear of the bf16 loss noise; the rest are listed.  The
    # oracle's |l+ - l-| is at least 1.19e-3 > 4 x 2.9e-4 on eight of the ten seeds of this golden file (3.7e-4 and
    # 4.1e-4 on the other two), so at least eight are checked whenever the noise bound holds.
    checked, below = 0, []
    for (lp, lm, g), st in zip(got, gold["steps"]):
        diff = st["l_plus"] - st["l_minus"]
        if abs(diff) > 4 * noise:
            assert np.sign(g) == np.sign(st["g"]), (st, g)
            # and its size: the two losses' errors are at most `noise` each
            assert abs(g - st["g"]) <= 2 * noise / (2 * c["eps"]) + 1e-9, (st, g)
            checked += 1
        else:
            below.append(st["seed"])
    print("bf16 loss noise %.3g; sign(g) checked on %d of 10 steps; below 4x noise: seeds %s" % (noise, checked, below))
    print("gpu g:", ["%.3f" % r[2] for r in got], "oracle g:", ["%.3f" % st["g"] for st in gold["steps"]])
    assert checked >= 8, (checked, below, noise)
    assert zo_amd.zo_device_flags(mdl.handle) == 0
    mdl.close()

"""Writes tests/golden/config2_opt125m_steps.json: the oracle's ten ZO-SGD steps of configuration 2
(OPT-125m shape, bf16 storage, batch 16 x seq 512, eps 1e-3, lr 1e-6, seeds 0..9, fused mode).

Calls only oracle/ and the shared input generator.  Takes about a quarter of an hour on 8 cores:

    python tests/golden/make_config2_golden.py
"""
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import zo_inputs as zi                      # noqa: E402
from oracle import zo_oracle as zo          # noqa: E402


def main():
    c = zi.CONFIGS["opt-125m"]
    cfg = zo.Config(c["n_layers"], c["d_model"], c["n_heads"], c["d_ffn"], c["vocab"], c["max_pos"], c["dtype"])
    theta = zi.make_weights(cfg.shapes(), c["dtype"], seed=0)
    tokens = zi.make_tokens(c["batch"], c["seq"], c["vocab"], seed=1)
    steps = []
    for seed in range(10):
        t0 = time.time()
        lp, lm, g = zo.zo_step_fused(cfg, theta, tokens, seed, c["eps"], c["lr"])
        steps.append({"seed": seed, "l_plus": lp, "l_minus": lm, "g": g})
        print(seed, lp, lm, g, "%.1fs" % (time.time() - t0), flush=True)
    out = {"config": "opt-125m", "weights_seed": 0, "tokens_seed": 1, "eps": c["eps"], "lr": c["lr"], "mode": "fused",
           "written_by": "tests/golden/make_config2_golden.py (oracle only)", "steps": steps}
    with open(os.path.join(ROOT, "tests", "golden", "config2_opt125m_steps.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()

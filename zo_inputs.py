"""Seeded synthetic inputs shared by the tests, the smoke run and the bench.

This module holds none of the method's arithmetic: it only draws weights and
tokens from numpy's own generators and lays them out in the canonical tensor
order.  Both the CPU oracle and the HIP library are fed from here, so neither
ever sees values produced by the other.

The paper's experiments fine-tune pretrained OPT checkpoints on SST-2 prompts
(DistZO2, Sec. 7 set-up); neither is available offline, and throughput and
parity do not depend on them.  The stand-in recipe: every weight matrix and
embedding ~ 0.02 * N(0,1), LayerNorm gain 1 and bias 0, linear biases 0,
tokens uniform over the vocabulary, labels = the same tokens shifted by one.
"""
import numpy as np

FP32, BF16, FP16 = 0, 1, 2
BLOCK_TENSORS = ("ln1_g", "ln1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
                 "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")

# name -> (n_layers, d_model, n_heads, d_ffn, vocab, max_pos, dtype, batch, seq, eps, lr)
CONFIGS = {
    "tiny":     dict(n_layers=2,  d_model=64,    n_heads=4,  d_ffn=256,   vocab=512,   max_pos=32,   dtype=FP32, batch=2,  seq=32,   eps=1e-3, lr=1e-5),
    "opt-125m": dict(n_layers=12, d_model=768,   n_heads=12, d_ffn=3072,  vocab=50272, max_pos=2048, dtype=BF16, batch=16, seq=512,  eps=1e-3, lr=1e-6),
    "opt-1.3b": dict(n_layers=24, d_model=2048,  n_heads=32, d_ffn=8192,  vocab=50272, max_pos=2048, dtype=BF16, batch=8,  seq=1024, eps=1e-3, lr=1e-7),
    "opt-13b":  dict(n_layers=40, d_model=5120,  n_heads=40, d_ffn=20480, vocab=50272, max_pos=2048, dtype=BF16, batch=4,  seq=2048, eps=1e-3, lr=1e-7),
    "opt-175b": dict(n_layers=96, d_model=12288, n_heads=96, d_ffn=49152, vocab=50272, max_pos=2048, dtype=FP16, batch=1,  seq=2048, eps=1e-3, lr=1e-7),
}


def tensor_shapes(n_layers, d_model, d_ffn, vocab, max_pos):
    """Canonical order: token embedding, position embedding, 16 tensors per
    block, final LayerNorm gain and bias.  Linear weights are [out, in]
    (y = x W^T + b), the storage order of the OPT checkpoints the paper fine-tunes."""
    d, f = d_model, d_ffn
    blk = {"ln1_g": (d,), "ln1_b": (d,), "wq": (d, d), "bq": (d,), "wk": (d, d), "bk": (d,),
           "wv": (d, d), "bv": (d,), "wo": (d, d), "bo": (d,), "ln2_g": (d,), "ln2_b": (d,),
           "w1": (f, d), "b1": (f,), "w2": (d, f), "b2": (d,)}
    out = [("embed_tokens", (vocab, d)), ("embed_pos", (max_pos, d))]
    for l in range(n_layers):
        out += [("l%d.%s" % (l, n), blk[n]) for n in BLOCK_TENSORS]
    out += [("lnf_g", (d,)), ("lnf_b", (d,))]
    return out


def round_to_storage(x32, dtype):
    """fp32 numpy array -> storage array (float32 / uint16 bf16 bits / float16),
    using the library casts of numpy and torch."""
    if dtype == FP32:
        return np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == FP16:
        return x32.astype(np.float16)
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def make_weights(shapes, dtype, seed=0, std=0.02, plain_small=True):
    """List of storage arrays in canonical order.  `plain_small=True` gives the
    recipe above (gain 1, biases 0); False draws every tensor at random, which
    the parity tests use so that biases and LayerNorm parameters matter."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for name, shape in shapes:
        leaf = name.split(".")[-1]
        if len(shape) == 2:
            x = (std * rng.standard_normal(shape)).astype(np.float32)
        elif plain_small:
            x = np.ones(shape, np.float32) if leaf.endswith("_g") else np.zeros(shape, np.float32)
        elif leaf.endswith("_g"):
            x = (1.0 + 0.1 * rng.standard_normal(shape)).astype(np.float32)
        else:
            x = (0.1 * rng.standard_normal(shape)).astype(np.float32)
        out.append(round_to_storage(x, dtype))
    return out


def make_tokens(batch, seq, vocab, seed=1):
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, vocab, size=(batch, seq), dtype=np.int64).astype(np.int32)

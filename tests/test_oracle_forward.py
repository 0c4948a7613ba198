"""Pins for the oracle's decoder forward and loss (oracle/zo_oracle.py):
a library model class fed the same weights, closed-form special cases and
structural invariants."""
import numpy as np
import pytest

import zo_inputs as zi
from oracle import zo_oracle as zo


def _cfg(n_layers=2, d=32, h=4, f=64, v=50, p=16, dtype=zo.FP32):
    return zo.Config(n_layers, d, h, f, v, p, dtype)


def _weights64(cfg, seed=0, plain_small=False, std=0.2):
    th = zi.make_weights(cfg.shapes(), zo.FP32, seed=seed, std=std, plain_small=plain_small)
    return [t.astype(np.float64) for t in th]


def test_shapes_agree_with_input_module():
    cfg = _cfg()
    assert cfg.shapes() == zi.tensor_shapes(cfg.n_layers, cfg.d_model, cfg.d_ffn, cfg.vocab, cfg.max_pos)
    assert cfg.n_tensors == len(cfg.shapes()) == 4 + 16 * cfg.n_layers
    assert zi.BLOCK_TENSORS == zo.BLOCK_TENSORS


def test_logits_match_transformers_opt_class():
    """The `transformers` OPT decoder (an independent implementation of the same
    architecture) given our weights: linear weights as they are (its layout is
    [out, in] too) and positions shifted by its two reserved rows."""
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    cfg = _cfg(n_layers=2, d=32, h=4, f=64, v=50, p=16)
    w = _weights64(cfg, seed=3)
    hf_cfg = tr.OPTConfig(vocab_size=cfg.vocab, hidden_size=cfg.d_model, num_hidden_layers=cfg.n_layers,
                          ffn_dim=cfg.d_ffn, num_attention_heads=cfg.n_heads, max_position_embeddings=cfg.max_pos,
                          do_layer_norm_before=True, word_embed_proj_dim=cfg.d_model, dropout=0.0,
                          attention_dropout=0.0, activation_function="relu", layerdrop=0.0, enable_bias=True,
                          layer_norm_elementwise_affine=True, tie_word_embeddings=True)
    model = tr.OPTForCausalLM(hf_cfg).double().eval()
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    dec = model.model.decoder
    with torch.no_grad():
        dec.embed_tokens.weight.copy_(T(w[0]))
        dec.embed_positions.weight.zero_()
        dec.embed_positions.weight[2:].copy_(T(w[1]))
        for l, layer in enumerate(dec.layers):
            p = dict(zip(zo.BLOCK_TENSORS, [w[i] for i in cfg.block_ids(l)]))
            layer.self_attn_layer_norm.weight.copy_(T(p["ln1_g"])); layer.self_attn_layer_norm.bias.copy_(T(p["ln1_b"]))
            for name, wn, bn in (("q_proj", "wq", "bq"), ("k_proj", "wk", "bk"), ("v_proj", "wv", "bv"), ("out_proj", "wo", "bo")):
                lin = getattr(layer.self_attn, name)
                lin.weight.copy_(T(p[wn])); lin.bias.copy_(T(p[bn]))
            layer.final_layer_norm.weight.copy_(T(p["ln2_g"])); layer.final_layer_norm.bias.copy_(T(p["ln2_b"]))
            layer.fc1.weight.copy_(T(p["w1"])); layer.fc1.bias.copy_(T(p["b1"]))
            layer.fc2.weight.copy_(T(p["w2"])); layer.fc2.bias.copy_(T(p["b2"]))
        g_id, b_id = cfg.head_ids()
        dec.final_layer_norm.weight.copy_(T(w[g_id])); dec.final_layer_norm.bias.copy_(T(w[b_id]))
        model.lm_head.weight = dec.embed_tokens.weight
        tokens = zi.make_tokens(3, 12, cfg.vocab, seed=4)
        ids = torch.from_numpy(tokens.astype(np.int64))
        out = model(input_ids=ids, labels=ids)
    ours = zo.logits_of(cfg, w, tokens)
    assert np.max(np.abs(ours - out.logits.numpy())) < 1e-10
    # the class reports its loss in fp32; torch's own cross entropy on its fp64 logits is the sharp check
    assert abs(zo.loss(cfg, w, tokens) - float(out.loss)) < 1e-6
    ce = torch.nn.functional.cross_entropy(out.logits[:, :-1].reshape(-1, cfg.vocab), ids[:, 1:].reshape(-1))
    assert abs(zo.loss(cfg, w, tokens) - float(ce)) < 1e-12


def test_blocks_are_identity_when_output_projections_vanish():
    cfg = _cfg()
    w = _weights64(cfg, seed=5)
    for l in range(cfg.n_layers):
        ids = dict(zip(zo.BLOCK_TENSORS, cfg.block_ids(l)))
        for name in ("wo", "bo", "w2", "b2"):
            w[ids[name]][...] = 0
    tokens = zi.make_tokens(2, 9, cfg.vocab, seed=6)
    h = w[0][tokens] + w[1][:9][None]
    mu = h.mean(-1, keepdims=True)
    var = h.var(-1, keepdims=True)
    g_id, b_id = cfg.head_ids()
    want = ((h - mu) / np.sqrt(var + cfg.ln_eps) * w[g_id] + w[b_id]) @ w[0].T
    assert np.allclose(zo.logits_of(cfg, w, tokens), want, rtol=0, atol=1e-12)


def test_zero_model_has_loss_log_vocab_and_small_init_is_close():
    cfg = _cfg(v=64)
    w = [np.zeros(s) for _, s in cfg.shapes()]
    tokens = zi.make_tokens(2, 10, cfg.vocab)
    assert abs(zo.loss(cfg, w, tokens) - np.log(64)) < 1e-12
    c = zi.CONFIGS["tiny"]
    tiny = zo.Config(c["n_layers"], c["d_model"], c["n_heads"], c["d_ffn"], c["vocab"], c["max_pos"], c["dtype"])
    th = zi.make_weights(tiny.shapes(), tiny.dtype, seed=0)
    tok = zi.make_tokens(c["batch"], c["seq"], c["vocab"])
    assert abs(zo.loss_of_storage(tiny, th, tok) / np.log(512) - 1) < 0.01


def test_causality_and_batch_independence():
    cfg = _cfg()
    w = _weights64(cfg, seed=8)
    tokens = zi.make_tokens(2, 12, cfg.vocab, seed=9)
    base = zo.logits_of(cfg, w, tokens)
    changed = tokens.copy()
    changed[0, 7] = (changed[0, 7] + 1) % cfg.vocab
    out = zo.logits_of(cfg, w, changed)
    assert np.array_equal(out[0, :7], base[0, :7])        # earlier positions untouched
    assert not np.allclose(out[0, 7:], base[0, 7:])       # later ones move
    assert np.array_equal(out[1], base[1])                # other sequences untouched
    assert np.allclose(zo.logits_of(cfg, w, tokens[1:]), base[1:], atol=1e-13)


def test_loss_against_direct_definition():
    cfg = _cfg()
    w = _weights64(cfg, seed=10)
    tokens = zi.make_tokens(2, 7, cfg.vocab, seed=11)
    logits = zo.logits_of(cfg, w, tokens)
    total = 0.0
    for b in range(2):
        for t in range(6):
            p = np.exp(logits[b, t]) / np.exp(logits[b, t]).sum()
            total -= np.log(p[tokens[b, t + 1]])
    assert abs(zo.next_token_loss(logits, tokens) - total / 12) < 1e-12


def test_softmax_scale_and_head_split():
    """A single block against a direct per-head loop with explicit 1/sqrt(d_h)."""
    cfg = _cfg(n_layers=1, d=24, h=3, f=48)
    w = _weights64(cfg, seed=12)
    p = dict(zip(zo.BLOCK_TENSORS, [w[i] for i in cfg.block_ids(0)]))
    rng = np.random.default_rng(13)
    h = rng.standard_normal((1, 5, 24))
    ln = lambda x, g, b: (x - x.mean(-1, keepdims=True)) / np.sqrt(x.var(-1, keepdims=True) + cfg.ln_eps) * g + b
    a = ln(h[0], p["ln1_g"], p["ln1_b"])
    lin = lambda x, wgt, b: np.einsum("ti,oi->to", x, wgt) + b            # y[t, o] = sum_i x[t, i] W[o, i] + b[o]
    q, k, v = lin(a, p["wq"], p["bq"]), lin(a, p["wk"], p["bk"]), lin(a, p["wv"], p["bv"])
    o = np.zeros((5, 24))
    for head in range(3):
        sl = slice(8 * head, 8 * head + 8)
        for t in range(5):
            sc = np.array([q[t, sl] @ k[u, sl] / np.sqrt(8.0) for u in range(t + 1)])
            pr = np.exp(sc - sc.max()); pr /= pr.sum()
            o[t, sl] = sum(pr[u] * v[u, sl] for u in range(t + 1))
    h1 = h[0] + lin(o, p["wo"], p["bo"])
    f = np.maximum(lin(ln(h1, p["ln2_g"], p["ln2_b"]), p["w1"], p["b1"]), 0)
    want = h1 + lin(f, p["w2"], p["b2"])
    got = zo.block_forward(h, p, 3, cfg.ln_eps)[0]
    assert np.allclose(got, want, rtol=0, atol=1e-12)

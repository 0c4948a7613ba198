"""CPU oracle, part 2: the OPT-style decoder loss and the ZO-SGD step.

TEST INFRASTRUCTURE ONLY.  Plain numpy in fp64, written from the paper
(DistZO2, arXiv 2507.03211), slow on purpose and free of any blocking, fusion
or reordering.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import it; it shares no code with the HIP library and
imports nothing from the product package.

What each function follows:
  * `loss` and the module functions below it: the forward L(theta; B) that
    Eq. 1 evaluates twice.  The paper's experiments use the OPT family
    (Sec. 7 set-up); the architecture constants are the usual OPT ones
    (pre-LayerNorm decoder, ReLU FFN, learned positions, LM head tied to the
    token embedding, mean next-token cross-entropy).
  * `zo_step_literal`:  App. A, Alg. 1 (MeZO): +eps, loss, -2 eps, loss, +eps,
    g = (l+ - l-)/(2 eps)  [Eq. 1],  theta <- theta - eta g z  [Eq. 2].
  * `zo_step_fused`: the same step with W+- = rn(theta +- eps z) formed from an
    untouched theta (PertP workflow, Step 2: W+ = W_H + eps z, W- = W_H - eps z).
  * `Alg2Runner`: App. A, Alg. 2 (ZO2): module by module, the previous step's
    update applied to a module right before this step's perturbation of it.

Storage types: a parameter tensor is held as a numpy array in its storage type
(float32; uint16 holding bfloat16 bits; float16).  The random direction and the
rounding into the storage type come from the C part (zo_oracle_rng.c); all
forward arithmetic is fp64 on the widened values.

Pins: tests/test_oracle_forward.py and tests/test_oracle_step.py (a library
model class given the same weights, autograd's directional derivative, brute
force finite differences on a tiny model, closed-form special cases).
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))

FP32, BF16, FP16 = 0, 1, 2
TENSORS_PER_BLOCK = 16
# order inside one block (tensor id = 2 + 16*layer + position in this list)
BLOCK_TENSORS = ("ln1_g", "ln1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
                 "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


# --------------------------------------------------------------------------
# the C part
# --------------------------------------------------------------------------
_lib = None


def _clib():
    global _lib
    if _lib is None:
        path = os.path.join(_HERE, "_build", "liboracle_zo.so")
        if not os.path.exists(path):
            import importlib.util
            spec = importlib.util.spec_from_file_location("_oracle_build", os.path.join(_HERE, "build.py"))
            mod = importlib.util.module_from_spec(spec)
            spec.loader.exec_module(mod)
            mod.build()
        lib = ctypes.CDLL(path)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        lib.zo_oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        lib.zo_oracle_normal_pair.argtypes = [ctypes.c_uint32, ctypes.c_uint32,
                                              ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
        lib.zo_oracle_normal_pairs.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64]
        lib.zo_oracle_z.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint64,
                                    ctypes.c_uint64, ctypes.c_void_p]
        lib.zo_oracle_axpy_z.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64,
                                         ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_float]
        lib.zo_oracle_axpy_z_sr.argtypes = lib.zo_oracle_axpy_z.argtypes
        lib.zo_oracle_sr_array.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64]
        lib.zo_oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        lib.zo_oracle_f32_to_bf16.restype = ctypes.c_uint16
        lib.zo_oracle_f32_to_f16.argtypes = [ctypes.c_float]
        lib.zo_oracle_f32_to_f16.restype = ctypes.c_uint16
        lib.zo_oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        lib.zo_oracle_bf16_to_f32.restype = ctypes.c_float
        lib.zo_oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        lib.zo_oracle_f16_to_f32.restype = ctypes.c_float
        _lib = lib
    return _lib


def philox(counter, key):
    lib = _clib()
    c = (ctypes.c_uint32 * 4)(*counter)
    k = (ctypes.c_uint32 * 2)(*key)
    o = (ctypes.c_uint32 * 4)()
    lib.zo_oracle_philox4x32_10(c, k, o)
    return tuple(int(x) for x in o)


def normal_pair(ra, rb):
    a, b = ctypes.c_float(), ctypes.c_float()
    _clib().zo_oracle_normal_pair(ra, rb, ctypes.byref(a), ctypes.byref(b))
    return np.float32(a.value), np.float32(b.value)


def normal_pairs(words):
    """The transform over a uint32 array of word pairs (even length) -> fp32 array of the same length."""
    words = np.ascontiguousarray(words, dtype=np.uint32)
    assert words.size % 2 == 0
    out = np.empty(words.size, dtype=np.float32)
    _clib().zo_oracle_normal_pairs(words.ctypes.data, out.ctypes.data, words.size // 2)
    return out


def z_values(seed, tensor_id, first, n, stream_tag=0):
    """fp32 z for elements [first, first+n) of tensor `tensor_id`."""
    out = np.empty(int(n), dtype=np.float32)
    _clib().zo_oracle_z(int(seed), int(tensor_id), int(stream_tag), int(first), int(n), out.ctypes.data)
    return out


def storage_dtype(dtype):
    return {FP32: np.float32, BF16: np.uint16, FP16: np.float16}[dtype]


def axpy_z(src, dtype, seed, tensor_id, scale, first=0, out=None, stochastic=False):
    """rn(fma(scale, z, src)) element-wise, in the storage type.  `src` is the
    slice of the tensor that starts at element `first`.  Returns a new array
    unless `out` is given (out may be src: in place).  `stochastic=True`
    replaces the round-to-nearest by the opt-in stochastic rounding (2-byte
    types only; random words from Philox tag 3)."""
    src = np.ascontiguousarray(src)
    assert src.dtype == storage_dtype(dtype), (src.dtype, dtype)
    if out is None:
        out = np.empty_like(src)
    assert out.flags.c_contiguous and out.dtype == src.dtype and out.shape == src.shape
    assert not (stochastic and dtype == FP32), "stochastic rounding is for the 2-byte storage types"
    fn = _clib().zo_oracle_axpy_z_sr if stochastic else _clib().zo_oracle_axpy_z
    fn(src.ctypes.data, out.ctypes.data, int(dtype), int(seed), int(tensor_id),
       int(first), int(src.size), ctypes.c_float(float(np.float32(scale))))
    return out


def sr_round(values, words, dtype):
    """Stochastic rounding of fp32 `values` with the given uint32 random words,
    element-wise, into the 2-byte storage type (bf16 as uint16 patterns)."""
    v = np.ascontiguousarray(values, dtype=np.float32)
    w = np.ascontiguousarray(words, dtype=np.uint32)
    assert v.shape == w.shape and dtype in (BF16, FP16)
    out = np.empty(v.shape, dtype=np.uint16)
    _clib().zo_oracle_sr_array(v.ctypes.data, w.ctypes.data, out.ctypes.data, int(dtype), int(v.size))
    return out if dtype == BF16 else out.view(np.float16)


def to_storage(x, dtype):
    """Round an fp32/fp64 array to the storage type (nearest even)."""
    x32 = np.asarray(x, dtype=np.float32)
    if dtype == FP32:
        return x32.copy()
    if dtype == FP16:
        return x32.astype(np.float16)
    # bf16: nearest-even on the bit pattern (NaN is not expected in weights)
    bits = x32.ravel().view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    return ((bits + 0x7FFF + lsb) >> 16).astype(np.uint16).reshape(x32.shape)


def widen(a, dtype):
    """Storage array -> fp64 values."""
    if dtype == BF16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# --------------------------------------------------------------------------
# model description
# --------------------------------------------------------------------------
class Config:
    def __init__(self, n_layers, d_model, n_heads, d_ffn, vocab, max_pos, dtype=FP32, ln_eps=1e-5):
        assert d_model % n_heads == 0
        self.n_layers, self.d_model, self.n_heads = n_layers, d_model, n_heads
        self.d_ffn, self.vocab, self.max_pos = d_ffn, vocab, max_pos
        self.dtype, self.ln_eps = dtype, ln_eps

    @property
    def n_tensors(self):
        return 4 + TENSORS_PER_BLOCK * self.n_layers

    def shapes(self):
        """Canonical tensor order; linear weights are [out, in] row-major (y = x W^T + b): the order in which
        the OPT checkpoints of the paper's experiments (Sec. 7) keep them, hence the order in which Alg. 1's
        "for each theta_i" meets the elements of a matrix when it draws z."""
        d, f = self.d_model, self.d_ffn
        out = [("embed_tokens", (self.vocab, d)), ("embed_pos", (self.max_pos, d))]
        blk = {"ln1_g": (d,), "ln1_b": (d,), "wq": (d, d), "bq": (d,), "wk": (d, d), "bk": (d,),
               "wv": (d, d), "bv": (d,), "wo": (d, d), "bo": (d,), "ln2_g": (d,), "ln2_b": (d,),
               "w1": (f, d), "b1": (f,), "w2": (d, f), "b2": (d,)}
        for l in range(self.n_layers):
            for name in BLOCK_TENSORS:
                out.append(("l%d.%s" % (l, name), blk[name]))
        out += [("lnf_g", (d,)), ("lnf_b", (d,))]
        return out

    def block_ids(self, layer):
        base = 2 + TENSORS_PER_BLOCK * layer
        return list(range(base, base + TENSORS_PER_BLOCK))

    def head_ids(self):
        return [self.n_tensors - 2, self.n_tensors - 1]


# --------------------------------------------------------------------------
# forward, module by module (fp64)
# --------------------------------------------------------------------------
def layer_norm(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def embed(tokens, w_tok, w_pos):
    """h[b, t, :] = E[x[b, t]] + Pos[t]."""
    S = tokens.shape[1]
    return w_tok[tokens] + w_pos[:S][None, :, :]


def causal_attention(q, k, v, n_heads):
    """softmax(q k^T / sqrt(d_head), keys <= query) v per head; q, k, v are [B, S, d]."""
    B, S, d = q.shape
    dh = d // n_heads
    q = q.reshape(B, S, n_heads, dh).transpose(0, 2, 1, 3)
    k = k.reshape(B, S, n_heads, dh).transpose(0, 2, 1, 3)
    v = v.reshape(B, S, n_heads, dh).transpose(0, 2, 1, 3)
    scores = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(float(dh))
    future = np.triu(np.ones((S, S), dtype=bool), k=1)
    scores = np.where(future[None, None], -np.inf, scores)
    scores = scores - scores.max(axis=-1, keepdims=True)
    prob = np.exp(scores)
    prob = prob / prob.sum(axis=-1, keepdims=True)
    return (prob @ v).transpose(0, 2, 1, 3).reshape(B, S, d)


def block_forward(h, p, n_heads, ln_eps):
    """One pre-LN decoder block.  `p` maps the names of BLOCK_TENSORS to fp64 arrays."""
    a = layer_norm(h, p["ln1_g"], p["ln1_b"], ln_eps)
    q = a @ p["wq"].T + p["bq"]
    k = a @ p["wk"].T + p["bk"]
    v = a @ p["wv"].T + p["bv"]
    o = causal_attention(q, k, v, n_heads)
    h = h + o @ p["wo"].T + p["bo"]
    f = layer_norm(h, p["ln2_g"], p["ln2_b"], ln_eps)
    f = np.maximum(f @ p["w1"].T + p["b1"], 0.0)
    return h + f @ p["w2"].T + p["b2"]


def head_logits(h, lnf_g, lnf_b, w_tok, ln_eps):
    return layer_norm(h, lnf_g, lnf_b, ln_eps) @ w_tok.T


def next_token_loss(logits, tokens):
    """Mean over b and t < S-1 of logsumexp(logits[b,t]) - logits[b,t,x[b,t+1]]."""
    lg = logits[:, :-1, :]
    tgt = tokens[:, 1:]
    mx = lg.max(axis=-1, keepdims=True)
    lse = np.log(np.exp(lg - mx).sum(axis=-1)) + mx[..., 0]
    picked = np.take_along_axis(lg, tgt[..., None], axis=-1)[..., 0]
    return float((lse - picked).mean())


def logits_of(cfg, w64, tokens):
    """Whole-model logits from a list of fp64 tensors in canonical order."""
    h = embed(tokens, w64[0], w64[1])
    for l in range(cfg.n_layers):
        ids = cfg.block_ids(l)
        p = {name: w64[i] for name, i in zip(BLOCK_TENSORS, ids)}
        h = block_forward(h, p, cfg.n_heads, cfg.ln_eps)
    g_id, b_id = cfg.head_ids()
    return head_logits(h, w64[g_id], w64[b_id], w64[0], cfg.ln_eps)


def loss(cfg, w64, tokens):
    return next_token_loss(logits_of(cfg, w64, tokens), tokens)


def loss_of_storage(cfg, theta, tokens):
    return loss(cfg, [widen(t, cfg.dtype) for t in theta], tokens)


# --------------------------------------------------------------------------
# the step
# --------------------------------------------------------------------------
def projected_gradient(l_plus, l_minus, eps):
    """Eq. 1, in fp64, with eps the fp32 value the perturbation used."""
    return (l_plus - l_minus) / (2.0 * float(np.float32(eps)))


def step_scalar(lr, g):
    """The fp32 scalar multiplying z in Eq. 2: -(lr * g), formed in fp64, rounded once."""
    return np.float32(-(float(np.float32(lr)) * g))


def perturb_all(cfg, theta, seed, scale, ids=None, stochastic=False):
    """Alg. 1 PerturbParameters over the tensors `ids` (all by default), in place."""
    for t in (range(cfg.n_tensors) if ids is None else ids):
        axpy_z(theta[t], cfg.dtype, seed, t, scale, out=theta[t], stochastic=stochastic)


def zo_step_literal(cfg, theta, tokens, seed, eps, lr):
    """Alg. 1 body.  `theta` (list of storage arrays) is modified in place.
    Returns (l_plus, l_minus, g)."""
    perturb_all(cfg, theta, seed, eps)
    l_plus = loss_of_storage(cfg, theta, tokens)
    perturb_all(cfg, theta, seed, -2.0 * np.float32(eps))
    l_minus = loss_of_storage(cfg, theta, tokens)
    perturb_all(cfg, theta, seed, eps)
    g = projected_gradient(l_plus, l_minus, eps)
    perturb_all(cfg, theta, seed, step_scalar(lr, g))
    return l_plus, l_minus, g


def perturbed_pair(cfg, theta, seed, eps):
    plus = [axpy_z(t, cfg.dtype, seed, i, eps) for i, t in enumerate(theta)]
    minus = [axpy_z(t, cfg.dtype, seed, i, -np.float32(eps)) for i, t in enumerate(theta)]
    return plus, minus


def dual_loss_fused(cfg, theta, tokens, seed, eps):
    plus, minus = perturbed_pair(cfg, theta, seed, eps)
    return loss_of_storage(cfg, plus, tokens), loss_of_storage(cfg, minus, tokens)


def zo_step_fused(cfg, theta, tokens, seed, eps, lr, stochastic_update=False):
    """Same step with theta untouched by the perturbation: W+- = rn(theta +- eps z).
    `stochastic_update` rounds the update of Eq. 2 (and only it) stochastically."""
    l_plus, l_minus = dual_loss_fused(cfg, theta, tokens, seed, eps)
    g = projected_gradient(l_plus, l_minus, eps)
    perturb_all(cfg, theta, seed, step_scalar(lr, g), stochastic=stochastic_update)
    return l_plus, l_minus, g


class Alg2Runner:
    """Alg. 2: per-module DualForward with the update of the previous step
    deferred to the module's next visit.  `literal=True` perturbs in place
    (+eps, -2 eps, +eps) as printed; `literal=False` forms W+- out of place.
    The pending update is tracked by an explicit flag rather than by g != 0,
    and `flush()` applies the one left after the last step (as printed, the
    algorithm never applies it)."""

    def __init__(self, cfg, theta, eps, lr, literal=False):
        self.cfg, self.theta, self.eps, self.lr, self.literal = cfg, theta, eps, lr, literal
        self.pending = None   # (seed, scalar)

    def _dual(self, ids, update_ids, seed, fn, in_plus, in_minus):
        cfg, th = self.cfg, self.theta
        if self.pending is not None:
            perturb_all(cfg, th, self.pending[0], self.pending[1], update_ids)
        if self.literal:
            perturb_all(cfg, th, seed, self.eps, ids)
            out_plus = fn([widen(th[i], cfg.dtype) for i in ids], in_plus)
            perturb_all(cfg, th, seed, -2.0 * np.float32(self.eps), ids)
            out_minus = fn([widen(th[i], cfg.dtype) for i in ids], in_minus)
            perturb_all(cfg, th, seed, self.eps, ids)
        else:
            wp = [widen(axpy_z(th[i], cfg.dtype, seed, i, self.eps), cfg.dtype) for i in ids]
            wm = [widen(axpy_z(th[i], cfg.dtype, seed, i, -np.float32(self.eps)), cfg.dtype) for i in ids]
            out_plus, out_minus = fn(wp, in_plus), fn(wm, in_minus)
        return out_plus, out_minus

    def step(self, tokens, seed):
        cfg = self.cfg
        hp, hm = self._dual([0, 1], [0, 1], seed, lambda w, x: embed(x, w[0], w[1]), tokens, tokens)
        for l in range(cfg.n_layers):
            ids = cfg.block_ids(l)
            fn = lambda w, x: block_forward(x, dict(zip(BLOCK_TENSORS, w)), cfg.n_heads, cfg.ln_eps)
            hp, hm = self._dual(ids, ids, seed, fn, hp, hm)
        # LM head: final LayerNorm plus the tied embedding matrix, which was
        # already updated at its first visit and is only perturbed here.
        hid = cfg.head_ids()
        fn = lambda w, x: head_logits(x, w[0], w[1], w[2], cfg.ln_eps)
        lp, lm = self._dual(hid + [0], hid, seed, fn, hp, hm)
        l_plus, l_minus = next_token_loss(lp, tokens), next_token_loss(lm, tokens)
        g = projected_gradient(l_plus, l_minus, self.eps)
        self.pending = (seed, step_scalar(self.lr, g))
        return l_plus, l_minus, g

    def flush(self):
        if self.pending is not None:
            perturb_all(self.cfg, self.theta, self.pending[0], self.pending[1])
            self.pending = None

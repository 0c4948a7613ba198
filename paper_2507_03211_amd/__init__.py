"""Thin ctypes binding over libzo.so (include/zo.h): argument marshalling only.

Every function here has the name and argument order of the C entry point it
calls.  Pointer arguments accept torch tensors (their data_ptr() is passed),
ints (raw addresses) or None (NULL); `stream` arguments accept a
torch.cuda.Stream, an int or None.  A non-zero status raises ZoError carrying
zo_last_error().  There is no fallback: if the HIP library has not been built
(python -m paper_2507_03211_amd.build) importing any entry point fails loudly.
"""
import ctypes
import os

ZO_OK, ZO_EINVAL, ZO_ENOMEM, ZO_EHIP, ZO_ESTATE = 0, 1, 2, 3, 4
ZO_FP32, ZO_BF16, ZO_FP16 = 0, 1, 2
ZO_RESIDENT, ZO_STREAMED = 0, 1
ZO_MODE_LITERAL, ZO_MODE_FUSED = 0, 1
ZO_PHASE_PREFETCH, ZO_PHASE_COMPUTE, ZO_PHASE_WRITEBACK = 1, 2, 4
ZO_ROUND_NEAREST, ZO_ROUND_STOCHASTIC = 0, 1

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "libzo.so")

EXPORTS = (
    "zo_workspace_bytes", "zo_init_model", "zo_perturb", "zo_dual_forward", "zo_step", "zo_stream_block",
    "zo_stream_begin", "zo_stream_end", "zo_flush_pending", "zo_set_writeback_interval", "zo_set_stream_lookahead", "zo_set_deferred_update", "zo_set_update_rounding", "zo_device_flags", "zo_free",
    "zo_last_error", "zo_profile_begin", "zo_profile_end", "zo_profile_spans",
    "zo_kernel_z", "zo_kernel_normal_pairs", "zo_kernel_axpy_z", "zo_kernel_axpy_z_sr", "zo_kernel_stage_pm", "zo_kernel_stage_update_pm", "zo_kernel_linear_pm",
    "zo_kernel_layernorm_pm", "zo_kernel_attention", "zo_kernel_lmhead_scratch_bytes", "zo_kernel_lmhead_ce",
    "zo_kernel_lmhead_ce_noalloc",
)


class ZoError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("libzo status %d: %s" % (status, message))
        self.status = status


class zo_config(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32),
                ("d_ffn", ctypes.c_int32), ("vocab", ctypes.c_int32), ("max_pos", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("residency", ctypes.c_int32), ("ln_eps", ctypes.c_float)]


_lib = None


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libzo.so is missing at %s: build it with `python -m paper_2507_03211_amd.build`" % _LIB_PATH)
        L = ctypes.CDLL(_LIB_PATH)
        vp, u64, u32, i32, f32, sz = (ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_float,
                                      ctypes.c_size_t)
        cfgp = ctypes.POINTER(zo_config)
        L.zo_last_error.restype = ctypes.c_char_p
        L.zo_last_error.argtypes = []
        L.zo_workspace_bytes.restype = sz
        L.zo_workspace_bytes.argtypes = [cfgp, i32, i32]
        L.zo_init_model.argtypes = [cfgp, ctypes.POINTER(vp), i32, vp, sz, i32, i32, vp, vp, ctypes.POINTER(vp)]
        L.zo_perturb.argtypes = [vp, u64, f32, i32, i32]
        L.zo_dual_forward.argtypes = [vp, vp, i32, i32, u64, f32, i32, vp, vp]
        L.zo_step.argtypes = [vp, vp, i32, i32, u64, f32, f32, i32, vp, vp]
        L.zo_stream_block.argtypes = [vp, i32, i32]
        L.zo_stream_begin.argtypes = [vp, vp, i32, i32, u64, f32]
        L.zo_stream_end.argtypes = [vp, f32, vp, vp]
        L.zo_flush_pending.argtypes = [vp]
        L.zo_set_update_rounding.argtypes = [vp, i32]
        L.zo_set_writeback_interval.argtypes = [vp, i32]
        L.zo_set_stream_lookahead.argtypes = [vp, i32]
        L.zo_set_deferred_update.argtypes = [vp, i32]
        L.zo_device_flags.argtypes = [vp, ctypes.POINTER(u32)]
        L.zo_free.argtypes = [vp]
        L.zo_profile_begin.argtypes = [vp, i32]
        L.zo_profile_end.argtypes = [vp, vp, vp, vp]
        L.zo_profile_spans.argtypes = [vp, i32, vp, vp, vp, vp, vp]
        L.zo_kernel_z.argtypes = [vp, u64, u64, u32, u64, vp]
        L.zo_kernel_normal_pairs.argtypes = [vp, vp, u64, vp]
        L.zo_kernel_axpy_z.argtypes = [vp, vp, i32, u64, u64, u32, f32, vp, vp]
        L.zo_kernel_axpy_z_sr.argtypes = [vp, vp, i32, u64, u64, u32, f32, vp, vp]
        L.zo_kernel_stage_pm.argtypes = [vp, vp, vp, i32, i32, i32, i32, u64, u32, f32, vp]
        L.zo_kernel_stage_update_pm.argtypes = [vp, vp, vp, i32, i32, i32, i32, u64, u32, f32, u64, vp, i32, vp]
        L.zo_kernel_linear_pm.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]
        L.zo_kernel_layernorm_pm.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, vp]
        L.zo_kernel_attention.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        L.zo_kernel_lmhead_scratch_bytes.restype = sz
        L.zo_kernel_lmhead_scratch_bytes.argtypes = [i32, i32, i32]
        L.zo_kernel_lmhead_ce.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]
        L.zo_kernel_lmhead_ce_noalloc.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]
        _lib = L
    return _lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    raise TypeError("expected a tensor, an address or None, got %r" % type(x))


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def _check(status):
    if status != ZO_OK:
        raise ZoError(status, lib().zo_last_error().decode("utf-8", "replace"))


def zo_last_error():
    return lib().zo_last_error().decode("utf-8", "replace")


def make_config(n_layers, d_model, n_heads, d_ffn, vocab, max_pos, dtype, residency=ZO_RESIDENT, ln_eps=1e-5):
    return zo_config(n_layers, d_model, n_heads, d_ffn, vocab, max_pos, dtype, residency, ln_eps)


def zo_workspace_bytes(cfg, batch, seq):
    return int(lib().zo_workspace_bytes(ctypes.byref(cfg), batch, seq))


def zo_init_model(cfg, tensor_ptrs, workspace, workspace_bytes, batch, seq, compute_stream=None, copy_stream=None):
    """Returns the opaque model handle (an int address)."""
    arr = (ctypes.c_void_p * len(tensor_ptrs))(*[_ptr(t) for t in tensor_ptrs])
    out = ctypes.c_void_p()
    _check(lib().zo_init_model(ctypes.byref(cfg), arr, len(tensor_ptrs), _ptr(workspace), workspace_bytes, batch, seq,
                               _stream(compute_stream), _stream(copy_stream), ctypes.byref(out)))
    return out.value


def zo_perturb(model, seed, scale, first_tensor, n_tensors):
    _check(lib().zo_perturb(model, seed, scale, first_tensor, n_tensors))


def zo_dual_forward(model, tokens, batch, seq, seed, eps, mode=ZO_MODE_FUSED, dev_loss_pm=None, want_host=True):
    """Returns (l_plus, l_minus) when want_host (synchronises), else None."""
    host = (ctypes.c_double * 2)() if want_host else None
    _check(lib().zo_dual_forward(model, _ptr(tokens), batch, seq, seed, eps, mode, _ptr(dev_loss_pm),
                                 ctypes.addressof(host) if want_host else None))
    return (host[0], host[1]) if want_host else None


def zo_step(model, tokens, batch, seq, seed, eps, lr, mode=ZO_MODE_FUSED, want_host=True):
    """Returns (l_plus, l_minus, g) when want_host (synchronises), else None."""
    g = ctypes.c_double() if want_host else None
    host = (ctypes.c_double * 2)() if want_host else None
    _check(lib().zo_step(model, _ptr(tokens), batch, seq, seed, eps, lr, mode,
                         ctypes.addressof(g) if want_host else None, ctypes.addressof(host) if want_host else None))
    return (host[0], host[1], g.value) if want_host else None


def zo_stream_begin(model, tokens, batch, seq, seed, eps):
    _check(lib().zo_stream_begin(model, _ptr(tokens), batch, seq, seed, eps))


def zo_stream_block(model, block, phase_flags):
    _check(lib().zo_stream_block(model, block, phase_flags))


def zo_stream_end(model, lr, want_host=True):
    g = ctypes.c_double() if want_host else None
    host = (ctypes.c_double * 2)() if want_host else None
    _check(lib().zo_stream_end(model, lr, ctypes.addressof(g) if want_host else None,
                               ctypes.addressof(host) if want_host else None))
    return (host[0], host[1], g.value) if want_host else None


def zo_flush_pending(model):
    _check(lib().zo_flush_pending(model))


def zo_set_stream_lookahead(handle, steps):
    _check(lib().zo_set_stream_lookahead(handle, steps))


def zo_set_writeback_interval(model, steps):
    _check(lib().zo_set_writeback_interval(model, steps))


def zo_set_deferred_update(model, on):
    _check(lib().zo_set_deferred_update(model, int(on)))


def zo_set_update_rounding(model, mode):
    _check(lib().zo_set_update_rounding(model, mode))


def zo_device_flags(model):
    v = ctypes.c_uint32()
    _check(lib().zo_device_flags(model, ctypes.byref(v)))
    return v.value


ZO_K_NAMES = ("linear", "attention", "stage", "update", "norm", "ce", "other")


def zo_profile_begin(model, max_launches):
    _check(lib().zo_profile_begin(model, max_launches))


def zo_profile_end(model):
    """Returns {class name: (milliseconds, launches, algorithmic work)}."""
    n = len(ZO_K_NAMES)
    ms, cnt, work = (ctypes.c_double * n)(), (ctypes.c_uint64 * n)(), (ctypes.c_double * n)()
    _check(lib().zo_profile_end(model, ctypes.addressof(ms), ctypes.addressof(cnt), ctypes.addressof(work)))
    return {ZO_K_NAMES[i]: (ms[i], int(cnt[i]), work[i]) for i in range(n)}


ZO_SPAN_UPLOAD, ZO_SPAN_COMPUTE, ZO_SPAN_WRITEBACK = 0, 1, 2


def zo_profile_spans(model, max_spans=4096):
    """Returns a list of (kind, block, start_ms, end_ms)."""
    kind, block = (ctypes.c_int32 * max_spans)(), (ctypes.c_int32 * max_spans)()
    t0, t1 = (ctypes.c_double * max_spans)(), (ctypes.c_double * max_spans)()
    n = ctypes.c_int()
    _check(lib().zo_profile_spans(model, max_spans, ctypes.addressof(kind), ctypes.addressof(block), ctypes.addressof(t0),
                                  ctypes.addressof(t1), ctypes.addressof(n)))
    return [(int(kind[i]), int(block[i]), t0[i], t1[i]) for i in range(n.value)]


def zo_free(model):
    _check(lib().zo_free(model))


def zo_kernel_z(out, n, seed, tensor_id, first=0, stream=None):
    _check(lib().zo_kernel_z(_ptr(out), n, seed, tensor_id, first, _stream(stream)))


def zo_kernel_normal_pairs(words, z, n_pairs, stream=None):
    _check(lib().zo_kernel_normal_pairs(_ptr(words), _ptr(z), n_pairs, _stream(stream)))


def zo_kernel_axpy_z(src, dst, dtype, n, seed, tensor_id, scale, dev_scale=None, stream=None):
    _check(lib().zo_kernel_axpy_z(_ptr(src), _ptr(dst), dtype, n, seed, tensor_id, scale, _ptr(dev_scale), _stream(stream)))


def zo_kernel_axpy_z_sr(src, dst, dtype, n, seed, tensor_id, scale, dev_scale=None, stream=None):
    _check(lib().zo_kernel_axpy_z_sr(_ptr(src), _ptr(dst), dtype, n, seed, tensor_id, scale, _ptr(dev_scale), _stream(stream)))


def zo_kernel_stage_pm(theta, w_plus, w_minus, dtype, rows, cols, transpose, seed, tensor_id, eps, stream=None):
    _check(lib().zo_kernel_stage_pm(_ptr(theta), _ptr(w_plus), _ptr(w_minus), dtype, rows, cols, int(transpose), seed,
                                    tensor_id, eps, _stream(stream)))


def zo_kernel_stage_update_pm(theta, w_plus, w_minus, dtype, rows, cols, transpose, seed, tensor_id, eps, upd_seed, dev_scale,
                              stochastic=False, stream=None):
    _check(lib().zo_kernel_stage_update_pm(_ptr(theta), _ptr(w_plus), _ptr(w_minus), dtype, rows, cols, int(transpose), seed,
                                           tensor_id, eps, upd_seed, _ptr(dev_scale), int(stochastic), _stream(stream)))


def zo_kernel_linear_pm(x, wt_plus, wt_minus, b_plus, b_minus, y, dtype, m_half, n, k, epilogue, stream=None):
    _check(lib().zo_kernel_linear_pm(_ptr(x), _ptr(wt_plus), _ptr(wt_minus), _ptr(b_plus), _ptr(b_minus), _ptr(y), dtype,
                                     m_half, n, k, epilogue, _stream(stream)))


def zo_kernel_layernorm_pm(resid, g_plus, g_minus, b_plus, b_minus, y, dtype, m_half, d, ln_eps, stream=None):
    _check(lib().zo_kernel_layernorm_pm(_ptr(resid), _ptr(g_plus), _ptr(g_minus), _ptr(b_plus), _ptr(b_minus), _ptr(y),
                                        dtype, m_half, d, ln_eps, _stream(stream)))


def zo_kernel_attention(qkv, out, dtype, n_seq, seq, n_heads, d_head, stream=None):
    _check(lib().zo_kernel_attention(_ptr(qkv), _ptr(out), dtype, n_seq, seq, n_heads, d_head, _stream(stream)))


def zo_kernel_lmhead_scratch_bytes(dtype, m_half, vocab):
    return int(lib().zo_kernel_lmhead_scratch_bytes(dtype, m_half, vocab))


def zo_kernel_lmhead_ce(x, e_plus, e_minus, target, row_loss, scratch, dtype, m_half, d, vocab, stream=None):
    _check(lib().zo_kernel_lmhead_ce(_ptr(x), _ptr(e_plus), _ptr(e_minus), _ptr(target), _ptr(row_loss), _ptr(scratch),
                                     dtype, m_half, d, vocab, _stream(stream)))


ZO_NOALLOC_SCRATCH_BYTES = 32 << 20


def zo_kernel_lmhead_ce_noalloc(x, e_plus, e_minus, target, row_loss, dtype, m_half, d, vocab, stream=None):
    _check(lib().zo_kernel_lmhead_ce_noalloc(_ptr(x), _ptr(e_plus), _ptr(e_minus), _ptr(target), _ptr(row_loss),
                                             dtype, m_half, d, vocab, _stream(stream)))

"""Helpers for the GPU parity tests: moving the shared synthetic inputs onto the device and
building a model handle over them.  No arithmetic of the method lives here."""
import numpy as np
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from oracle import zo_oracle as zo

DEV = "cuda:0"


def to_dev(arr, dtype):
    """Storage numpy array -> device tensor of the matching torch dtype."""
    if dtype == zi.BF16:
        return torch.from_numpy(arr.view(np.int16).copy()).view(torch.bfloat16).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(arr)).to(DEV)


def to_host(t, dtype):
    """Device tensor -> storage numpy array (uint16 bits for bf16)."""
    t = t.detach().cpu().contiguous()
    if dtype == zi.BF16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def act_to_dev(x64, dtype):
    """fp64 activations -> the activation type of a precision (fp64 for fp32 parameters)."""
    t = torch.from_numpy(np.ascontiguousarray(x64))
    if dtype == zi.FP32:
        return t.to(DEV)
    return t.to(torch.bfloat16 if dtype == zi.BF16 else torch.float16).to(DEV)


def act_dtype(dtype):
    return {zi.FP32: torch.float64, zi.BF16: torch.bfloat16, zi.FP16: torch.float16}[dtype]


def resid_dtype(dtype):
    return torch.float64 if dtype == zi.FP32 else torch.float32


class Model:
    """A resident or streamed model over seeded synthetic weights.  `device_blocks`: blocks of a streamed model
    that are kept in device memory instead of pinned host memory."""

    def __init__(self, n_layers, d_model, n_heads, d_ffn, vocab, max_pos, dtype, batch, seq, seed=0, plain_small=False,
                 std=0.02, streamed=False, device_blocks=()):
        self.dtype, self.batch, self.seq = dtype, batch, seq
        self.ocfg = zo.Config(n_layers, d_model, n_heads, d_ffn, vocab, max_pos, dtype)
        self.theta0 = zi.make_weights(self.ocfg.shapes(), dtype, seed=seed, std=std, plain_small=plain_small)
        self.cfg = zo_amd.make_config(n_layers, d_model, n_heads, d_ffn, vocab, max_pos, dtype,
                                      zo_amd.ZO_STREAMED if streamed else zo_amd.ZO_RESIDENT)
        self.streamed = streamed
        self.compute = torch.cuda.Stream(device=DEV)
        self.copy = torch.cuda.Stream(device=DEV) if streamed else None
        if not streamed:
            self.tensors = [to_dev(t, dtype) for t in self.theta0]
            ptrs = self.tensors
        else:
            tdt = act_dtype(dtype) if dtype != zi.FP32 else torch.float32
            per_block = sum(int(np.prod(s)) for _, s in self.ocfg.shapes()[2:18])
            self.host_blocks = torch.empty((n_layers, per_block), dtype=tdt, pin_memory=True)
            self.tensors, ptrs = [], []
            esz = self.host_blocks.element_size()
            for i, t in enumerate(self.theta0):
                if 2 <= i < 2 + 16 * n_layers and (i - 2) // 16 not in device_blocks:
                    l, k = divmod(i - 2, 16)
                    off = sum(int(np.prod(s)) for _, s in self.ocfg.shapes()[2:2 + k])
                    view = self.host_blocks[l, off:off + t.size]
                    src = torch.from_numpy(t.view(np.int16).copy()).view(torch.bfloat16) if dtype == zi.BF16 else torch.from_numpy(t.copy())
                    view.copy_(src.reshape(-1))
                    self.tensors.append(view)
                    ptrs.append(self.host_blocks.data_ptr() + (l * per_block + off) * esz)
                else:
                    self.tensors.append(to_dev(t, dtype))
                    ptrs.append(self.tensors[-1])
        nbytes = zo_amd.zo_workspace_bytes(self.cfg, batch, seq)
        assert nbytes > 0
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        torch.cuda.synchronize()
        self.handle = zo_amd.zo_init_model(self.cfg, ptrs, self.workspace, nbytes, batch, seq, self.compute, self.copy)

    def theta(self):
        torch.cuda.synchronize()
        return [to_host(t, self.dtype).reshape(s) for t, (_, s) in zip(self.tensors, self.ocfg.shapes())]

    def tokens(self, seed=1, batch=None, seq=None):
        tok = zi.make_tokens(batch or self.batch, seq or self.seq, self.ocfg.vocab, seed=seed)
        return tok, torch.from_numpy(tok).to(DEV)

    def close(self):
        if self.handle:
            zo_amd.zo_free(self.handle)
            self.handle = None

"""The C-ABI boundary, checked without a GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2507_03211_amd as zo_amd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "zo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zo_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert "zo_init_model" in names and "zo_stream_block" in names and len(names) >= 15
    L = zo_amd.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(zo_amd.EXPORTS) == names
    for n in names:                       # the binding carries the same names
        assert hasattr(zo_amd, n), n


def test_host_side_argument_checks():
    good = zo_amd.make_config(2, 64, 4, 256, 512, 32, zo_amd.ZO_FP32)
    assert zo_amd.zo_workspace_bytes(good, 2, 32) > 0
    assert zo_amd.zo_workspace_bytes(good, 2, 33) == 0                     # seq > max_pos
    assert zo_amd.zo_workspace_bytes(zo_amd.make_config(2, 64, 5, 256, 512, 32, 0), 2, 32) == 0   # heads do not divide d
    assert zo_amd.zo_workspace_bytes(zo_amd.make_config(2, 60, 4, 256, 512, 32, 0), 2, 32) == 0   # d not a multiple of 8
    assert zo_amd.zo_workspace_bytes(zo_amd.make_config(2, 64, 4, 256, 512, 32, 7), 2, 32) == 0   # unknown dtype
    L = zo_amd.lib()
    out = ctypes.c_void_p()
    ptrs = (ctypes.c_void_p * 36)(*([4096] * 36))
    st = L.zo_init_model(ctypes.byref(good), ptrs, 35, 4096, 1 << 30, 2, 32, None, None, ctypes.byref(out))
    assert st == zo_amd.ZO_EINVAL and "tensors" in zo_amd.zo_last_error()
    st = L.zo_init_model(ctypes.byref(good), ptrs, 36, 4096 + 256, 16, 2, 32, None, None, ctypes.byref(out))
    assert st == zo_amd.ZO_ENOMEM
    st = L.zo_init_model(ctypes.byref(good), None, 36, 4096, 1 << 30, 2, 32, None, None, ctypes.byref(out))
    assert st == zo_amd.ZO_EINVAL
    streamed = zo_amd.make_config(2, 64, 4, 256, 512, 32, 0, zo_amd.ZO_STREAMED)
    st = L.zo_init_model(ctypes.byref(streamed), ptrs, 36, 4096 + 256, 1 << 30, 2, 32, None, None, ctypes.byref(out))
    assert st == zo_amd.ZO_EINVAL and "copy stream" in zo_amd.zo_last_error()
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_perturb(None, 1, 1e-3, 0, 1)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_kernel_axpy_z(4096, 4096, 9, 16, 1, 0, 1e-3)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_kernel_axpy_z_sr(4096, 4096, zo_amd.ZO_FP32, 16, 1, 0, 1e-3)   # nothing to round stochastically in fp32
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_update_rounding(None, zo_amd.ZO_ROUND_STOCHASTIC)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_kernel_stage_pm(4096, 4096, 4096, 0, 8, 6, 1, 1, 0, 1e-3)     # transposed, cols % 4 != 0
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_kernel_stage_update_pm(4096, 4096, 4096, zo_amd.ZO_BF16, 8, 8, 0, 1, 0, 1e-3, 2, None)     # no step scalar
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_kernel_stage_update_pm(4096, 4096, 4096, zo_amd.ZO_FP32, 8, 8, 0, 1, 0, 1e-3, 2, 4096, True)   # fp32 + stochastic
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_set_deferred_update(None, 1)
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_kernel_lmhead_ce_noalloc(None, 4096, 4096, 4096, 4096, zo_amd.ZO_BF16, 8, 64, 512)      # NULL input
    with pytest.raises(zo_amd.ZoError):
        zo_amd.zo_kernel_lmhead_ce_noalloc(4096, 4096, 4096, 4096, 4096, zo_amd.ZO_BF16, 8, 60, 512)      # d not a multiple of 8
    assert zo_amd.zo_free(None) is None


def test_bench_refuses_more_than_one_gpu():
    """One GPU is the whole target: `bench.py --gpus N` with N > 1 says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "--gpus 1" in r.stderr and r.stdout.strip() == ""

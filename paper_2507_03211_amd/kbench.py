"""Per-kernel timing at real shapes through the kernel-level C-ABI entry points.

    python -m paper_2507_03211_amd.kbench linear --m-half 8192 --n 20480 --k 5120 --epilogue 1
    python -m paper_2507_03211_amd.kbench attention --n-seq 8 --seq 2048 --heads 40 --d-head 128
    python -m paper_2507_03211_amd.kbench axpy --n 314572800 --dtype bf16
    python -m paper_2507_03211_amd.kbench stage --rows 5120 --cols 20480 --transpose 1
    python -m paper_2507_03211_amd.kbench mfma-rate --dtype bf16

`mfma-rate` is no kernel of the path: it issues nothing but matrix multiplies, once on zeros and once on operands of
random sign and mantissa, and prints both rates: the second is what the chip sustains under its power limit and is
the ceiling the GEMM's fraction of the nominal peak has to be read against.

Prints one JSON line per run: milliseconds per launch (HIP events on the launch stream) and the
achieved rate against the roofline that bounds the kernel (bf16/fp16 MFMA 2.5 PFLOP/s, HBM 8 TB/s).
Inputs are random device tensors; nothing is checked here (the parity tests do that).
"""
import argparse
import json

import torch

import paper_2507_03211_amd as zo

DT = {"f32": (zo.ZO_FP32, torch.float32), "bf16": (zo.ZO_BF16, torch.bfloat16), "f16": (zo.ZO_FP16, torch.float16)}


def timed(fn, reps, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("kernel", choices=["linear", "attention", "axpy", "stage", "layernorm", "mfma-rate"])
    ap.add_argument("--dtype", default="bf16", choices=list(DT))
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--m-half", type=int, default=8192)
    ap.add_argument("--n", type=int, default=5120)
    ap.add_argument("--k", type=int, default=5120)
    ap.add_argument("--epilogue", type=int, default=0)
    ap.add_argument("--n-seq", type=int, default=8)
    ap.add_argument("--seq", type=int, default=2048)
    ap.add_argument("--heads", type=int, default=40)
    ap.add_argument("--d-head", type=int, default=128)
    ap.add_argument("--rows", type=int, default=5120)
    ap.add_argument("--cols", type=int, default=5120)
    ap.add_argument("--transpose", type=int, default=1)
    ap.add_argument("--workgroups", type=int, default=1024, help="mfma-rate: workgroups of 4 waves")
    ap.add_argument("--iters", type=int, default=20000, help="mfma-rate: 16 multiplies per wave and iteration")
    ap.add_argument("--operands", default="random", choices=["random", "zero"],
                    help="linear: all-zero operands take the chip's power limit out of the timing (what is left is the kernel's own stalls)")
    ap.add_argument("--stochastic", action="store_true", help="axpy: the stochastically rounded update (16-bit types)")
    a = ap.parse_args()
    code, tdt = DT[a.dtype]
    dev = "cuda:0"
    esz = torch.empty(0, dtype=tdt).element_size()
    out = {"kernel": a.kernel, "dtype": a.dtype}
    if a.kernel == "linear":
        act = torch.float64 if code == zo.ZO_FP32 else tdt
        scale = 0.0 if a.operands == "zero" else 1.0
        x = (scale * torch.randn(2 * a.m_half, a.k, device=dev)).to(act)
        w = [(0.02 * scale * torch.randn(a.n, a.k, device=dev)).to(tdt) for _ in range(2)]
        b = [torch.zeros(a.n, device=dev, dtype=tdt) for _ in range(2)]
        ydt = act if a.epilogue in (0, 1) else (torch.float64 if code == zo.ZO_FP32 else torch.float32)
        y = torch.zeros(2 * a.m_half, a.n, device=dev, dtype=ydt)
        ms = timed(lambda: zo.zo_kernel_linear_pm(x, w[0], w[1], b[0], b[1], y, code, a.m_half, a.n, a.k, a.epilogue), a.reps)
        flops = 2.0 * 2 * a.m_half * a.n * a.k
        out.update(shape=[2 * a.m_half, a.n, a.k], epilogue=a.epilogue, operands=a.operands, ms=ms, tflops=flops / ms / 1e9,
                   frac_of_peak=flops / ms / 1e9 / 2500.0)
    elif a.kernel == "attention":
        d = a.heads * a.d_head
        qkv = torch.randn(a.n_seq * a.seq, 3 * d, device=dev).to(tdt if code != zo.ZO_FP32 else torch.float64)
        o = torch.empty(a.n_seq * a.seq, d, device=dev, dtype=qkv.dtype)
        ms = timed(lambda: zo.zo_kernel_attention(qkv, o, code, a.n_seq, a.seq, a.heads, a.d_head), a.reps)
        flops = 2.0 * a.n_seq * a.heads * a.seq * (a.seq + 1) * a.d_head
        out.update(shape=[a.n_seq, a.seq, a.heads, a.d_head], ms=ms, tflops=flops / ms / 1e9, frac_of_peak=flops / ms / 1e9 / 2500.0)
    elif a.kernel == "axpy":
        t = (0.02 * torch.randn(a.n, device=dev)).to(tdt)
        fn = zo.zo_kernel_axpy_z_sr if a.stochastic else zo.zo_kernel_axpy_z
        ms = timed(lambda: fn(t, t, code, a.n, 1, 2, 1e-3), a.reps)
        out["rounding"] = "stochastic" if a.stochastic else "nearest"
        gb = 2.0 * a.n * esz / 1e9
        out.update(n=a.n, ms=ms, gbs=gb / (ms * 1e-3), frac_of_hbm=gb / (ms * 1e-3) / 8000.0, gelem_per_s=a.n / ms / 1e6)
    elif a.kernel == "stage":
        t = (0.02 * torch.randn(a.rows, a.cols, device=dev)).to(tdt)
        wp, wm = torch.empty_like(t), torch.empty_like(t)
        ms = timed(lambda: zo.zo_kernel_stage_pm(t, wp, wm, code, a.rows, a.cols, a.transpose, 1, 2, 1e-3), a.reps)
        gb = 3.0 * a.rows * a.cols * esz / 1e9
        out.update(shape=[a.rows, a.cols], transpose=a.transpose, ms=ms, gbs=gb / (ms * 1e-3), frac_of_hbm=gb / (ms * 1e-3) / 8000.0,
                   gelem_per_s=a.rows * a.cols / ms / 1e6)
    elif a.kernel == "mfma-rate":
        if code == zo.ZO_FP32:
            raise SystemExit("mfma-rate issues 16-bit multiplies: --dtype bf16 or f16")
        sink = torch.empty(a.workgroups * 256, device=dev, dtype=torch.float32)
        flops = a.workgroups * 4.0 * a.iters * 16 * 2 * 32 * 32 * 16
        out.update(workgroups=a.workgroups, iters=a.iters)
        for name, rnd in (("zero_operands", False), ("random_operands", True)):
            ms = timed(lambda: zo.zo_probe_mfma_rate(sink, code, a.workgroups, a.iters, rnd), a.reps)
            out[name] = {"ms": ms, "tflops": flops / ms / 1e9, "frac_of_peak": flops / ms / 1e9 / 2500.0}
    else:
        rdt = torch.float64 if code == zo.ZO_FP32 else torch.float32
        adt = torch.float64 if code == zo.ZO_FP32 else tdt
        h = torch.randn(2 * a.m_half, a.n, device=dev, dtype=rdt)
        g = [torch.ones(a.n, device=dev, dtype=tdt) for _ in range(2)]
        b = [torch.zeros(a.n, device=dev, dtype=tdt) for _ in range(2)]
        y = torch.empty(2 * a.m_half, a.n, device=dev, dtype=adt)
        ms = timed(lambda: zo.zo_kernel_layernorm_pm(h, g[0], g[1], b[0], b[1], y, code, a.m_half, a.n, 1e-5), a.reps)
        gb = 2.0 * a.m_half * a.n * (h.element_size() + y.element_size()) / 1e9
        out.update(shape=[2 * a.m_half, a.n], ms=ms, gbs=gb / (ms * 1e-3), frac_of_hbm=gb / (ms * 1e-3) / 8000.0)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Throughput of the ZO-SGD step (dual +-eps z forward + update) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config opt-13b]

A step is one zo_step through the C-ABI: stage W+- = rn(theta +- eps z) block by block, the
sign-batched forward of both perturbed models, g, and the regenerated-z update of every
parameter.  Inputs (weights ~ 0.02 N(0,1) drawn on the device by torch, uniform random
tokens) are resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f64": 78.6}
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 20; 3 for the streamed configuration)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default 3; 1 streamed)")
    ap.add_argument("--batch", type=int, default=None, help="override the configuration's batch size")
    ap.add_argument("--seq", type=int, default=None, help="override the configuration's sequence length (longer-context variants)")
    ap.add_argument("--config", default="opt-13b", help="tiny | opt-125m | opt-1.3b | opt-13b | opt-175b (streamed)")
    ap.add_argument("--host-blocks", type=int, default=6,
                    help="streamed configs: number of distinct real-shape pinned host blocks; the layers cycle through them "
                         "(the full 175B model needs 348 GB of pinned memory, more than a box may pin)")
    ap.add_argument("--hbm-blocks", type=int, default=0,
                    help="streamed configs: keep this many of the blocks in device memory (each with memory of its own), spread "
                         "evenly between the ones that are uploaded from pinned host memory for every visit; 0 = the paper's "
                         "configuration, every block streamed")
    ap.add_argument("--mode", default="fused", choices=["fused", "literal"],
                    help="fused: W+- = rn(theta +- eps z) staged, theta untouched, both signs in one batched pass (default); "
                         "literal: Alg. 1 as printed, theta perturbed in place (+eps, -2 eps, +eps) with one forward after each "
                         "of the first two (resident configurations only)")
    ap.add_argument("--writeback-interval", type=int, default=1,
                    help="streamed configuration: write the updated blocks back to the host every K-th step (1 = every step, "
                         "the paper's schedule)")
    ap.add_argument("--stochastic-update", action="store_true",
                    help="round the update of Eq. 2 stochastically into the 16-bit storage type (opt-in variant)")
    ap.add_argument("--update", default="deferred", choices=["deferred", "immediate"],
                    help="resident fused mode: 'deferred' applies a step's update inside the next step's staging pass (Alg. 2's "
                         "order; the last one is flushed inside the timed region), 'immediate' in a pass of its own at the end "
                         "of the step; theta ends up bit-identical either way")
    ap.add_argument("--lookahead", type=int, default=0, choices=[0, 1],
                    help="streamed configuration: steps the host may run ahead of the device (0: every step returns drained)")
    ap.add_argument("--timeline", default=None, metavar="FILE",
                    help="streamed configuration: write the event timeline of the LAST timed step (per block: upload, kernels, "
                         "write-back start / end from HIP events), the link rates and the share of the copy time that kernels "
                         "ran under, as text")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one 1 GiB device-to-device copy, a kernel of known HBM traffic that calibrates "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters in the same run")
    return ap.parse_args()


def device_weights(torch, shapes, dtype_code, dev, seed=0):
    tdt = {0: torch.float32, 1: torch.bfloat16, 2: torch.float16}[dtype_code]
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    out = []
    for name, shape in shapes:
        leaf = name.split(".")[-1]
        if len(shape) == 2:
            t = torch.empty(shape, dtype=tdt, device=dev).normal_(0.0, 0.02, generator=gen)
        elif leaf.endswith("_g"):
            t = torch.ones(shape, dtype=tdt, device=dev)
        else:
            t = torch.zeros(shape, dtype=tdt, device=dev)
        out.append(t)
    return out


def _cores():
    n = os.cpu_count() or 1
    try:
        n = min(n, int(os.environ.get("OMP_NUM_THREADS", n)))
    except ValueError:
        pass
    return n


def cpu_baseline(cfgd, name):
    """The oracle, as it stands, on a bounded sample of the same workload: one decoder block at the
    real width (both signs: z, W+-, forward; then its update) plus embeddings / LM head / loss, on a
    reduced token count.  Per-parameter cost is extrapolated to all blocks, per-token cost to the
    full batch."""
    import numpy as np
    import zo_inputs as zi
    from oracle import zo_oracle as zo
    d, f, V, L = cfgd["d_model"], cfgd["d_ffn"], cfgd["vocab"], cfgd["n_layers"]
    dt = cfgd["dtype"]
    full_tokens = cfgd["batch"] * cfgd["seq"]
    if name == "tiny":
        ocfg = zo.Config(L, d, cfgd["n_heads"], f, V, cfgd["max_pos"], dt)
        theta = zi.make_weights(ocfg.shapes(), dt, seed=0)
        tok = zi.make_tokens(cfgd["batch"], cfgd["seq"], V)
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < 5.0:
            zo.zo_step_fused(ocfg, theta, tok, n, cfgd["eps"], cfgd["lr"])
            n += 1
        dtm = (time.perf_counter() - t0) / n
        return {"value": full_tokens / dtm, "unit": "tokens/s", "cores": _cores(), "kind": "oracle",
                "sample": "%d whole steps of the same workload" % n}
    s_vocab = min(V, 8192)
    ocfg = zo.Config(1, d, cfgd["n_heads"], f, s_vocab, cfgd["seq"], dt)
    theta = zi.make_weights(ocfg.shapes(), dt, seed=0)
    blk = ocfg.block_ids(0)
    eps = cfgd["eps"]
    t0 = time.perf_counter()
    wp = [zo.widen(zo.axpy_z(theta[i], dt, 0, i, eps), dt) for i in blk]
    wm = [zo.widen(zo.axpy_z(theta[i], dt, 0, i, -np.float32(eps)), dt) for i in blk]
    t_stage = time.perf_counter() - t0
    t0 = time.perf_counter()
    for i in blk:
        zo.axpy_z(theta[i], dt, 0, i, -1e-7, out=theta[i])
    t_upd = time.perf_counter() - t0
    e64 = zo.widen(theta[0], dt)
    # token sample: grown until the whole sample is worth about ten seconds of CPU work (or the full sequence)
    s_seq, s_batch = min(cfgd["seq"], 64), 1
    while True:
        tok = zi.make_tokens(s_batch, s_seq, s_vocab)
        h = zo.embed(tok, e64, zo.widen(theta[1], dt))
        t0 = time.perf_counter()
        hp = zo.block_forward(h, dict(zip(zo.BLOCK_TENSORS, wp)), ocfg.n_heads, ocfg.ln_eps)
        hm = zo.block_forward(h, dict(zip(zo.BLOCK_TENSORS, wm)), ocfg.n_heads, ocfg.ln_eps)
        t_fwd = time.perf_counter() - t0
        t0 = time.perf_counter()
        for hh in (hp, hm):
            zo.next_token_loss(zo.head_logits(hh, zo.widen(theta[2 + 16], dt), zo.widen(theta[3 + 16], dt), e64, ocfg.ln_eps), tok)
        t_head = time.perf_counter() - t0
        if t_stage + t_upd + t_fwd + t_head >= 10.0 or (s_seq >= cfgd["seq"] and s_batch >= cfgd["batch"]):
            break
        if s_seq < cfgd["seq"]:
            s_seq = min(cfgd["seq"], s_seq * 4)
        else:
            s_batch = min(cfgd["batch"], s_batch * 4)
    per_block_params = sum(theta[i].size for i in blk)
    embed_params = V * d + cfgd["max_pos"] * d
    fixed = (t_stage + t_upd) * (L + embed_params / per_block_params)
    per_token = (L * t_fwd + t_head * (V / s_vocab)) / (s_seq * s_batch)
    step_s = fixed + per_token * full_tokens
    return {"value": full_tokens / step_s, "unit": "tokens/s", "cores": _cores(), "kind": "oracle",
            "sample": "1 of %d blocks at real width with %d x %d tokens and a %d-row LM head, timed %.1f s; per-parameter cost "
                      "(z, W+-, update) scaled to all parameters, per-token cost to %d tokens (extrapolated)"
                      % (L, s_batch, s_seq, s_vocab, t_stage + t_fwd + t_upd + t_head, full_tokens)}


def _union_ms(intervals):
    """Total length of the union of (start, end) intervals."""
    tot, cur_a, cur_b = 0.0, None, None
    for a, b in sorted(intervals):
        if cur_b is None or a > cur_b:
            if cur_b is not None:
                tot += cur_b - cur_a
            cur_a, cur_b = a, b
        else:
            cur_b = max(cur_b, b)
    return tot + (cur_b - cur_a if cur_b is not None else 0.0)


def _overlap_ms(a_list, b_list):
    """Length of (union of a) intersected with (union of b)."""
    return _union_ms(a_list) + _union_ms(b_list) - _union_ms(list(a_list) + list(b_list))


def write_timeline(args, c, spans, block_bytes, step_s):
    """Alg. 3 as the device ran it: the records of the last timed step (upload U, kernels C, write-back O per block),
    achieved link rates over the copies themselves, and how much of the time the link was busy had kernels running
    beside it.  Returns the summary figures; writes the text file when --timeline names one."""
    L = c["n_layers"]
    comp = [s for s in spans if s[0] == 1]
    # the last step = the last L compute records; copies belong to it from its first upload on
    last = comp[-L:]
    all_ups = [s for s in spans if s[0] == 0]
    n_up = len(all_ups) // max(len(comp) // L, 1)          # uploads per step (the same in every step)
    ups = all_ups[-n_up:] if n_up else []
    t_begin = min([last[0][2]] + [s[2] for s in ups[:1]])
    t_end = last[-1][3]
    wbs = [s for s in spans if s[0] == 2 and s[2] >= t_begin]       # this step's write-backs (the last may end after the kernels)
    up_ms = sum(s[3] - s[2] for s in ups)
    wb_ms = sum(s[3] - s[2] for s in wbs)
    link = [(s[2], s[3]) for s in ups + wbs]
    kern = [(s[2], s[3]) for s in last]
    link_busy = _union_ms(link)
    hidden = _overlap_ms(link, kern)
    kern_busy = _union_ms(kern)
    summ = {"timeline_step_ms": t_end - t_begin,
            "h2d_gbs_while_copying": block_bytes * len(ups) / (up_ms * 1e-3) / 1e9 if up_ms else 0.0,
            "d2h_gbs_while_copying": block_bytes * len(wbs) / (wb_ms * 1e-3) / 1e9 if wb_ms else 0.0,
            "link_busy_ms": link_busy, "kernels_busy_ms": kern_busy,
            "kernel_time_under_copies_frac": hidden / kern_busy if kern_busy else 0.0,
            "copy_time_with_kernels_beside_frac": hidden / link_busy if link_busy else 0.0}
    if args.timeline:
        with open(args.timeline, "w") as f:
            f.write("Alg. 3 timeline of one streamed ZO-SGD step (the last timed one), from HIP events on the stream each operation ran on\n")
            f.write("command: python bench.py %s\n" % " ".join(sys.argv[1:]))
            f.write("%s, batch %d x seq %d, %d blocks (%d in pinned host memory, %d in HBM), write-back every %d step(s), look-ahead %d; "
                    "block = %.3f GB\n" % (args.config, c["batch"], c["seq"], L, len({s[1] for s in ups}) if ups else 0,
                                            L - (len({s[1] for s in ups}) if ups else 0), args.writeback_interval, args.lookahead,
                                            block_bytes / 1e9))
            f.write("step %.1f ms by the wall clock (%.1f tokens/s); first kernel to last kernel of the step %.1f ms\n"
                    % (step_s * 1e3, c["batch"] * c["seq"] / step_s, t_end - t_begin))
            f.write("uploads: %d, %.1f ms each on average, %.1f GB/s while copying; write-backs: %d, %.1f ms each, %.1f GB/s while copying\n"
                    % (len(ups), up_ms / max(len(ups), 1), summ["h2d_gbs_while_copying"], len(wbs), wb_ms / max(len(wbs), 1),
                       summ["d2h_gbs_while_copying"]))
            f.write("link busy (either direction) %.1f ms, kernels busy %.1f ms; %.1f %% of the kernel time ran under a copy, "
                    "%.1f %% of the link-busy time had kernels beside it\n"
                    % (link_busy, kern_busy, 100 * summ["kernel_time_under_copies_frac"], 100 * summ["copy_time_with_kernels_beside_frac"]))
            f.write("\nms since the step's first upload or kernel; U = upload of the block into its slot, C = the block's kernels (pending updates, "
                    "staging, dual forward), O = write-back\n")
            f.write("%5s  %21s  %21s  %21s\n" % ("block", "U start .. end", "C start .. end", "O start .. end"))
            by_u = {s[1]: s for s in ups}
            by_o = {s[1]: s for s in wbs}
            for s in last:
                b = s[1]
                u = "%9.1f .. %9.1f" % (by_u[b][2] - t_begin, by_u[b][3] - t_begin) if b in by_u else "%21s" % "(in HBM)"
                o = "%9.1f .. %9.1f" % (by_o[b][2] - t_begin, by_o[b][3] - t_begin) if b in by_o else "%21s" % "-"
                f.write("%5d  %21s  %9.1f .. %9.1f  %21s\n" % (b, u, s[2] - t_begin, s[3] - t_begin, o))
    return summ


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X runs the whole ZO-SGD step); run with --gpus 1. "
              "No figure for %d GPUs exists." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2507_03211_amd.build import ensure_built
    ensure_built()                      # loads what is built, compiles only when nothing is
    import paper_2507_03211_amd as zo_amd
    import zo_inputs as zi

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    c = dict(zi.CONFIGS[args.config])
    dname = {0: "f64", 1: "bf16", 2: "f16"}[c["dtype"]]
    if args.batch:
        c["batch"] = args.batch
    if args.seq:
        c["seq"] = args.seq
        c["max_pos"] = max(c["max_pos"], args.seq)
    dev = "cuda:0"
    shapes = zi.tensor_shapes(c["n_layers"], c["d_model"], c["d_ffn"], c["vocab"], c["max_pos"])
    streamed = args.config == "opt-175b"
    if args.steps is None:
        args.steps = 3 if streamed else 20
    if args.warmup is None:
        args.warmup = 1 if streamed else 3
    host_ring = None
    if not streamed:
        tensors = device_weights(torch, shapes, c["dtype"], dev)
    else:
        # embeddings and final LayerNorm on the device; blocks in pinned host memory, one contiguous region each
        tdt = {0: torch.float32, 1: torch.bfloat16, 2: torch.float16}[c["dtype"]]
        resident = device_weights(torch, shapes[:2] + shapes[-2:], c["dtype"], dev)
        block_shapes = shapes[2:18]
        per_block = sum(int(torch.Size(sh).numel()) for _, sh in block_shapes)
        nring = max(1, min(args.host_blocks, c["n_layers"]))
        # one pinned allocation per block (a single allocation of tens of GB can be refused where these are not);
        # if the box will not pin as many as asked for, the layers cycle through those it gave
        one = torch.cat([t.reshape(-1) for t in device_weights(torch, block_shapes, c["dtype"], dev, seed=7)]).cpu()
        host_ring = []
        for r in range(nring):
            try:
                blk_host = torch.empty(per_block, dtype=tdt, pin_memory=True)
            except RuntimeError:
                if not host_ring:
                    raise
                break
            blk_host.copy_(one)
            host_ring.append(blk_host)
        nring = len(host_ring)
        del one
        offs, o = [], 0
        for _, sh in block_shapes:
            offs.append(o)
            o += int(torch.Size(sh).numel())
        esz = host_ring[0].element_size()
        tensors = [resident[0], resident[1]]
        n_host = c["n_layers"] - max(0, min(args.hbm_blocks, c["n_layers"]))
        host_at = {int((i + 0.5) * c["n_layers"] / n_host) for i in range(n_host)}       # evenly spread
        hbm_keep, nh = [], 0
        for l in range(c["n_layers"]):
            if l in host_at:
                base = host_ring[nh % nring].data_ptr()
                nh += 1
                tensors += [base + off * esz for off in offs]
            else:
                blk = device_weights(torch, block_shapes, c["dtype"], dev, seed=100 + l)
                hbm_keep.append(blk)
                tensors += blk
        tensors += [resident[2], resident[3]]
    tokens = torch.randint(0, c["vocab"], (c["batch"], c["seq"]), dtype=torch.int32, device=dev,
                           generator=torch.Generator(device=dev).manual_seed(1))
    cfg = zo_amd.make_config(c["n_layers"], c["d_model"], c["n_heads"], c["d_ffn"], c["vocab"], c["max_pos"], c["dtype"],
                             zo_amd.ZO_STREAMED if streamed else zo_amd.ZO_RESIDENT)
    nbytes = zo_amd.zo_workspace_bytes(cfg, c["batch"], c["seq"])
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream(device=dev)
    copy_stream = torch.cuda.Stream(device=dev) if streamed else None
    torch.cuda.synchronize()
    h = zo_amd.zo_init_model(cfg, tensors, ws, nbytes, c["batch"], c["seq"], stream, copy_stream)
    if args.stochastic_update:
        zo_amd.zo_set_update_rounding(h, zo_amd.ZO_ROUND_STOCHASTIC)
    if streamed and args.writeback_interval != 1:
        zo_amd.zo_set_writeback_interval(h, args.writeback_interval)
    if streamed:
        zo_amd.zo_set_stream_lookahead(h, args.lookahead)

    mode = zo_amd.ZO_MODE_LITERAL if args.mode == "literal" else zo_amd.ZO_MODE_FUSED
    deferred = (not streamed) and mode == zo_amd.ZO_MODE_FUSED and args.update == "deferred"
    if deferred:
        zo_amd.zo_set_deferred_update(h, 1)

    def step(i):
        zo_amd.zo_step(h, tokens, c["batch"], c["seq"], i, c["eps"], c["lr"], mode, want_host=False)

    for i in range(args.warmup):
        step(i)
    if deferred:
        zo_amd.zo_flush_pending(h)          # the timed region starts with nothing pending and ends the same way
    torch.cuda.synchronize()
    launches_per_step = 16 * c["n_layers"] + 64 + 4 * ((2 * c["batch"] * c["seq"]) // 2048 + 2)
    zo_amd.zo_profile_begin(h, launches_per_step * args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    if deferred:
        zo_amd.zo_flush_pending(h)          # the last step's update: every one of the K updates lies inside the timed region
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = zo_amd.zo_profile_end(h)
    spans = zo_amd.zo_profile_spans(h) if streamed else []
    if args.traffic_probe:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        b = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        a.copy_(b)
        torch.cuda.synchronize()
        del a, b
    lp, lm, g = zo_amd.zo_step(h, tokens, c["batch"], c["seq"], 10**6, c["eps"], c["lr"], mode)
    flags = zo_amd.zo_device_flags(h)
    zo_amd.zo_free(h)

    tokens_per_step = c["batch"] * c["seq"]
    kernels = {}
    for name, (ms, n, work) in prof.items():
        if n == 0:
            continue
        rate = work / (ms * 1e-3) if ms > 0 else 0.0
        is_flop = name in ("linear", "attention")
        ach_k = rate / (1e12 if is_flop else 1e9)
        peak_k = PEAK_TFLOPS[dname] if is_flop else PEAK_HBM_GBS
        kernels[name] = {"ms_per_step": ms / args.steps, "launches_per_step": n / args.steps,
                         "achieved": ach_k, "unit": "TFLOP/s" if is_flop else "GB/s", "frac_of_peak": ach_k / peak_k}
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    dom_ms, dom_n, dom_work = prof[dom]
    if dom in ("linear", "attention"):
        peak = PEAK_TFLOPS[dname]
        ach = dom_work / (dom_ms * 1e-3) / 1e12
        roof = {"bound": "mfma" if dname != "f64" else "alu", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak}
    else:
        ach = dom_work / (dom_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS}
    roof["kernel"] = dom
    roof["avg_launch_ms"] = dom_ms / max(dom_n, 1)
    roof["work_per_launch"] = dom_work / max(dom_n, 1)
    # HBM-side bytes per launch of the dominant kernel as rocprofv3's FETCH_SIZE + WRITE_SIZE counted them (a
    # committed summary under profiles/, made with this same command); null for workloads that were not profiled
    roof["traffic"] = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and not (args.batch or args.seq):
        try:
            detail = json.load(open(tpath)).get(args.config, {}).get(dom)
            if detail:
                roof["traffic"] = detail["fetch_bytes_per_launch"] + detail["write_bytes_per_launch"]
                roof["traffic_detail"] = detail
        except Exception:
            roof["traffic"] = None

    out = {
        "metric": "ZO-SGD tokens/s on 1 MI355X (dual +-eps z forward + update)",
        "value": tokens_per_step * args.steps / dt,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dname, "data": "synthetic",
        "config": {"workload": args.config, "n_layers": c["n_layers"], "d_model": c["d_model"], "n_heads": c["n_heads"],
                   "d_ffn": c["d_ffn"], "vocab": c["vocab"], "batch": c["batch"], "seq_len": c["seq"], "eps": c["eps"],
                   "lr": c["lr"], "mode": args.mode, "update_rounding": "stochastic" if args.stochastic_update else "nearest",
                   "update": ("deferred: applied in the next step's staging pass, the last one flushed inside the timed region"
                              if deferred else "deferred per block (Alg. 2 / Alg. 3)" if streamed else "immediate"),
                   "residency": "pinned-host blocks, streamed" if streamed else "hbm"},
        "roofline": roof,
        "kernels": kernels,
        "last_step": {"l_plus": lp, "l_minus": lm, "g": g, "device_flags": flags},
    }
    if streamed:
        block_bytes = host_ring[0].numel() * host_ring[0].element_size()
        step_s = dt / args.steps
        out["streaming"] = {"block_bytes": block_bytes, "blocks_per_step": c["n_layers"], "distinct_host_blocks": len(host_ring),
                            "h2d_gbs": block_bytes * n_host / step_s / 1e9,
                            "d2h_gbs": (block_bytes * n_host / step_s / 1e9 / args.writeback_interval
                                        if args.warmup + args.steps > 1 else 0.0),
                            "writeback_interval": args.writeback_interval,
                            "blocks_in_hbm": c["n_layers"] - n_host, "blocks_streamed": n_host,
                            "compute_ms_per_block": sum(v["ms_per_step"] for v in kernels.values()) / c["n_layers"],
                            "note": ("every streamed layer has a host block of its own" if n_host <= len(host_ring) else
                                     "the streamed layers cycle through fewer distinct host blocks than there are layers (the full "
                                     "model would pin 348 GB): layers that share a region write it back and upload it on different "
                                     "streams without ordering between them, so the host VALUES are not those of one model and are "
                                     "not meaningful; traffic, kernels and schedule are those of the full model")}
        if spans:
            out["streaming"].update(write_timeline(args, c, spans, block_bytes, dt / args.steps))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(c, args.config)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the stage hot path on one MI355X.  One step = F + B + W of one chunk for one
microbatch, all through the C ABI.  The headline workload is the largest single-GPU stage of the
build's configurations: the attention-heavy bf16 stage C4 (2 layers per chunk, hidden 5120, 40
heads, FFN 20480, 4096 tokens, causal; weights N(0, 0.02^2), activations and upstream gradients
N(0, 1), all synthetic and seeded).  The smaller bf16 stages C2 and C3 are timed the same way and
nested under `other_workloads`, and the full d = 4, n = 16 schedule replay at the C5 shape under
`replay`.

Prints ONE JSON line.  `value` is algorithmic TFLOP/s of the whole step with inputs resident in HBM;
`roofline` is the bf16 matrix-core GEMM (the dominant kernel) from HIP events recorded around each of
its launches, on the stream they are launched on, inside traced steps of this very run;
`cpu_baseline` is the fp64 numpy oracle timed on the host on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix-core peak (published)
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E peak (published)


def flops_per_layer(h: int, ffn: int, s: int, b: int = 1):
    """Algorithmic FLOP of one layer per pass.  GEMMs: 2*s*h*(3h + h + 2 ffn) in each of F, B, W.
    Attention (causal): F 2*s^2*h; B twice that (the model-FLOPs convention the paper inherits for
    its MFU, Appendix D.1); B_executed counts what the backward kernels execute."""
    gemm = 2 * s * b * h * (4 * h + 2 * ffn)
    att = b * s * s * h          # one causal score-sized product over all heads of b sequences
    return {"F": gemm + 2 * att, "B": gemm + 4 * att, "W": gemm, "B_executed": gemm + ATTN_BWD_UNITS * att, "gemm": gemm}


# causal score-sized products the attention backward executes (S and dP in both kernels, dQ, dK, dV)
ATTN_BWD_UNITS = 7


def run_workload(P, R, synth, torch, np, name, cfg, steps, warmup, queued, want_host=False):
    """Times F + B + W of one chunk of shape `cfg`: whole steps, single passes, and (traced) every
    operation of the passes.  Returns (result dict, host tensors for the cpu baseline or None)."""
    L, h, f, s = cfg.layers, cfg.hidden, cfg.ffn, cfg.seq
    fl = flops_per_layer(h, f, s, cfg.microbatch)
    params = synth.chunk_params(cfg, name)
    x_h, dy_h = synth.chunk_input(cfg, name), synth.upstream_grad(cfg, name)
    ctx = R.Context(R.cfg_from_synth(cfg), slabs=max(1, queued))
    ch = ctx.add_chunk(params, cfg.dtype)
    x, dy = R.to_device(x_h, cfg.dtype), R.to_device(dy_h, cfg.dtype)
    y, dx = torch.empty_like(x), torch.empty_like(x)

    def step():
        P.stage_forward(ch.handle, 0, x, y)
        P.stage_backward_input(ch.handle, 0, dy, dx)
        P.stage_backward_weight(ch.handle, [0])

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    step_flop = L * (fl["F"] + fl["B"] + fl["W"])
    value = step_flop / (ms_per_step * 1e-3) / 1e12

    # per-pass times with HIP events (the context runs on torch's current stream), medians
    def timed(fn):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); fn(); b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b)

    reps = max(5, min(steps, 20))
    pass_ms = {"F": [], "B": [], "W": []}
    for _ in range(reps):
        pass_ms["F"].append(timed(lambda: P.stage_forward(ch.handle, 0, x, y)))
        pass_ms["B"].append(timed(lambda: P.stage_backward_input(ch.handle, 0, dy, dx)))
        pass_ms["W"].append(timed(lambda: P.stage_backward_weight(ch.handle, [0])))
    passes = {}
    for k in "FBW":
        ms = float(np.median(pass_ms[k]))
        tf = L * fl[k] / (ms * 1e-3) / 1e12
        passes[k] = {"ms": round(ms, 4), "tflops": round(tf, 1), "achieved_over_bf16_peak": round(tf / PEAK_BF16_TFLOPS, 4)}
    passes["B"]["tflops_executed"] = round(L * fl["B_executed"] / (passes["B"]["ms"] * 1e-3) / 1e12, 1)
    if queued > 1:
        # deferred W: F and B of q microbatches (untimed), then ONE W call for all of them
        qms = []
        for _ in range(5):
            for j in range(queued):
                P.stage_forward(ch.handle, j, x, y)
                P.stage_backward_input(ch.handle, j, dy, dx)
            qms.append(timed(lambda: P.stage_backward_weight(ch.handle, list(range(queued)))))
        ms = float(np.median(qms)) / queued
        tf = L * fl["W"] / (ms * 1e-3) / 1e12
        passes[f"W_queued{queued}"] = {"ms_per_microbatch": round(ms, 4), "tflops": round(tf, 1),
                                       "achieved_over_bf16_peak": round(tf / PEAK_BF16_TFLOPS, 4)}

    # every operation of the passes between HIP events (on the context's stream) in traced steps
    P.pmc_trace_begin(ctx.ctx, 8192)
    for _ in range(reps):
        step()
    recs = P.pmc_trace_end(ctx.ctx, 8192)
    by_op = {}
    for r in recs:
        by_op.setdefault(r["op"], []).append(r["ms"])
    op_ms_per_step = {op: round(sum(v) / reps, 4) for op, v in by_op.items()}
    gemms = [r for r in recs if r["op"] == "gemm"]
    gemm_flop = sum(2.0 * r["m"] * r["n"] * r["k"] for r in gemms)
    gemm_ms = sum(r["ms"] for r in gemms)
    shapes = {}
    for r in gemms:
        shapes.setdefault((r["pass_"], r["m"], r["n"], r["k"]), []).append(r["ms"])
    gemm_table = [{"pass": k[0], "m": k[1], "n": k[2], "k": k[3], "us": round(1e3 * float(np.mean(v)), 1),
                   "tflops": round(2.0 * k[1] * k[2] * k[3] / (float(np.mean(v)) * 1e-3) / 1e12, 1)}
                  for k, v in sorted(shapes.items())]
    achieved = gemm_flop / (gemm_ms * 1e-3) / 1e12
    gemm_by_pass = {}
    for k in "FBW":
        sel = [r for r in gemms if r["pass_"] == k]
        if sel:
            tf = sum(2.0 * r["m"] * r["n"] * r["k"] for r in sel) / (sum(r["ms"] for r in sel) * 1e-3) / 1e12
            gemm_by_pass[k] = {"tflops": round(tf, 1), "frac": round(tf / PEAK_BF16_TFLOPS, 4)}

    # HBM-bound row kernels: algorithmic bytes (read + written) per launch over its traced time
    e = 2 if cfg.dtype == "bf16" else 4
    T = cfg.tokens

    def rate(sel, nbytes):
        ms = [r["ms"] for r in recs if sel(r)]
        if not ms:
            return None
        t = float(np.median(ms))
        gbs = nbytes / (t * 1e-3) / 1e9
        return {"us_per_launch": round(1e3 * t, 2), "GB_per_s": round(gbs, 1), "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 3),
                "bytes_per_launch": nbytes}

    elementwise = {
        "ln_fwd": rate(lambda r: r["op"] == "ln_fwd", 2 * T * h * e),                          # x in, y out
        "ln_bwd": rate(lambda r: r["op"] == "ln_bwd" and not r["trans_a"], 4 * T * h * e),      # dy, x, resid in, dx out
        "colsum": rate(lambda r: r["op"] == "colsum", T * (5 * h + f) * e),                     # the four dY of a layer
        "copy": rate(lambda r: r["op"] == "copy", 2 * T * h * e),
    }
    att_f = [r["ms"] for r in recs if r["op"] == "attn_fwd"]
    att_b = [r["ms"] for r in recs if r["op"] == "attn_bwd"]
    att_unit = cfg.microbatch * s * s * h          # one causal score-sized product over all heads
    fwd_tf = 2 * att_unit / (float(np.median(att_f)) * 1e-3) / 1e12
    bwd_t = float(np.median(att_b)) * 1e-3
    attention = {"fwd_us": round(1e3 * float(np.median(att_f)), 1), "fwd_tflops": round(fwd_tf, 1),
                 "fwd_frac_of_bf16_peak": round(fwd_tf / PEAK_BF16_TFLOPS, 4),
                 "bwd_us": round(1e6 * bwd_t, 1),
                 "bwd_tflops_model": round(4 * att_unit / bwd_t / 1e12, 1),
                 "bwd_frac_of_bf16_peak_model": round(4 * att_unit / bwd_t / 1e12 / PEAK_BF16_TFLOPS, 4),
                 "bwd_tflops_executed": round(ATTN_BWD_UNITS * att_unit / bwd_t / 1e12, 1),
                 "flop": f"causal: forward 2 s^2 h; backward 4 s^2 h by the model convention, {ATTN_BWD_UNITS} s^2 h executed"}

    def gemm_bytes(r):
        """Algorithmic HBM bytes of one product: both operands once, the result once (W: fp32
        read-modify-write), plus the tensor its epilogue reads or writes besides (residual, GeLU
        output, GeLU input)."""
        m, n, k = r["m"], r["n"], r["k"]
        if r["pass_"] == "W":
            return 2 * (m * k + k * n) + 8 * m * n
        extra = 2 * m * n if (n == f or (r["pass_"] == "F" and n == h)) else 0
        return 2 * (m * k + k * n) + 2 * m * n + extra

    traffic, traffic_src = stored_traffic(name)
    roofline = {"bound": "mfma",
                "kernel": "gemm_bf16_dma_kernel / gemm_bf16_wgrad_persistent_kernel / gemm_bf16_wgrad_pair_kernel, with "
                          "splitk_reduce_kernel where K is split (every product of a step: 4 projections x F,B,W x layers)",
                "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic, "traffic_source": traffic_src,
                "timing": "HIP events around every GEMM launch of traced steps in this run, on the stream of the launches "
                          "(while traced, the W pass keeps its products on that one stream)",
                "avg_launch_us": round(1e3 * gemm_ms / len(gemms), 2), "flop_per_launch": gemm_flop / len(gemms),
                "algorithmic_bytes_per_launch": round(sum(gemm_bytes(r) for r in gemms) / len(gemms)),
                "launches_per_step": len(gemms) // reps, "by_pass": gemm_by_pass}

    res = {"value": round(value, 2), "ms_per_step": round(ms_per_step, 4), "flop_per_step": step_flop,
           "step_over_bf16_peak": round(value / PEAK_BF16_TFLOPS, 4),
           "roofline": roofline, "passes": passes, "op_ms_per_step": op_ms_per_step, "gemm_shapes": gemm_table,
           "elementwise_hbm": elementwise, "attention": attention}
    ctx.close()
    del ctx, ch
    torch.cuda.empty_cache()
    return res, ((params, x_h, dy_h) if want_host else None)


def workload_text(name, cfg):
    return (f"{name}: GPT stage, {cfg.layers} layers/chunk, hidden {cfg.hidden}, {cfg.heads} heads, FFN {cfg.ffn}, "
            f"seq {cfg.seq}, microbatch {cfg.microbatch}, causal, {cfg.dtype} storage + fp32 accumulate; "
            "one step = F + B + W of one chunk")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C4", help="headline workload (C4: the largest single-GPU stage)")
    ap.add_argument("--also", default="C2,C3", help="workloads timed the same way and nested under other_workloads")
    ap.add_argument("--microbatch", type=int, default=0,
                    help="override the workload's microbatch size (sequences per pass): the arithmetic-intensity "
                         "sweep of Appendix D.2; 0 keeps the workload's own (1)")
    ap.add_argument("--queued", type=int, default=4,
                    help="also time W for this many queued microbatches in one call (deferred W, contracted "
                         "together); 0 or 1 skips it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-replay", action="store_true", help="skip the d=4, n=16 schedule replay at the C5 shape")
    ap.add_argument("--profile", action="store_true",
                    help="for profiler runs: the headline workload only (no other workloads, replay, queued W or cpu baseline)")
    ap.add_argument("--w-streams", type=int, default=0, choices=(0, 1, 2),
                    help="streams of the W pass (library switch w_streams): 1 keeps every kernel on one stream, which is "
                         "how the traced steps behind `roofline` run; a kernel trace of such a run shows un-overlapped "
                         "kernel durations.  0: the library's default (2)")
    ap.add_argument("--microbatch-study", action="store_true",
                    help="instead of the benchmark line: the single-pass table over microbatch sizes (Appendix D.2) and "
                         "V-Half at twice the microbatch size against 1F1B (Section 4.3), as one JSON object")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="before the timed region, copy a cold device buffer of this many MiB three times "
                         "(a plain copy kernel of known size that scales the profiler's HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2
    if args.profile:
        args.also, args.no_replay, args.no_cpu_baseline, args.queued = "", True, True, 0

    import numpy as np
    import torch

    import paper_2405_15362_amd as P
    import synth
    from paper_2405_15362_amd import runtime as R

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    def shape_of(tag):
        cfg, name = synth.CONFIGS[tag], tag
        if args.microbatch > 0 and args.microbatch != cfg.microbatch:
            cfg = dataclasses.replace(cfg, microbatch=args.microbatch)
            name = f"{tag}x{args.microbatch}"
        return name, cfg

    if args.w_streams:
        P.pmc_tuning_set("w_streams", args.w_streams)
    if args.microbatch_study:
        print(json.dumps(microbatch_study(P, R, synth, torch, np, args.steps, args.warmup)))
        return 0

    if args.copy_calibration > 0:
        src = torch.ones(args.copy_calibration << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    name, cfg = shape_of(args.config)
    head, host = run_workload(P, R, synth, torch, np, name, cfg, args.steps, args.warmup, args.queued,
                              want_host=not args.no_cpu_baseline)
    out = {
        "metric": "stage F+B+W TFLOP/s per microbatch", "value": head["value"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": workload_text(name, cfg), "flop_per_step": head["flop_per_step"],
                   "flop_convention": "algorithmic; attention backward = 2x forward"},
        "roofline": head["roofline"],
        "step_over_bf16_peak": head["step_over_bf16_peak"],
        "passes": head["passes"], "op_ms_per_step": head["op_ms_per_step"], "gemm_shapes": head["gemm_shapes"],
        "elementwise_hbm": head["elementwise_hbm"], "attention": head["attention"],
    }

    others = {}
    for tag in [t for t in args.also.split(",") if t and t != args.config]:
        oname, ocfg = shape_of(tag)
        res, _ = run_workload(P, R, synth, torch, np, oname, ocfg, args.steps, args.warmup, args.queued)
        res["workload"] = workload_text(oname, ocfg)
        res.pop("gemm_shapes")
        others[tag] = res
    if others:
        out["other_workloads"] = others

    # per schedule at d=4, n=16: peak activation bytes vs 1F1B (C5 chunk shape, accounting) and the
    # scheduler's bubble rate (Appendix D: idle share of the squeezed schedule's run time) with the
    # F, B, W times just measured for one chunk of the headline workload
    c5 = R.cfg_from_synth(synth.CONFIGS["C5"])
    m5, st5 = P.pmc_activation_bytes(c5), P.pmc_activation_stats_bytes(c5)
    d_sim, n_sim = 4, 16
    t_f, t_b, t_w = (head["passes"][k]["ms"] for k in "FBW")
    mem = {}
    for kind in ("1f1b", "vzb", "vhalf", "vmin", "1f1bv"):
        sch = P.pmc_schedule_build(kind, d_sim, n_sim)
        acc = P.pmc_schedule_account(sch, m5, st5)
        span = P.pmc_schedule_makespan(sch, t_f, t_b, t_w)
        reo = P.pmc_schedule_reorder(sch)
        span_reo = P.pmc_schedule_makespan(reo, t_f, t_b, t_w)
        P.pmc_schedule_destroy(reo)
        P.pmc_schedule_destroy(sch)
        work = 2 * n_sim * (t_f + t_b + t_w)
        mem[kind] = {"peak_units": [a[0] for a in acc], "max_peak_bytes": max(a[1] for a in acc),
                     "bubble_rate": round(1.0 - work / span, 4),
                     "bubble_rate_reordered": round(1.0 - work / span_reo, 4)}
    for kind in list(mem):
        mem[kind]["vs_1f1b"] = round(mem[kind]["max_peak_bytes"] / mem["1f1b"]["max_peak_bytes"], 4)
    # the adaptive scheduler (Appendix A/B) under a limit of k live units per device, same pass times
    adaptive = {}
    for k in range(4, 9):
        sch, res = P.pmc_schedule_search(d_sim, n_sim, k, t_f, t_b, t_w)
        P.pmc_schedule_destroy(sch)
        adaptive[str(k)] = {"peak_units": res["peak_units"], "vs_1f1b": round(res["peak_units"] / 8.0, 4),
                            "bubble_rate": round(1.0 - 2 * n_sim * (t_f + t_b + t_w) / res["makespan"], 4)}
    mem["adaptive_by_limit_units"] = adaptive
    out["peak_activation"] = {"config": "d=4, n=16, 2-layer chunks hidden 4096 seq 2048 bf16 (accounting); "
                                        f"bubble rate from the headline workload's measured F/B/W = {t_f}/{t_b}/{t_w} ms", **mem}

    if not args.no_replay:
        out["replay"] = replay_c5(P, R, synth, torch)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, name, *host)

    print(json.dumps(out))
    return 0


def stored_traffic(name):
    """HBM-side bytes per product (fetch + write) from the profiler's FETCH_SIZE and WRITE_SIZE
    counters on this workload.  Counters cannot be read from inside this process: the figure comes
    from the committed summary of two profiler runs of `bench.py --profile --config <name>`, named
    in the second return value.  (None, None) if there is no summary for this workload."""
    rel = os.path.join("profiles", f"gemm_bf16_{name.lower()}_hbm_traffic.txt")
    try:
        with open(os.path.join(ROOT, rel)) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(float(line.split(":", 1)[1])), rel
    except OSError:
        pass
    return None, None


def cpu_baseline(cfg, name, params, x_h, dy_h):
    """The oracle as it stands (numpy, fp64) on the host, on a bounded sample of the headline
    workload: F + B + W of its FIRST LAYER (a one-layer chunk of the same shape, same inputs), whole
    passes repeated until about ten seconds are on the clock."""
    import numpy as np
    from oracle import layer as OL
    try:
        import threadpoolctl
        cores = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=os.cpu_count())
    except Exception:
        cores = os.cpu_count()
    p64 = OL.cast_params(params[:1])
    x64, dy64 = x_h.astype(np.float64), dy_h.astype(np.float64)
    fl = flops_per_layer(cfg.hidden, cfg.ffn, cfg.seq, cfg.microbatch)
    layer_flop = fl["F"] + fl["B"] + fl["W"]
    reps, t0 = 0, time.perf_counter()
    while True:
        y, saved = OL.chunk_forward(x64, p64, cfg.heads, cfg.causal, cfg.ln_eps, cfg.microbatch)
        _, stash, _ = OL.chunk_backward_input(dy64, p64, saved, cfg.heads, cfg.microbatch)
        OL.chunk_backward_weight(saved, stash)
        reps += 1
        sec = time.perf_counter() - t0
        if sec >= 10.0 or reps >= 20:
            break
    return {"value": round(reps * layer_flop / sec / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{reps} x (F+B+W of one layer of {name}, 1 microbatch; the step has {cfg.layers} such layers) "
                      f"in fp64 numpy, {sec:.1f} s",
            "seconds_per_step_extrapolated": round(sec / reps * cfg.layers, 2)}


def replay_run(P, R, synth, torch, cfg, d, n, kinds, seed=5):
    """Replays the schedules `kinds` for d simulated devices and n microbatches with 2d chunks of shape
    cfg (random-initialised weights made on the GPU): per kind the wall time of one iteration on one
    stream, summed F/B/W pass times, measured peaks, and the finish time the schedule would have on d
    devices with the measured mean pass times (squeezed, then reordered: Appendix C)."""
    pcfg = R.cfg_from_synth(cfg)
    res = {}
    gen = torch.Generator(device="cuda").manual_seed(seed)
    shapes = synth.param_shapes(cfg)
    scheds = {k: P.pmc_schedule_build(k, d, n) for k in kinds}
    ws = max(P.pmc_replay_workspace_bytes(s, pcfg) for s in scheds.values())
    ctx = R.Context(pcfg, slabs=2 * d * d, workspace_bytes=ws)
    chunks = []
    for c in range(2 * d):
        ch = R.Chunk.__new__(R.Chunk)
        ch.context = ctx
        ch.params, ch.grads = [], []
        for l in range(cfg.layers):
            p = {}
            for k_, shp in shapes.items():
                t = torch.randn(shp, device="cuda", generator=gen) * 0.02
                if k_ in ("ln1_g", "ln2_g"):
                    t += 1.0
                p[k_] = t.to(torch.bfloat16)
            ch.params.append(p)
            ch.grads.append({k_: torch.zeros(shp, dtype=torch.float32, device="cuda") for k_, shp in shapes.items()})
        ch.handle = P.pmc_chunk_create(ctx.ctx, pcfg)
        P.pmc_chunk_bind(ch.handle, [p[k_] for p in ch.params for k_ in R.PARAM_NAMES],
                         [g[k_] for g in ch.grads for k_ in R.PARAM_NAMES])
        ctx.chunks.append(ch)
        chunks.append(ch)
    xs = [torch.randn(cfg.tokens, cfg.hidden, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(n)]
    dys = [torch.randn(cfg.tokens, cfg.hidden, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(n)]
    fl = flops_per_layer(cfg.hidden, cfg.ffn, cfg.seq, cfg.microbatch)
    iter_flop = 2 * d * n * cfg.layers * (fl["F"] + fl["B"] + fl["W"])
    for kind, s in scheds.items():
        P.schedule_replay(ctx.ctx, s, [c.handle for c in chunks], xs, dys)          # warm-up iteration
        rep, peaks = P.schedule_replay(ctx.ctx, s, [c.handle for c in chunks], xs, dys, flags=P.REPLAY_TIME_PASSES)
        t_f, t_b, t_w = (rep[k] / (2 * d * n) for k in ("ms_f", "ms_b", "ms_w"))     # mean time of one chunk pass
        reo = P.pmc_schedule_reorder(s)
        span = P.pmc_schedule_makespan(reo, t_f, t_b, t_w)
        P.pmc_schedule_destroy(reo)
        res[kind] = {"ms_per_iteration": round(rep["ms_total"], 2), "ms_f": round(rep["ms_f"], 2),
                     "ms_b": round(rep["ms_b"], 2), "ms_w": round(rep["ms_w"], 2),
                     "tflops": round(iter_flop / (rep["ms_total"] * 1e-3) / 1e12, 1),
                     "peak_units": [p[0] for p in peaks], "peak_bytes": [p[1] for p in peaks],
                     "simulated_ms_on_d_devices": round(span, 3),
                     "simulated_bubble_rate": round(1.0 - 2 * n * (t_f + t_b + t_w) / span, 4)}
        P.pmc_schedule_destroy(s)
    ctx.close()
    del ctx, chunks
    torch.cuda.empty_cache()
    return res


def replay_c5(P, R, synth, torch):
    """Full schedule replay at the large configuration: 4 simulated devices, 8 two-layer chunks
    (hidden 4096, seq 2048, bf16), 16 microbatches."""
    res = {"config": "C5: 4 simulated devices x 2 chunks (8 two-layer chunks, hidden 4096, 32 heads, FFN 16384, seq 2048, "
                     "bf16), 16 microbatches, 384 chunk passes per iteration on one stream"}
    res.update(replay_run(P, R, synth, torch, synth.CONFIGS["C5"], 4, 16, ("1f1b", "vzb", "vhalf", "vmin", "1f1bv")))
    for kind in ("vzb", "vhalf", "vmin", "1f1bv"):
        res[kind]["max_peak_bytes_vs_1f1b"] = round(max(res[kind]["peak_bytes"]) / max(res["1f1b"]["peak_bytes"]), 4)
    return res


def microbatch_study(P, R, synth, torch, np, steps, warmup):
    """Appendix D.2's single-pass table on this chip (F / B / W of one chunk at growing microbatch
    size), and Section 4.3's comparison measured: V-Half at twice the microbatch size against 1F1B,
    same number of sequences per iteration, d = 4 simulated devices with chunks of the C2 and C3
    shapes (peak bytes from the pool, throughput from the schedules' finish times with the measured
    pass times)."""
    out = {"single_pass": {}, "vhalf_at_2x_microbatch_vs_1f1b": {}}
    for tag, sizes in (("C2", (1, 2, 4, 8)), ("C3", (1, 2, 4)), ("C4", (1, 2))):
        for b in sizes:
            cfg = dataclasses.replace(synth.CONFIGS[tag], microbatch=b)
            res, _ = run_workload(P, R, synth, torch, np, f"{tag}x{b}", cfg, steps, warmup, 0)
            out["single_pass"][f"{tag} b={b}"] = {"step_tflops": res["value"], "ms_per_step": res["ms_per_step"],
                                                  **{k: res["passes"][k]["tflops"] for k in "FBW"},
                                                  "gemm_frac_of_bf16_peak": res["roofline"]["frac"]}
    d, seqs = 4, 16
    for tag in ("C2", "C3"):
        base = dataclasses.replace(synth.CONFIGS[tag], layers=2)
        one = replay_run(P, R, synth, torch, base, d, seqs, ("1f1b", "vhalf"))
        two = replay_run(P, R, synth, torch, dataclasses.replace(base, microbatch=2), d, seqs // 2, ("vhalf", "vmin"))
        row = {}
        # at d = 4 V-Half holds 6 units against 1F1B's 8, so at twice the microbatch size 1.5 x the bytes (equal
        # only in the many-device limit); V-Min holds 4, so at twice the microbatch size exactly 1F1B's bytes
        for label, r in (("1f1b b=1", one["1f1b"]), ("vhalf b=1", one["vhalf"]), ("vhalf b=2", two["vhalf"]),
                         ("vmin b=2", two["vmin"])):
            row[label] = {"max_peak_bytes": max(r["peak_bytes"]), "ms_one_stream": r["ms_per_iteration"],
                          "simulated_ms_on_d_devices": r["simulated_ms_on_d_devices"],
                          "simulated_bubble_rate": r["simulated_bubble_rate"],
                          "sequences_per_s_simulated": round(seqs / (r["simulated_ms_on_d_devices"] * 1e-3), 1)}
        ref = row["1f1b b=1"]
        for label in ("vhalf b=1", "vhalf b=2", "vmin b=2"):
            row[label]["peak_bytes_vs_1f1b"] = round(row[label]["max_peak_bytes"] / ref["max_peak_bytes"], 4)
            row[label]["throughput_vs_1f1b"] = round(row[label]["sequences_per_s_simulated"] / ref["sequences_per_s_simulated"], 4)
        out["vhalf_at_2x_microbatch_vs_1f1b"][f"{tag} shape, 2-layer chunks, d={d}, {seqs} sequences"] = row
    return out


if __name__ == "__main__":
    sys.exit(main())

#!/usr/bin/env python3
"""Benchmark of the stage hot path on one MI355X: one step = F + B + W of one chunk for one
microbatch (all through the C ABI), on the bf16 GPT-stage workload (2 layers, hidden 2048, 16 heads,
FFN 8192, seq 1024, microbatch 1; weights N(0, 0.02^2), activations and upstream gradients N(0,1),
all synthetic and seeded).

Prints ONE JSON line.  `value` is algorithmic TFLOP/s of the whole step with inputs resident in HBM;
`roofline` is the bf16 matrix-core GEMM kernel (the dominant kernel) from HIP-event timings of its
own launches inside traced steps; `cpu_baseline` is the fp64 numpy oracle timed on the host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix-core peak


def flops_per_layer(h: int, ffn: int, s: int, b: int = 1):
    """Algorithmic FLOP of one layer per pass.  GEMMs: 2*s*h*(3h + h + 2 ffn) in each of F, B, W.
    Attention (causal): F 2*s^2*h; B twice that (the model-FLOPs convention the paper inherits for
    its MFU, Appendix D.1); the two backward kernels execute 3.5x (scores and dP are recomputed in both)."""
    gemm = 2 * s * b * h * (4 * h + 2 * ffn)
    att = b * s * s * h          # one causal score-sized product over all heads of b sequences
    return {"F": gemm + 2 * att, "B": gemm + 4 * att, "W": gemm, "B_executed": gemm + 7 * att, "gemm": gemm}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C2", help="workload shape (C2 is the metric's; C3/C4 for study)")
    ap.add_argument("--microbatch", type=int, default=0,
                    help="override the workload's microbatch size (sequences per pass): the arithmetic-intensity "
                         "sweep of Appendix D.2; 0 keeps the workload's own (1)")
    ap.add_argument("--queued", type=int, default=4,
                    help="also time W for this many queued microbatches in one call (deferred W, contracted "
                         "together); 0 or 1 skips it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--replay", action="store_true", help="also replay the d=4, n=16 schedules at the C5 shape")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="before the timed region, copy a cold device buffer of this many MiB three times "
                         "(a plain copy kernel of known size that scales the profiler's HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2405_15362_amd as P
    import synth
    from paper_2405_15362_amd import runtime as R

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    name = args.config
    if args.microbatch > 0 and args.microbatch != cfg.microbatch:
        import dataclasses
        cfg = dataclasses.replace(cfg, microbatch=args.microbatch)
        name = f"{args.config}x{args.microbatch}"
    L, h, f, s = cfg.layers, cfg.hidden, cfg.ffn, cfg.seq
    fl = flops_per_layer(h, f, s, cfg.microbatch)

    params = synth.chunk_params(cfg, name)
    x_h, dy_h = synth.chunk_input(cfg, name), synth.upstream_grad(cfg, name)
    ctx = R.Context(R.cfg_from_synth(cfg), slabs=max(1, args.queued))
    ch = ctx.add_chunk(params, cfg.dtype)
    x, dy = R.to_device(x_h, cfg.dtype), R.to_device(dy_h, cfg.dtype)
    y, dx = torch.empty_like(x), torch.empty_like(x)

    def step():
        P.stage_forward(ch.handle, 0, x, y)
        P.stage_backward_input(ch.handle, 0, dy, dx)
        P.stage_backward_weight(ch.handle, [0])

    if args.copy_calibration > 0:
        src = torch.ones(args.copy_calibration << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    step_flop = L * (fl["F"] + fl["B"] + fl["W"])
    value = step_flop / (ms_per_step * 1e-3) / 1e12

    # per-pass times with HIP events (same stream), medians over the traced steps
    def timed(fn, reps):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        out = []
        for a, b in ev:
            a.record(); fn(); b.record()
            out.append((a, b))
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in out]))

    reps = max(5, min(args.steps, 20))
    pass_ms = {"F": [], "B": [], "W": []}
    for _ in range(reps):
        pass_ms["F"].append(timed(lambda: P.stage_forward(ch.handle, 0, x, y), 1))
        pass_ms["B"].append(timed(lambda: P.stage_backward_input(ch.handle, 0, dy, dx), 1))
        pass_ms["W"].append(timed(lambda: P.stage_backward_weight(ch.handle, [0]), 1))
    passes = {}
    for k in "FBW":
        ms = float(np.median(pass_ms[k]))
        passes[k] = {"ms": round(ms, 4), "tflops": round(L * fl[k] / (ms * 1e-3) / 1e12, 1),
                     "frac_of_bf16_peak": round(L * fl[k] / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
    passes["B"]["tflops_executed"] = round(L * fl["B_executed"] / (passes["B"]["ms"] * 1e-3) / 1e12, 1)
    if args.queued > 1:
        # deferred W: F and B of q microbatches (untimed), then ONE W call for all of them
        q, qms = args.queued, []
        for _ in range(5):
            for j in range(q):
                P.stage_forward(ch.handle, j, x, y)
                P.stage_backward_input(ch.handle, j, dy, dx)
            qms.append(timed(lambda: P.stage_backward_weight(ch.handle, list(range(q))), 1))
        ms = float(np.median(qms)) / q
        passes[f"W_queued{q}"] = {"ms_per_microbatch": round(ms, 4), "tflops": round(L * fl["W"] / (ms * 1e-3) / 1e12, 1),
                                  "frac_of_bf16_peak": round(L * fl["W"] / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}

    # dominant kernel: the bf16 GEMM.  Its launches are bracketed by HIP events inside traced steps.
    P.pmc_trace_begin(ctx.ctx, 4096)
    for _ in range(reps):
        step()
    recs = P.pmc_trace_end(ctx.ctx, 4096)
    by_op = {}
    for r in recs:
        by_op.setdefault(r["op"], []).append(r["ms"])
    op_ms_per_step = {op: round(sum(v) / reps, 4) for op, v in by_op.items()}
    gemms = [r for r in recs if r["op"] == "gemm"]
    gemm_flop = sum(2.0 * r["m"] * r["n"] * r["k"] for r in gemms)
    gemm_ms = sum(r["ms"] for r in gemms)
    shapes = {}
    for r in gemms:
        key = (r["pass_"], r["m"], r["n"], r["k"])
        shapes.setdefault(key, []).append(r["ms"])
    gemm_table = [{"pass": k[0], "m": k[1], "n": k[2], "k": k[3], "us": round(1e3 * float(np.mean(v)), 1),
                   "tflops": round(2.0 * k[1] * k[2] * k[3] / (float(np.mean(v)) * 1e-3) / 1e12, 1)}
                  for k, v in sorted(shapes.items())]
    achieved = gemm_flop / (gemm_ms * 1e-3) / 1e12

    # HBM-bound row kernels: algorithmic bytes (read + written) per launch over its traced time
    e = 2 if cfg.dtype == "bf16" else 4
    T = cfg.tokens

    def rate(sel, nbytes):
        ms = [r["ms"] for r in recs if sel(r)]
        if not ms:
            return None
        t = float(np.median(ms))
        return {"us_per_launch": round(1e3 * t, 2), "GB_per_s": round(nbytes / (t * 1e-3) / 1e9, 1), "bytes_per_launch": nbytes}

    elementwise = {
        "ln_fwd": rate(lambda r: r["op"] == "ln_fwd", 2 * T * h * e),                          # x in, y out
        "ln_bwd": rate(lambda r: r["op"] == "ln_bwd" and not r["trans_a"], 4 * T * h * e),      # dy, x, resid in, dx out
        "colsum": rate(lambda r: r["op"] == "colsum", T * (5 * h + f) * e),                     # the four dY of a layer
        "copy": rate(lambda r: r["op"] == "copy", 2 * T * h * e),
    }
    att_f = [r["ms"] for r in recs if r["op"] == "attn_fwd"]
    att_b = [r["ms"] for r in recs if r["op"] == "attn_bwd"]
    att_unit = cfg.microbatch * s * s * h          # one causal score-sized product over all heads
    attention = {"fwd_us": round(1e3 * float(np.median(att_f)), 1), "fwd_tflops": round(2 * att_unit / (float(np.median(att_f)) * 1e-3) / 1e12, 1),
                 "bwd_us": round(1e3 * float(np.median(att_b)), 1),
                 "bwd_tflops_executed": round(7 * att_unit / (float(np.median(att_b)) * 1e-3) / 1e12, 1),
                 "flop": "causal: forward 2 s^2 h; backward executes 7 s^2 h (scores and dP recomputed in both kernels)"}

    def gemm_bytes(r):
        """Algorithmic HBM bytes of one product: both operands once, the result once (W: fp32
        read-modify-write), plus the tensor its epilogue reads or writes besides (residual, GeLU
        output, GeLU input)."""
        m, n, k = r["m"], r["n"], r["k"]
        if r["pass_"] == "W":
            return 2 * (m * k + k * n) + 8 * m * n
        extra = 2 * m * n if (n == f or (r["pass_"] == "F" and n == h)) else 0
        return 2 * (m * k + k * n) + 2 * m * n + extra

    roofline = {"bound": "mfma",
                "kernel": "gemm_bf16_dma_kernel / gemm_bf16_wgrad_persistent_kernel, with splitk_reduce_kernel "
                          "where K is split (every product of a step: 4 projections x F,B,W x layers)",
                "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": stored_traffic(name),
                "avg_launch_us": round(1e3 * gemm_ms / len(gemms), 2), "flop_per_launch": gemm_flop / len(gemms),
                "algorithmic_bytes_per_launch": round(sum(gemm_bytes(r) for r in gemms) / len(gemms)),
                "launches_per_step": len(gemms) // reps}

    out = {
        "metric": "stage F+B+W TFLOP/s per microbatch", "value": round(value, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{name}: GPT stage, {L} layers/chunk, hidden {h}, {cfg.heads} heads, FFN {f}, seq {s}, "
                               f"microbatch {cfg.microbatch}, causal, {cfg.dtype} storage + fp32 accumulate; "
                               "one step = F + B + W of one chunk",
                   "flop_per_step": step_flop, "flop_convention": "algorithmic; attention backward = 2x forward"},
        "roofline": roofline,
        "passes": passes,
        "op_ms_per_step": op_ms_per_step,
        "gemm_shapes": gemm_table,
        "elementwise_hbm": elementwise,
        "attention": attention,
        "mfma_util_vs_peak": round(value / PEAK_BF16_TFLOPS, 4),
    }

    # per schedule at d=4, n=16: peak activation bytes vs 1F1B (C5 chunk shape, accounting) and the
    # scheduler's bubble rate (Appendix D: idle share of the squeezed schedule's run time) with the
    # F, B, W times just measured for one chunk of this workload
    c5 = R.cfg_from_synth(synth.CONFIGS["C5"])
    m5, st5 = P.pmc_activation_bytes(c5), P.pmc_activation_stats_bytes(c5)
    d_sim, n_sim = 4, 16
    t_f, t_b, t_w = passes["F"]["ms"], passes["B"]["ms"], passes["W"]["ms"]
    mem = {}
    for kind in ("1f1b", "vzb", "vhalf", "vmin"):
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
                                        f"bubble rate from this workload's measured F/B/W = {t_f}/{t_b}/{t_w} ms", **mem}

    ctx.close()
    del ctx, ch

    if args.replay:
        out["replay"] = replay_c5(P, R, synth, torch)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, name, params, x_h, dy_h, step_flop)

    print(json.dumps(out))
    return 0


def stored_traffic(name):
    """HBM bytes per product (fetch + write) measured with the profiler's FETCH_SIZE and WRITE_SIZE
    counters on this workload; the figure lives in the committed profile summary.  None if there is
    no summary for this workload."""
    path = os.path.join(ROOT, "profiles", f"gemm_bf16_{name.lower()}_hbm_traffic.txt")
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(float(line.split(":", 1)[1]))
    except OSError:
        pass
    return None


def cpu_baseline(cfg, name, params, x_h, dy_h, step_flop):
    """The oracle as it stands (numpy, fp64), one full step of the same workload on the host."""
    import numpy as np
    from oracle import layer as OL
    try:
        import threadpoolctl
        cores = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=os.cpu_count())
    except Exception:
        cores = os.cpu_count()
    p64 = OL.cast_params(params)
    x64, dy64 = x_h.astype(np.float64), dy_h.astype(np.float64)
    steps, t0 = 0, time.perf_counter()
    while True:  # whole steps until about ten seconds of host work are on the clock
        y, saved = OL.chunk_forward(x64, p64, cfg.heads, cfg.causal, cfg.ln_eps, cfg.microbatch)
        _, stash, _ = OL.chunk_backward_input(dy64, p64, saved, cfg.heads, cfg.microbatch)
        OL.chunk_backward_weight(saved, stash)
        steps += 1
        sec = time.perf_counter() - t0
        if sec >= 10.0 or steps >= 20:
            break
    return {"value": round(steps * step_flop / sec / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{steps} full steps (F+B+W, 1 microbatch) of {name} in fp64 numpy, {sec:.1f} s",
            "seconds_per_step": round(sec / steps, 2)}


def replay_c5(P, R, synth, torch):
    """Full schedule replay at the large configuration: 4 simulated devices, 8 two-layer chunks
    (hidden 4096, seq 2048, bf16), 16 microbatches; random-initialised weights made on the GPU."""
    cfg = synth.CONFIGS["C5"]
    pcfg = R.cfg_from_synth(cfg)
    d, n = 4, 16
    res = {}
    gen = torch.Generator(device="cuda").manual_seed(5)
    shapes = synth.param_shapes(cfg)
    m = P.pmc_activation_bytes(pcfg)
    scheds = {k: P.pmc_schedule_build(k, d, n) for k in ("1f1b", "vzb", "vhalf", "vmin")}
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
    for kind, s in scheds.items():
        P.schedule_replay(ctx.ctx, s, [c.handle for c in chunks], xs, dys)          # warm-up iteration
        rep, peaks = P.schedule_replay(ctx.ctx, s, [c.handle for c in chunks], xs, dys, flags=P.REPLAY_TIME_PASSES)
        res[kind] = {"ms_per_iteration": round(rep["ms_total"], 2), "ms_f": round(rep["ms_f"], 2),
                     "ms_b": round(rep["ms_b"], 2), "ms_w": round(rep["ms_w"], 2),
                     "peak_units": [p[0] for p in peaks], "peak_bytes": [p[1] for p in peaks]}
        P.pmc_schedule_destroy(s)
    ctx.close()
    return res


if __name__ == "__main__":
    sys.exit(main())

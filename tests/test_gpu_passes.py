"""GPU parity of the chunk passes F, B, W and of the schedule replay against the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2405_15362_amd as P
import synth
from oracle import layer as OL
from oracle import schedule as OS
from paper_2405_15362_amd import runtime as R
from gpu_util import assert_close, dev, host, oracle_chunk, rel_l2, tol

pytestmark = pytest.mark.gpu

CASES = {
    # the fp32 configuration of the build (1 layer, hidden 256, 4 heads, FFN 1024, seq 128)
    "c1_f32": synth.CONFIGS["C1"],
    "multi_f32": synth.ChunkCfg(layers=2, hidden=64, heads=4, ffn=200, seq=40, microbatch=2, dtype="f32"),
    "noncausal_f32": synth.ChunkCfg(layers=1, hidden=96, heads=3, ffn=256, seq=52, dtype="f32", causal=False),
    "dh128_bf16": synth.ChunkCfg(layers=2, hidden=256, heads=2, ffn=1024, seq=192, dtype="bf16"),
    "dh64_ragged_bf16": synth.ChunkCfg(layers=3, hidden=192, heads=3, ffn=328, seq=104, microbatch=2, dtype="bf16"),
    # head size 112 (the paper's hidden 7168 over 64 heads): attention tiles 128 wide, 16 columns held at zero
    "dh112_bf16": synth.ChunkCfg(layers=2, hidden=336, heads=3, ffn=512, seq=136, dtype="bf16"),
    # the workload bench.py times, at full size and in the launch configuration it runs in (large GEMM
    # tiles, 64x128 tiles, split K, short-sequence attention shapes, W pass on two streams): every
    # output and gradient element against the oracle (a few seconds of fp64 numpy)
    "c2_full_bf16": synth.CONFIGS["C2"],
    # one layer of the hidden-4096, 2048-token shape: the many-block attention shapes and GEMMs that are
    # neither split nor skinny
    "c3_one_layer_bf16": synth.ChunkCfg(layers=1, hidden=4096, heads=32, ffn=16384, seq=2048, dtype="bf16"),
    # the attention-heavy workload at full size: 2 layers, hidden 5120, 40 heads, FFN 20480, 4096 tokens,
    # causal; the 256x320 tiles, the persistent W kernel, the many-block attention shapes.  Every output
    # and gradient element (all 40 heads through the chunk oracle; about a minute of fp64 numpy)
    "c4_full_bf16": synth.CONFIGS["C4"],
}


def _run_fbw(cfg, tag, n_mb=1, defer=False):
    params = synth.chunk_params(cfg, tag)
    ctx = R.Context(R.cfg_from_synth(cfg), slabs=n_mb)
    ch = ctx.add_chunk(params, cfg.dtype)
    out = []
    xs = [synth.chunk_input(cfg, tag, j) for j in range(n_mb)]
    dys = [synth.upstream_grad(cfg, tag, j) for j in range(n_mb)]
    ys = [dev(np.zeros_like(x), cfg.dtype) for x in xs]
    dxs = [dev(np.zeros_like(x), cfg.dtype) for x in xs]
    for j in range(n_mb):
        P.stage_forward(ch.handle, j, dev(xs[j], cfg.dtype), ys[j])
        if not defer:
            P.stage_backward_input(ch.handle, j, dev(dys[j], cfg.dtype), dxs[j])
            P.stage_backward_weight(ch.handle, [j])
    if defer:
        for j in range(n_mb):
            P.stage_backward_input(ch.handle, j, dev(dys[j], cfg.dtype), dxs[j])
        assert P.pmc_pool_live_slabs(ctx.ctx) == n_mb
        P.stage_backward_weight(ch.handle, list(range(n_mb)))
    torch.cuda.synchronize()
    assert P.pmc_pool_live_slabs(ctx.ctx) == 0 and P.pmc_pool_peak_slabs(ctx.ctx) == (n_mb if defer else 1)
    grads = ch.grads_numpy()
    res = ([host(y) for y in ys], [host(d) for d in dxs], grads)
    ctx.close()
    return params, xs, dys, res


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", list(CASES))
def test_f_b_w_match_oracle(name):
    cfg = CASES[name]
    print("pass parity case", name, cfg, flush=True)
    params, xs, dys, (ys, dxs, grads) = _run_fbw(cfg, name)
    y, dx, ln, wg = oracle_chunk(cfg, params, xs[0], dys[0])
    assert_close(ys[0], y, cfg.dtype, f"{name} y")
    assert_close(dxs[0], dx, cfg.dtype, f"{name} dx")
    for l in range(cfg.layers):
        for k, v in {**ln[l], **wg[l]}.items():
            assert_close(grads[l][k], v, cfg.dtype, f"{name} L{l}.{k}")


@pytest.mark.timeout(900)
def test_config3_four_layers_four_queued_w():
    """The third workload as stated: one chunk of 4 layers (hidden 4096, 32 heads, FFN 16384, 2048
    tokens, bf16); F and B of 4 microbatches, then ONE stage_backward_weight call for the 4 queued
    microbatches into zero-initialised fp32 gradients (each weight gradient one product over the four
    microbatches' concatenated token axis).  Outputs and input gradients of every microbatch and the
    accumulated gradient of every parameter, every element, against the oracle's sum over the
    microbatches (about two minutes of fp64 numpy; one microbatch at a time, only the sums are kept)."""
    cfg, n_mb = synth.CONFIGS["C3"], 4
    params, xs, dys, (ys, dxs, grads) = _run_fbw(cfg, "C3", n_mb, defer=True)
    p64 = OL.cast_params(params)
    total = OL.zero_grads(p64)
    for j in range(n_mb):
        print("config 3 oracle microbatch", j, flush=True)
        y, saved = OL.chunk_forward(xs[j].astype(np.float64), p64, cfg.heads, cfg.causal, cfg.ln_eps, cfg.microbatch)
        dx, stash, ln = OL.chunk_backward_input(dys[j].astype(np.float64), p64, saved, cfg.heads, cfg.microbatch)
        OL.accumulate(total, ln, OL.chunk_backward_weight(saved, stash))
        del saved, stash
        assert_close(ys[j], y, "bf16", f"C3 y[{j}]")
        assert_close(dxs[j], dx, "bf16", f"C3 dx[{j}]")
    for l in range(cfg.layers):
        for k in OL.PARAM_NAMES:
            assert_close(grads[l][k], total[l][k], "bf16", f"C3 L{l}.{k}")


@pytest.mark.parametrize("name", ["multi_f32", "dh128_bf16"])
def test_deferred_w_accumulates_over_microbatches(name):
    cfg = CASES[name]
    n_mb = 3
    params, xs, dys, (ys, dxs, grads) = _run_fbw(cfg, name + "_defer", n_mb, defer=True)
    total = OL.zero_grads(OL.cast_params(params))
    for j in range(n_mb):
        y, dx, ln, wg = oracle_chunk(cfg, params, xs[j], dys[j])
        OL.accumulate(total, ln, wg)
        assert_close(ys[j], y, cfg.dtype, f"{name} y[{j}]")
        assert_close(dxs[j], dx, cfg.dtype, f"{name} dx[{j}]")
    for l in range(cfg.layers):
        for k in OL.PARAM_NAMES:
            assert_close(grads[l][k], total[l][k], cfg.dtype, f"{name} L{l}.{k}")
    # immediate W per microbatch: in fp32 mode the queued pass runs the same products in the same
    # order (same bits); in bf16 mode it contracts the queued microbatches in one product per weight
    # (same sum up to fp32 summation order), LayerNorm and bias gradients keep their order
    _, _, _, (_, _, grads2) = _run_fbw(cfg, name + "_defer", n_mb, defer=False)
    for l in range(cfg.layers):
        for k in OL.PARAM_NAMES:
            if cfg.dtype == "f32" or k not in ("w_qkv", "w_o", "w_1", "w_2"):
                assert np.array_equal(grads[l][k], grads2[l][k]), (l, k)
            else:
                assert rel_l2(grads[l][k], grads2[l][k]) <= 1e-5, (l, k, rel_l2(grads[l][k], grads2[l][k]))


def test_queued_w_groups_larger_than_the_maximum():
    """More queued microbatches than one grouped product takes (8): the list is cut into groups; ragged
    token count (not a multiple of 64) falls back to one microbatch at a time.  Both against the oracle."""
    for name, n_mb in (("dh128_bf16", 10), ("dh64_ragged_bf16", 3)):
        cfg = CASES[name]
        params, xs, dys, (ys, dxs, grads) = _run_fbw(cfg, name + "_q", n_mb, defer=True)
        total = OL.zero_grads(OL.cast_params(params))
        for j in range(n_mb):
            _, _, ln, wg = oracle_chunk(cfg, params, xs[j], dys[j])
            OL.accumulate(total, ln, wg)
        for l in range(cfg.layers):
            for k in OL.PARAM_NAMES:
                assert_close(grads[l][k], total[l][k], cfg.dtype, f"{name} L{l}.{k}")


def test_pass_order_errors():
    cfg = CASES["multi_f32"]
    ctx = R.Context(R.cfg_from_synth(cfg), slabs=1)
    ch = ctx.add_chunk(synth.chunk_params(cfg, "err"), cfg.dtype)
    x = dev(synth.chunk_input(cfg, "err"), cfg.dtype)
    y, dx = torch.empty_like(x), torch.empty_like(x)

    def code(fn, *a):
        with pytest.raises(P.PmcError) as e:
            fn(*a)
        return e.value.code

    assert code(P.stage_backward_input, ch.handle, 0, x, dx) == P.PMC_ERR_STATE       # B before F
    assert code(P.stage_backward_weight, ch.handle, [0]) == P.PMC_ERR_STATE           # W before F
    P.stage_forward(ch.handle, 0, x, y)
    assert code(P.stage_forward, ch.handle, 0, x, y) == P.PMC_ERR_STATE               # live id reused
    assert code(P.stage_forward, ch.handle, 1, x, y) == P.PMC_ERR_NOMEM               # pool exhausted
    assert code(P.stage_backward_weight, ch.handle, [0]) == P.PMC_ERR_STATE           # W before B
    P.stage_backward_input(ch.handle, 0, x, dx)
    assert code(P.stage_backward_input, ch.handle, 0, x, dx) == P.PMC_ERR_STATE       # B twice
    assert code(P.stage_backward_weight, ch.handle, [0, 0]) == P.PMC_ERR_INVALID
    P.stage_backward_weight(ch.handle, [0])
    assert code(P.stage_backward_weight, ch.handle, [0]) == P.PMC_ERR_STATE           # W twice
    torch.cuda.synchronize()
    assert P.pmc_pool_live_slabs(ctx.ctx) == 0
    ctx.close()


def _oracle_model(cfg, chunk_params, xs, dys):
    """The whole model (chunks in order), microbatch after microbatch, in fp64."""
    p64 = [OL.cast_params(p) for p in chunk_params]
    grads = [OL.zero_grads(p) for p in p64]
    ys, dxs = [], []
    for x, dy in zip(xs, dys):
        a = x.astype(np.float64)
        saved = []
        for p in p64:
            a, sv = OL.chunk_forward(a, p, cfg.heads, cfg.causal, cfg.ln_eps, cfg.microbatch)
            saved.append(sv)
        ys.append(a)
        g = dy.astype(np.float64)
        for c in reversed(range(len(p64))):
            g, stash, ln = OL.chunk_backward_input(g, p64[c], saved[c], cfg.heads, cfg.microbatch)
            OL.accumulate(grads[c], ln, OL.chunk_backward_weight(saved[c], stash))
        dxs.append(g)
    return ys, dxs, grads


def _replay(cfg, tag, kind, d, n, chunk_params, xs, dys, reorder=False, sched=None, slabs=None):
    if sched is None:
        sched = P.pmc_schedule_build(kind, d, n)
        if reorder:
            plain = sched
            sched = P.pmc_schedule_reorder(plain)
            P.pmc_schedule_destroy(plain)
    pcfg = R.cfg_from_synth(cfg)
    ctx = R.Context(pcfg, slabs=slabs if slabs is not None else sum(OS.peak_units(kind, d, n)),
                    workspace_bytes=P.pmc_replay_workspace_bytes(sched, pcfg))
    chunks = [ctx.add_chunk(p, cfg.dtype) for p in chunk_params]
    xd = [dev(x, cfg.dtype) for x in xs]
    dyd = [dev(g, cfg.dtype) for g in dys]
    yl = [torch.empty_like(t) for t in xd]
    dxf = [torch.empty_like(t) for t in xd]
    report, peaks = P.schedule_replay(ctx.ctx, sched, [c.handle for c in chunks], xd, dyd, yl, dxf, P.REPLAY_TIME_PASSES)
    torch.cuda.synchronize()
    assert P.pmc_pool_live_slabs(ctx.ctx) == 0
    grads = [c.grads_numpy() for c in chunks]
    out = ([host(t) for t in yl], [host(t) for t in dxf], grads, report, peaks)
    ctx.close()
    P.pmc_schedule_destroy(sched)
    return out


def test_replay_config1_all_schedules():
    """2 simulated devices x 4 microbatches, 4 one-layer fp32 chunks (hidden 256, seq 128), replayed
    as 1F1B, V-Half, V-Min, V-ZB and 1F1B-V: outputs and accumulated gradients against the oracle's whole
    model, peaks against the oracle's accounting, gradients bit-identical across schedules."""
    cfg, d, n = synth.CONFIGS["C1"], 2, 4
    chunk_params = [synth.chunk_params(cfg, "C1", c) for c in range(2 * d)]
    xs = [synth.chunk_input(cfg, "C1", j) for j in range(n)]
    dys = [synth.upstream_grad(cfg, "C1", j) for j in range(n)]
    ys_ref, dxs_ref, grads_ref = _oracle_model(cfg, chunk_params, xs, dys)
    m = OL.chunk_activation_bytes(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, 4, cfg.microbatch, cfg.ffn)
    st = OL.chunk_stats_bytes(cfg.layers, cfg.heads, cfg.seq, cfg.microbatch)
    first = None
    for kind in ("1f1b", "vhalf", "vmin", "vzb", "1f1bv"):
        print("replay", kind, flush=True)
        ys, dxs, grads, report, peaks = _replay(cfg, "C1", kind, d, n, chunk_params, xs, dys)
        for j in range(n):
            assert_close(ys[j], ys_ref[j], "f32", f"{kind} y[{j}]")
            assert_close(dxs[j], dxs_ref[j], "f32", f"{kind} dx[{j}]")
        for c in range(2 * d):
            for k in OL.PARAM_NAMES:
                assert_close(grads[c][0][k], grads_ref[c][0][k], "f32", f"{kind} chunk {c} {k}")
        units = OS.peak_units(kind, d, n)
        want = OS.peak_bytes(kind, d, n, m, st)
        assert [p[0] for p in peaks] == units
        assert [(p[1], p[2]) for p in peaks] == want
        assert report["passes"] == 6 * d * n and report["ms_total"] > 0
        if first is None:
            first = grads
        else:
            for c in range(2 * d):
                for k in OL.PARAM_NAMES:
                    assert np.array_equal(grads[c][0][k], first[c][0][k]), (kind, c, k)


def test_replay_bf16_d4_reduced_width():
    """The d=4, n=16 replay of the large configuration at reduced width (2-layer bf16 chunks)."""
    cfg = synth.ChunkCfg(layers=2, hidden=128, heads=2, ffn=512, seq=64, dtype="bf16")
    d, n = 4, 16
    chunk_params = [synth.chunk_params(cfg, "C5r", c) for c in range(2 * d)]
    xs = [synth.chunk_input(cfg, "C5r", j) for j in range(n)]
    dys = [synth.upstream_grad(cfg, "C5r", j) for j in range(n)]
    ys_ref, dxs_ref, grads_ref = _oracle_model(cfg, chunk_params, xs, dys)
    first = None
    for kind in ("1f1b", "vzb", "vhalf", "vmin", "1f1bv"):
        print("replay", kind, flush=True)
        ys, dxs, grads, report, peaks = _replay(cfg, "C5r", kind, d, n, chunk_params, xs, dys)
        for j in range(n):
            # 16 layers deep: the bf16 roundings of 8 chunks add up, so the element and block bounds
            # are doubled here (the whole-tensor bound stays at 2e-2)
            assert_close(ys[j], ys_ref[j], "bf16", f"{kind} y[{j}]", atol_scale=2.0)
            assert_close(dxs[j], dxs_ref[j], "bf16", f"{kind} dx[{j}]", atol_scale=2.0)
        for c in range(2 * d):
            for l in range(cfg.layers):
                for k in OL.PARAM_NAMES:
                    assert_close(grads[c][l][k], grads_ref[c][l][k], "bf16", f"{kind} chunk {c} L{l}.{k}", atol_scale=2.0)
        assert [p[0] for p in peaks] == OS.peak_units(kind, d, n)
        if first is None:
            first = grads
        else:
            for c in range(2 * d):
                for l in range(cfg.layers):
                    for k in OL.PARAM_NAMES:
                        assert np.array_equal(grads[c][l][k], first[c][l][k]), (kind, c, l, k)


def test_replay_reordered_schedules():
    """Replay of the schedules after warm-up / cool-down reordering (d=4, n=16, reduced width):
    the same peaks of live units as before reordering and the same accumulated gradients, bit for
    bit, as the plain V-ZB replay (W passes of a chunk keep their microbatch order)."""
    cfg = synth.ChunkCfg(layers=1, hidden=128, heads=2, ffn=512, seq=64, dtype="bf16")
    d, n = 4, 16
    chunk_params = [synth.chunk_params(cfg, "C5o", c) for c in range(2 * d)]
    xs = [synth.chunk_input(cfg, "C5o", j) for j in range(n)]
    dys = [synth.upstream_grad(cfg, "C5o", j) for j in range(n)]
    _, _, first, _, _ = _replay(cfg, "C5o", "vzb", d, n, chunk_params, xs, dys)
    ys_ref, dxs_ref, _ = _oracle_model(cfg, chunk_params, xs, dys)
    for kind in ("vzb", "vhalf", "vmin", "1f1b"):
        print("replay reordered", kind, flush=True)
        ys, dxs, grads, report, peaks = _replay(cfg, "C5o", kind, d, n, chunk_params, xs, dys, reorder=True)
        for j in range(n):
            assert_close(ys[j], ys_ref[j], "bf16", f"{kind} y[{j}]", atol_scale=2.0)
            assert_close(dxs[j], dxs_ref[j], "bf16", f"{kind} dx[{j}]", atol_scale=2.0)
        assert [p[0] for p in peaks] == OS.peak_units(kind, d, n)
        assert report["passes"] == 6 * d * n
        for c in range(2 * d):
            for k in OL.PARAM_NAMES:
                assert np.array_equal(grads[c][0][k], first[c][0][k]), (kind, c, k)


def test_replay_adaptive_schedule():
    """A schedule found by the adaptive search under a limit of 5 live units per device (between
    V-Min's 4 and V-Half's 6 at d = 4), replayed with exactly that many slabs per device: the pool's
    measured peaks stay within the limit and the gradients are the plain V-ZB replay's, bit for bit."""
    cfg = synth.ChunkCfg(layers=1, hidden=128, heads=2, ffn=512, seq=64, dtype="bf16")
    d, n, limit = 4, 16, 5
    chunk_params = [synth.chunk_params(cfg, "C5o", c) for c in range(2 * d)]
    xs = [synth.chunk_input(cfg, "C5o", j) for j in range(n)]
    dys = [synth.upstream_grad(cfg, "C5o", j) for j in range(n)]
    _, _, first, _, _ = _replay(cfg, "C5o", "vzb", d, n, chunk_params, xs, dys)
    sched, res = P.pmc_schedule_search(d, n, limit, 1.0, 1.2, 0.8)
    print("adaptive block", res, flush=True)
    assert res["peak_units"] <= limit
    ys, dxs, grads, report, peaks = _replay(cfg, "C5o", None, d, n, chunk_params, xs, dys, sched=sched, slabs=limit * d)
    assert max(p[0] for p in peaks) == res["peak_units"]
    assert report["passes"] == 6 * d * n
    for c in range(2 * d):
        for k in OL.PARAM_NAMES:
            assert np.array_equal(grads[c][0][k], first[c][0][k]), (c, k)



def _gpu_chunks(ctx, cfg, count, seed):
    """`count` chunks of one shape with weights drawn on the GPU from a seeded generator (too many
    parameters to draw on the host in reasonable time): N(0, 0.02^2), LayerNorm gains 1 + N(0, 0.02^2)."""
    gen = torch.Generator(device="cuda").manual_seed(seed)
    shapes = synth.param_shapes(cfg)
    chunks = []
    for _ in range(count):
        ch = R.Chunk.__new__(R.Chunk)
        ch.context = ctx
        ch.params, ch.grads = [], []
        for _l in range(cfg.layers):
            p = {}
            for k, shp in shapes.items():
                t = torch.randn(shp, device="cuda", generator=gen) * 0.02
                if k in ("ln1_g", "ln2_g"):
                    t += 1.0
                p[k] = t.to(torch.bfloat16)
            ch.params.append(p)
            ch.grads.append({k: torch.zeros(shp, dtype=torch.float32, device="cuda") for k, shp in shapes.items()})
        ch.handle = P.pmc_chunk_create(ctx.ctx, ctx.cfg)
        P.pmc_chunk_bind(ch.handle, [p[k] for p in ch.params for k in R.PARAM_NAMES],
                         [g[k] for g in ch.grads for k in R.PARAM_NAMES])
        ctx.chunks.append(ch)
        chunks.append(ch)
    return chunks, gen


@pytest.mark.timeout(900)
def test_replay_config5_full_size():
    """The full schedule replay at its stated size: 4 simulated devices, 8 two-layer chunks (hidden 4096,
    32 heads, FFN 16384, 2048 tokens, bf16), 16 microbatches, as 1F1B, V-ZB, V-Half and V-Min (and as
    1F1B-V, the fused-backward V-shape block of Appendix H).
    The fp64 oracle of a whole iteration would take hours, so the chain is:
      (i)   a naive run on the GPU (F through all chunks, B back, W at once, microbatch after
            microbatch) in which ONE chunk's pass for microbatch 0 is compared with the oracle in
            full: its output, its input gradient and every parameter gradient, every element;
      (ii)  every schedule's replay must give the naive run's outputs, input gradients and accumulated
            gradients BIT FOR BIT (every chunk's W and B passes run in microbatch order in all of them);
      (iii) the machine's measured peaks per simulated device equal the oracle's accounting, units and
            bytes, and V-Half / V-Min hold 3/4 and 1/2 of 1F1B's worst device (the exact values at
            d = 4 of the paper's Section 3.2)."""
    cfg, d, n = synth.CONFIGS["C5"], 4, 16
    pcfg = R.cfg_from_synth(cfg)
    probe = 3                                            # the chunk checked against the oracle
    scheds = {k: P.pmc_schedule_build(k, d, n) for k in ("1f1b", "vzb", "vhalf", "vmin", "1f1bv")}
    ws = max(P.pmc_replay_workspace_bytes(s, pcfg) for s in scheds.values())
    ctx = R.Context(pcfg, slabs=2 * d * d, workspace_bytes=ws)
    chunks, gen = _gpu_chunks(ctx, cfg, 2 * d, seed=5)
    bf = torch.bfloat16
    xs = [torch.randn(cfg.tokens, cfg.hidden, device="cuda", generator=gen).to(bf) for _ in range(n)]
    dys = [torch.randn(cfg.tokens, cfg.hidden, device="cuda", generator=gen).to(bf) for _ in range(n)]
    handles = [c.handle for c in chunks]

    # (i) naive run
    print("config 5: naive run", flush=True)
    acts = [torch.empty_like(xs[0]) for _ in range(2 * d + 1)]
    grs = [torch.empty_like(xs[0]) for _ in range(2 * d + 1)]
    y_naive, dx_naive, probe_io, probe_grads = [], [], None, None
    for j in range(n):
        acts[0].copy_(xs[j])
        for c in range(2 * d):
            P.stage_forward(handles[c], j, acts[c], acts[c + 1])
        grs[2 * d].copy_(dys[j])
        for c in reversed(range(2 * d)):
            P.stage_backward_input(handles[c], j, grs[c + 1], grs[c])
            P.stage_backward_weight(handles[c], [j])
        y_naive.append(acts[2 * d].clone())
        dx_naive.append(grs[0].clone())
        if j == 0:
            probe_io = [t.clone() for t in (acts[probe], acts[probe + 1], grs[probe + 1], grs[probe])]
            probe_grads = [{k: v.clone() for k, v in g.items()} for g in chunks[probe].grads]
    torch.cuda.synchronize()
    assert P.pmc_pool_live_slabs(ctx.ctx) == 0
    naive = [[{k: v.clone() for k, v in g.items()} for g in ch.grads] for ch in chunks]

    print("config 5: oracle on chunk", probe, flush=True)
    params = [{k: v.float().cpu().numpy() for k, v in p.items()} for p in chunks[probe].params]
    x3, y3, dy3, dx3 = (host(t) for t in probe_io)
    y, dx, ln, wg = oracle_chunk(cfg, params, x3, dy3)
    assert_close(y3, y, "bf16", "C5 probe y")
    assert_close(dx3, dx, "bf16", "C5 probe dx")
    for l in range(cfg.layers):
        for k, v in {**ln[l], **wg[l]}.items():
            assert_close(host(probe_grads[l][k]), v, "bf16", f"C5 probe L{l}.{k}")
    del params, y, dx, ln, wg, probe_grads

    # (ii), (iii) the four schedules
    m = OL.chunk_activation_bytes(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, 2, cfg.microbatch, cfg.ffn)
    st = OL.chunk_stats_bytes(cfg.layers, cfg.heads, cfg.seq, cfg.microbatch)
    assert m == P.pmc_activation_bytes(pcfg) == 537460736
    worst = {}
    for kind, s in scheds.items():
        print("config 5: replay", kind, flush=True)
        for ch in chunks:
            ch.zero_grads()
        yl = [torch.empty_like(t) for t in xs]
        dxf = [torch.empty_like(t) for t in xs]
        report, peaks = P.schedule_replay(ctx.ctx, s, handles, xs, dys, yl, dxf)
        assert report["passes"] == 6 * d * n and P.pmc_pool_live_slabs(ctx.ctx) == 0
        assert [p[0] for p in peaks] == OS.peak_units(kind, d, n)
        assert [(p[1], p[2]) for p in peaks] == OS.peak_bytes(kind, d, n, m, st)
        worst[kind] = max(p[1] for p in peaks)
        for j in range(n):
            assert torch.equal(yl[j], y_naive[j]) and torch.equal(dxf[j], dx_naive[j]), (kind, j)
        for c, ch in enumerate(chunks):
            for l in range(cfg.layers):
                for k in OL.PARAM_NAMES:
                    assert torch.equal(ch.grads[l][k], naive[c][l][k]), (kind, c, l, k)
        P.pmc_schedule_destroy(s)
    assert worst["1f1b"] == worst["vzb"] == 8 * m
    assert worst["vhalf"] * 4 == worst["1f1b"] * 3 and worst["vmin"] * 2 == worst["1f1b"]
    assert worst["1f1bv"] == -(-(4 * d + 2) // 3) * m                     # ceil((4d + 2) / 3) units: 6 of 8 at d = 4
    ctx.close()

"""CPU-only checks of the C-ABI library: it loads without a GPU, exports every symbol the header
declares, and its host-only schedule generator agrees bit for bit with the oracle."""
import os
import re

import pytest

import paper_2405_15362_amd as P
from oracle import layer as OL
from oracle import schedule as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported_and_bound():
    text = open(os.path.join(ROOT, "include", "pmc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b((?:pmc|stage|schedule)_[a-z0-9_]+)\s*\(", text))
    assert len(declared) >= 30
    for name in declared:
        assert hasattr(P.lib, name), f"{name} is declared in pmc.h but not exported"
    assert declared == set(P.EXPORTS), declared ^ set(P.EXPORTS)


@pytest.mark.parametrize("kind", S.KINDS + S.MORE_KINDS)
@pytest.mark.parametrize("d,n", [(1, 3), (2, 4), (3, 7), (4, 16), (6, 13), (8, 32), (9, 20)])
def test_orders_match_oracle(kind, d, n):
    s = P.pmc_schedule_build(kind, d, n)
    try:
        assert P.pmc_schedule_devices(s) == d and P.pmc_schedule_microbatches(s) == n
        assert P.pmc_schedule_num_passes(s) == 6 * d * n
        assert P.pmc_schedule_block(s) == S.block(kind, d)
        passes = S.build(kind, d, n)
        want = [(p.time, p.device, p.op, p.chunk, p.mb, S.model_chunk(kind, d, p.device, p.chunk))
                for p in S.global_order(passes)]
        got = [(p.time, p.device, p.op, p.chunk, p.mb, p.model_chunk) for p in P.pmc_schedule_global_order(s)]
        assert got == want
        for i, order in enumerate(S.device_orders(passes, d)):
            got_i = [(p.time, p.op, p.chunk, p.mb) for p in P.pmc_schedule_device_order(s, i)]
            assert got_i == [(p.time, p.op, p.chunk, p.mb) for p in order]
    finally:
        P.pmc_schedule_destroy(s)


@pytest.mark.parametrize("kind,d,n", [(k, d, n) for k in S.KINDS + S.MORE_KINDS
                                      for d, n in [(2, 4), (4, 16), (5, 11), (8, 24), (64, 256)]
                                      if not (k == "1f1bv" and d == 64)] + [("1f1bv", 16, 64)])
def test_accounting_matches_oracle(kind, d, n):
    m, st = 537460736, 589824
    s = P.pmc_schedule_build(kind, d, n)
    try:
        got = P.pmc_schedule_account(s, m, st)
        units = S.peak_units(kind, d, n)
        bytes_ = S.peak_bytes(kind, d, n, m, st)
        assert [g[0] for g in got] == units
        assert [(g[1], g[2]) for g in got] == bytes_
    finally:
        P.pmc_schedule_destroy(s)


@pytest.mark.parametrize("kind", S.KINDS + S.MORE_KINDS)
@pytest.mark.parametrize("times", [(1.0, 1.0, 1.0), (1.0, 1.1, 0.7), (2.0, 1.0, 0.5)])
def test_makespan_matches_oracle(kind, times):
    for d, n in ((2, 4), (4, 16), (8, 24)):
        s = P.pmc_schedule_build(kind, d, n)
        try:
            assert P.pmc_schedule_makespan(s, *times) == pytest.approx(S.squeezed_makespan(kind, d, n, *times), rel=1e-12)
        finally:
            P.pmc_schedule_destroy(s)


def test_custom_vshape_block_and_collision():
    s = P.pmc_schedule_build_vshape(4, 8, 2, 1, 2, 4, 1)
    ref = P.pmc_schedule_build("vhalf", 4, 8)
    assert P.pmc_schedule_global_order(s) == P.pmc_schedule_global_order(ref)
    P.pmc_schedule_destroy(s)
    P.pmc_schedule_destroy(ref)
    with pytest.raises(P.PmcError) as e:
        P.pmc_schedule_build_vshape(4, 4, 2, 1, 1, 1, 1)
    assert e.value.code == P.PMC_ERR_ILLEGAL_BLOCK
    assert S.vshape_block(4, 2, 1, 1, 1, 1) is None
    # every (a, b, c) below the repeat interval: both sides agree on which blocks are legal
    for a in range(1, 6):
        for b in range(1, 6):
            for c in range(1, 6):
                legal = S.vshape_block(5, 4, 2, a, b, c) is not None
                try:
                    P.pmc_schedule_destroy(P.pmc_schedule_build_vshape(5, 2, 4, 2, a, b, c))
                    assert legal
                except P.PmcError:
                    assert not legal


def test_bad_arguments():
    for args in (("vhalf", 0, 4), ("vhalf", 4, 0), (17, 4, 4)):
        with pytest.raises(P.PmcError) as e:
            P.pmc_schedule_build(*args)
        assert e.value.code == P.PMC_ERR_INVALID
    assert "kind" in P.pmc_last_error()


@pytest.mark.parametrize("name,cfg", [
    ("C1", (1, 256, 4, 1024, 128, 1, "f32")), ("C2", (2, 2048, 16, 8192, 1024, 1, "bf16")),
    ("C3", (4, 4096, 32, 16384, 2048, 1, "bf16")), ("C4", (2, 5120, 40, 20480, 4096, 1, "bf16")),
    ("odd", (3, 192, 3, 320, 40, 2, "bf16"))])
def test_activation_bytes_match_oracle(name, cfg):
    L, h, nh, f, s, mb, dt = cfg
    c = P.make_cfg(L, h, nh, f, s, mb, dt)
    e = 4 if dt == "f32" else 2
    assert P.pmc_activation_bytes(c) == OL.chunk_activation_bytes(L, h, nh, s, e, mb, f)
    assert P.pmc_activation_stats_bytes(c) == OL.chunk_stats_bytes(L, nh, s, mb)
    assert P.pmc_pass_workspace_bytes(c) > 0


def test_bad_cfg_is_rejected():
    assert P.pmc_activation_bytes(P.make_cfg(1, 100, 3, 400, 64)) == 0       # hidden % heads
    assert P.pmc_activation_bytes(P.make_cfg(1, 2048, 4, 8192, 64)) == 0     # head size 512
    assert P.pmc_activation_bytes(P.make_cfg(0, 256, 4, 1024, 64)) == 0
    # bf16, head size 128: a sequence's q|k|v rows (seq x 3 x hidden x 2 bytes) must stay below 2 GB
    assert P.pmc_activation_bytes(P.make_cfg(1, 8192, 64, 8192, 43688)) > 0
    assert P.pmc_activation_bytes(P.make_cfg(1, 8192, 64, 8192, 43696)) == 0
    assert "2 GB" in P.pmc_last_error()
    # widths of the paper's Table 2 models (5120 .. 10240, head size 128) are accepted in bf16 mode
    for hidden, heads in ((5120, 40), (6144, 48), (7168, 56), (10240, 80), (12288, 96)):
        assert P.pmc_activation_bytes(P.make_cfg(2, hidden, heads, 4 * hidden, 2048)) > 0
    assert P.pmc_activation_bytes(P.make_cfg(2, 12296, 53, 8192, 2048)) == 0  # beyond the row kernels' width


@pytest.mark.parametrize("kind", S.KINDS + S.MORE_KINDS)
@pytest.mark.parametrize("d,n", [(1, 3), (2, 5), (3, 7), (4, 16), (6, 24), (8, 20), (9, 12)])
def test_reorder_matches_oracle(kind, d, n):
    """Warm-up / cool-down reordering: the library's orders, cells, accounting and makespan against
    the oracle's, pass for pass."""
    s = P.pmc_schedule_build(kind, d, n)
    r = P.pmc_schedule_reorder(s)
    try:
        ref = S.reordered(kind, d, n)
        got = [(p.time, p.device, p.op, p.chunk, p.mb) for p in P.pmc_schedule_global_order(r)]
        assert got == [(p.time, p.device, p.op, p.chunk, p.mb) for p in S.global_order(ref)]
        for i, order in enumerate(S.device_orders(ref, d)):
            dev = [(p.time, p.op, p.chunk, p.mb, p.model_chunk) for p in P.pmc_schedule_device_order(r, i)]
            assert dev == [(p.time, p.op, p.chunk, p.mb, S.model_chunk(kind, d, i, p.chunk)) for p in order]
        assert [a[0] for a in P.pmc_schedule_account(r, 1000, 40)] == S.peak_units_of(ref, kind, d)
        for times in ((1.0, 1.0, 1.0), (1.0, 1.3, 0.6)):
            assert P.pmc_schedule_makespan(r, *times) == pytest.approx(S.makespan_of(ref, kind, d, *times), rel=1e-12)
        # the input schedule is left as it was
        assert P.pmc_schedule_global_order(s) == P.pmc_schedule_global_order(P.pmc_schedule_build(kind, d, n))
    finally:
        P.pmc_schedule_destroy(s)
        P.pmc_schedule_destroy(r)


def test_reorder_rejects_null():
    with pytest.raises(P.PmcError) as e:
        P.pmc_schedule_reorder(None)
    assert e.value.code == P.PMC_ERR_INVALID


@pytest.mark.parametrize("d,n", [(2, 6), (3, 7)])
@pytest.mark.parametrize("times", [(1.0, 1.0, 1.0), (1.0, 1.3, 0.6)])
@pytest.mark.parametrize("reorder", [True, False])
def test_adaptive_search_matches_oracle(d, n, times, reorder):
    """Appendix A's search: winning block, finish time and pass orders against the oracle's
    exhaustive loop for every memory limit (offsets up to 3 so the oracle finishes in seconds)."""
    for limit in range(3, 2 * d + 1):
        ref = S.adaptive_search(d, n, limit, *times, max_delta=3, reorder=reorder)
        if ref is None:
            with pytest.raises(P.PmcError) as e:
                P.pmc_schedule_search(d, n, limit, *times, max_delta=3, reorder=reorder)
            assert e.value.code == P.PMC_ERR_ILLEGAL_BLOCK
            continue
        sch, res = P.pmc_schedule_search(d, n, limit, *times, max_delta=3, reorder=reorder)
        try:
            got = tuple(res[k] for k in ("split", "delta0_lo", "delta1_lo", "delta0_hi", "delta1_hi", "turn_f", "turn_fb", "turn_b"))
            assert got == ref[1]
            assert res["makespan"] == pytest.approx(ref[0], rel=1e-12)
            assert res["peak_units"] == max(S.peak_units_of(ref[2], "vshape", d)) <= limit
            for i, order in enumerate(S.device_orders(ref[2], d)):
                assert [(p.op, p.chunk, p.mb) for p in P.pmc_schedule_device_order(sch, i)] == [(p.op, p.chunk, p.mb) for p in order]
            assert [a[0] for a in P.pmc_schedule_account(sch, 1000, 40)] == S.peak_units_of(ref[2], "vshape", d)
        finally:
            P.pmc_schedule_destroy(sch)


def test_adaptive_search_larger_and_bad_arguments():
    """d = 4, n = 16 (the replay configuration): monotone in the limit, the uniform named schedules
    never beat it at their own peaks, 6n + d - 1 with room for 2d units."""
    spans = {}
    for limit in (4, 5, 6, 7, 8):
        sch, res = P.pmc_schedule_search(4, 16, limit)
        spans[limit] = res["makespan"]
        assert res["peak_units"] <= limit and res["feasible"] >= 1
        assert P.pmc_schedule_num_passes(sch) == 6 * 4 * 16
        P.pmc_schedule_destroy(sch)
    assert all(spans[a] >= spans[b] for a, b in zip((4, 5, 6, 7), (5, 6, 7, 8)))
    assert spans[8] == 6 * 16 + 3
    for kind, limit in (("vmin", 4), ("vhalf", 6), ("vzb", 8)):
        assert spans[limit] <= S.makespan_of(S.reordered(kind, 4, 16), kind, 4)
    for bad in ((0, 4, 4), (4, 0, 4)):
        with pytest.raises(P.PmcError):
            P.pmc_schedule_search(*bad)
    with pytest.raises(P.PmcError):
        P.pmc_schedule_search(4, 8, 8, max_delta=0)
    with pytest.raises(P.PmcError):
        P.pmc_schedule_search(4, 8, 8, t_f=-1.0)



def test_tuning_switches():
    """Switches are process-wide integers; -1 hands the choice back; unknown names and values out of
    range are refused (no GPU needed: nothing is launched)."""
    for name, good, bad in (("gemm_tile", 4, 5), ("gemm_wgrad", 2, 3), ("attn_shape", 2, 3), ("w_streams", 1, 0),
                            ("gemm_group", 8, 0)):
        P.pmc_tuning_set(name, good)
        assert P.pmc_tuning_get(name) == good
        with pytest.raises(P.PmcError) as e:
            P.pmc_tuning_set(name, bad)
        assert e.value.code == P.PMC_ERR_INVALID and P.pmc_tuning_get(name) == good
        P.pmc_tuning_set(name, -1)
        assert P.pmc_tuning_get(name) == -1
    with pytest.raises(P.PmcError):
        P.pmc_tuning_set("no_such_switch", 1)


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 on its own (no C++ or torch types)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-fsyntax-only", "-x", "c",
                        os.path.join(ROOT, "include", "pmc.h")], capture_output=True, text=True)
    assert r.returncode == 0 and not r.stderr.strip(), r.stderr

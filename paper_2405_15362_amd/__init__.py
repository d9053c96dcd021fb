"""Python binding of libpmc.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see include/pmc.h); tensors are
torch tensors on the GPU whose data_ptr() is handed over, and every step of F / B / W and of the
schedule replay runs inside the library's HIP kernels.  There is no fallback: if the library has
not been built (python paper_2405_15362_amd/build.py) importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpmc.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2405_15362_amd/build.py`")
lib = C.CDLL(LIB_PATH)

PMC_F32, PMC_BF16 = 0, 1
PMC_1F1B, PMC_VZB, PMC_VHALF, PMC_VMIN, PMC_1F1BV = 0, 1, 2, 3, 4
KINDS = {"1f1b": PMC_1F1B, "vzb": PMC_VZB, "vhalf": PMC_VHALF, "vmin": PMC_VMIN, "1f1bv": PMC_1F1BV}
PMC_F, PMC_B, PMC_W = 0, 1, 2
OPS = "FBW"
PARAMS_PER_LAYER = 12
EPI_NONE, EPI_BIAS, EPI_BIAS_RESID, EPI_BIAS_GELU, EPI_DGELU, EPI_ACCUM_F32, EPI_BIAS_GELU_GRAD, EPI_MUL = range(8)
REPLAY_TIME_PASSES = 1
PMC_OK, PMC_ERR_INVALID, PMC_ERR_STATE, PMC_ERR_NOMEM, PMC_ERR_HIP, PMC_ERR_ILLEGAL_BLOCK = 0, -1, -2, -3, -4, -5


class PmcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"pmc error {code}: {msg}")
        self.code = code


class ChunkCfg(C.Structure):
    _fields_ = [("layers", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32), ("ffn", C.c_int32),
                ("seq", C.c_int32), ("microbatch", C.c_int32), ("dtype", C.c_int32), ("causal", C.c_int32),
                ("ln_eps", C.c_float)]


class Pass(C.Structure):
    _fields_ = [("time", C.c_int32), ("device", C.c_int32), ("op", C.c_int32), ("chunk", C.c_int32),
                ("mb", C.c_int32), ("model_chunk", C.c_int32)]


class DevicePeak(C.Structure):
    _fields_ = [("peak_live_units", C.c_int64), ("peak_live_bytes", C.c_int64), ("peak_tensor_bytes", C.c_int64)]


class TraceRec(C.Structure):
    _fields_ = [("op", C.c_int32), ("pass_", C.c_int32), ("m", C.c_int32), ("n", C.c_int32), ("k", C.c_int32),
                ("variant", C.c_int32), ("ms", C.c_float)]


class ReplayReport(C.Structure):
    _fields_ = [("ms_total", C.c_double), ("ms_f", C.c_double), ("ms_b", C.c_double), ("ms_w", C.c_double),
                ("passes", C.c_int32), ("devices", C.c_int32), ("transit_peak_bytes", C.c_int64)]


_vp, _i32, _i64, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
_SIGS = {
    "pmc_last_error": (C.c_char_p, []),
    "pmc_create": (C.c_int, [_vp, C.POINTER(_vp)]),
    "pmc_destroy": (None, [_vp]),
    "pmc_pool_attach": (C.c_int, [_vp, _vp, _sz, _sz]),
    "pmc_pool_live_slabs": (_i64, [_vp]),
    "pmc_pool_peak_slabs": (_i64, [_vp]),
    "pmc_pool_reset_peak": (None, [_vp]),
    "pmc_workspace_attach": (C.c_int, [_vp, _vp, _sz]),
    "pmc_activation_bytes": (_sz, [C.POINTER(ChunkCfg)]),
    "pmc_activation_stats_bytes": (_sz, [C.POINTER(ChunkCfg)]),
    "pmc_pass_workspace_bytes": (_sz, [C.POINTER(ChunkCfg)]),
    "pmc_chunk_create": (C.c_int, [_vp, C.POINTER(ChunkCfg), C.POINTER(_vp)]),
    "pmc_chunk_destroy": (None, [_vp]),
    "pmc_chunk_bind": (C.c_int, [_vp, C.POINTER(_vp), C.POINTER(_vp)]),
    "stage_forward": (C.c_int, [_vp, _i32, _vp, _vp]),
    "stage_forward_on": (C.c_int, [_vp, _i32, _vp, _vp, _i32]),
    "stage_backward_input": (C.c_int, [_vp, _i32, _vp, _vp]),
    "stage_backward_weight": (C.c_int, [_vp, C.POINTER(_i32), _i32]),
    "stage_abandon": (C.c_int, [_vp, _i32]),
    "pmc_tuning_set": (C.c_int, [C.c_char_p, _i32]),
    "pmc_tuning_get": (C.c_int, [C.c_char_p, C.POINTER(_i32)]),
    "pmc_schedule_build": (C.c_int, [_i32, _i32, _i32, C.POINTER(_vp)]),
    "pmc_schedule_build_vshape": (C.c_int, [_i32] * 7 + [C.POINTER(_vp)]),
    "pmc_schedule_reorder": (C.c_int, [_vp, C.POINTER(_vp)]),
    "pmc_schedule_search": (C.c_int, [_i32, _i32, C.c_int64, C.c_double, C.c_double, C.c_double, _i32, _i32, _vp,
                                      C.POINTER(_vp)]),
    "pmc_schedule_destroy": (None, [_vp]),
    "pmc_schedule_devices": (_i32, [_vp]),
    "pmc_schedule_microbatches": (_i32, [_vp]),
    "pmc_schedule_num_passes": (_i32, [_vp]),
    "pmc_schedule_block": (C.c_int, [_vp, C.POINTER(_i32), _i32]),
    "pmc_schedule_device_order": (C.c_int, [_vp, _i32, C.POINTER(Pass), _i32]),
    "pmc_schedule_global_order": (C.c_int, [_vp, C.POINTER(Pass), _i32]),
    "pmc_schedule_account": (C.c_int, [_vp, _i64, _i64, C.POINTER(DevicePeak), _i32]),
    "pmc_schedule_makespan": (C.c_int, [_vp, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double)]),
    "pmc_replay_workspace_bytes": (_sz, [_vp, C.POINTER(ChunkCfg)]),
    "schedule_replay": (C.c_int, [_vp, _vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_vp),
                                  C.POINTER(_vp), C.c_uint32, C.POINTER(ReplayReport), C.POINTER(DevicePeak), _i32]),
    "pmc_trace_begin": (C.c_int, [_vp, _i32]),
    "pmc_trace_end": (C.c_int, [_vp, C.POINTER(TraceRec), _i32, C.POINTER(_i32)]),
    "pmc_gemm": (C.c_int, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _i32, _vp, _i32, _vp, _i32, _i32, _vp, _vp, _vp]),
    "pmc_gemm_grouped_wgrad": (C.c_int, [_vp, _i32, _i32, _i32, _i32, C.POINTER(_vp), _i32, C.POINTER(_vp), _i32, _vp, _i32]),
    "pmc_layernorm_forward": (C.c_int, [_vp, _i32, _i32, _i32, _vp, _vp, _vp, C.c_float, _vp, _vp, _vp, _vp]),
    "pmc_layernorm_backward": (C.c_int, [_vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "pmc_layernorm_backward_static": (C.c_int, [_vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "pmc_attention_forward": (C.c_int, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp]),
    "pmc_attention_backward": (C.c_int, [_vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp]),
    "pmc_column_sum": (C.c_int, [_vp, _i32, _i32, _i32, _vp, _i32, _vp]),
}
EXPORTS = tuple(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


def pmc_last_error() -> str:
    return lib.pmc_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise PmcError(rc, pmc_last_error())


def _ptr(t) -> int | None:
    """Device pointer of a torch tensor (None stays NULL)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _ptr_array(items):
    arr = (_vp * len(items))()
    for i, t in enumerate(items):
        arr[i] = _ptr(t)
    return arr


def make_cfg(layers, hidden, heads, ffn, seq, microbatch=1, dtype="bf16", causal=True, ln_eps=1e-5) -> ChunkCfg:
    return ChunkCfg(layers, hidden, heads, ffn, seq, microbatch, PMC_BF16 if dtype == "bf16" else PMC_F32,
                    1 if causal else 0, ln_eps)


# ---- context ---------------------------------------------------------------------------------

def pmc_create(hip_stream: int | None = None):
    out = _vp()
    _check(lib.pmc_create(hip_stream, C.byref(out)))
    return out


def pmc_destroy(ctx) -> None:
    lib.pmc_destroy(ctx)


def pmc_pool_attach(ctx, arena, slab_bytes: int) -> None:
    _check(lib.pmc_pool_attach(ctx, _ptr(arena), arena.numel() * arena.element_size(), slab_bytes))


def pmc_pool_live_slabs(ctx) -> int:
    return lib.pmc_pool_live_slabs(ctx)


def pmc_pool_peak_slabs(ctx) -> int:
    return lib.pmc_pool_peak_slabs(ctx)


def pmc_pool_reset_peak(ctx) -> None:
    lib.pmc_pool_reset_peak(ctx)


def pmc_workspace_attach(ctx, workspace) -> None:
    _check(lib.pmc_workspace_attach(ctx, _ptr(workspace), workspace.numel() * workspace.element_size()))


def pmc_activation_bytes(cfg: ChunkCfg) -> int:
    return lib.pmc_activation_bytes(C.byref(cfg))


def pmc_activation_stats_bytes(cfg: ChunkCfg) -> int:
    return lib.pmc_activation_stats_bytes(C.byref(cfg))


def pmc_pass_workspace_bytes(cfg: ChunkCfg) -> int:
    return lib.pmc_pass_workspace_bytes(C.byref(cfg))


# ---- chunks ----------------------------------------------------------------------------------

def pmc_chunk_create(ctx, cfg: ChunkCfg):
    out = _vp()
    _check(lib.pmc_chunk_create(ctx, C.byref(cfg), C.byref(out)))
    return out


def pmc_chunk_destroy(chunk) -> None:
    lib.pmc_chunk_destroy(chunk)


def pmc_chunk_bind(chunk, params, grads) -> None:
    """params / grads: flat lists of layers * 12 tensors in the header's parameter order."""
    _check(lib.pmc_chunk_bind(chunk, _ptr_array(params), _ptr_array(grads)))


def stage_forward(chunk, mb: int, x, y, device: int | None = None) -> None:
    if device is None:
        _check(lib.stage_forward(chunk, mb, _ptr(x), _ptr(y)))
    else:
        _check(lib.stage_forward_on(chunk, mb, _ptr(x), _ptr(y), device))


def stage_backward_input(chunk, mb: int, dy, dx) -> None:
    _check(lib.stage_backward_input(chunk, mb, _ptr(dy), _ptr(dx)))


def stage_backward_weight(chunk, mbs) -> None:
    mbs = list(mbs)
    arr = (_i32 * len(mbs))(*mbs)
    _check(lib.stage_backward_weight(chunk, arr, len(mbs)))


def stage_abandon(chunk, mb: int) -> None:
    _check(lib.stage_abandon(chunk, mb))


def pmc_tuning_set(name: str, value: int = -1) -> None:
    """Process-wide tuning switch (see pmc.h); -1 hands the choice back to the library."""
    _check(lib.pmc_tuning_set(name.encode(), value))


def pmc_tuning_get(name: str) -> int:
    out = _i32()
    _check(lib.pmc_tuning_get(name.encode(), C.byref(out)))
    return out.value


# ---- schedules (host only) ----------------------------------------------------------------------

@dataclass(frozen=True)
class PassRec:
    time: int
    device: int
    op: str
    chunk: int
    mb: int
    model_chunk: int


def _rec(p: Pass) -> PassRec:
    return PassRec(p.time, p.device, OPS[p.op], p.chunk, p.mb, p.model_chunk)


def pmc_schedule_build(kind, d: int, n: int):
    out = _vp()
    _check(lib.pmc_schedule_build(KINDS[kind] if isinstance(kind, str) else kind, d, n, C.byref(out)))
    return out


def pmc_schedule_build_vshape(d, n, delta0, delta1, turn_f, turn_fb, turn_b):
    out = _vp()
    _check(lib.pmc_schedule_build_vshape(d, n, delta0, delta1, turn_f, turn_fb, turn_b, C.byref(out)))
    return out


def pmc_schedule_reorder(s):
    """A new schedule with the warm-up and cool-down reordered; the caller destroys it."""
    out = _vp()
    _check(lib.pmc_schedule_reorder(s, C.byref(out)))
    return out


class SearchResult(C.Structure):
    _fields_ = [("split", C.c_int32), ("delta0_lo", C.c_int32), ("delta1_lo", C.c_int32), ("delta0_hi", C.c_int32),
                ("delta1_hi", C.c_int32), ("turn_f", C.c_int32), ("turn_fb", C.c_int32), ("turn_b", C.c_int32),
                ("peak_units", C.c_int64), ("makespan", C.c_double), ("candidates", C.c_int64), ("feasible", C.c_int64)]


def pmc_schedule_search(d, n, limit_units, t_f=1.0, t_b=1.0, t_w=1.0, max_delta=6, reorder=True):
    """Adaptive V-shape search under a memory limit: (schedule handle, dict of the winning block)."""
    out, res = _vp(), SearchResult()
    _check(lib.pmc_schedule_search(d, n, limit_units, t_f, t_b, t_w, max_delta, int(reorder), C.byref(res), C.byref(out)))
    return out, {k: getattr(res, k) for k, _ in SearchResult._fields_}


def pmc_schedule_destroy(s) -> None:
    lib.pmc_schedule_destroy(s)


def pmc_schedule_devices(s) -> int:
    return lib.pmc_schedule_devices(s)


def pmc_schedule_microbatches(s) -> int:
    return lib.pmc_schedule_microbatches(s)


def pmc_schedule_num_passes(s) -> int:
    return lib.pmc_schedule_num_passes(s)


def pmc_schedule_block(s) -> dict:
    d = pmc_schedule_devices(s)
    buf = (_i32 * (6 * d))()
    _check(lib.pmc_schedule_block(s, buf, 6 * d))
    rows = [("F", 0), ("F", 1), ("B", 1), ("B", 0), ("W", 1), ("W", 0)]
    return {key: [buf[r * d + i] for i in range(d)] for r, key in enumerate(rows)}


def pmc_schedule_device_order(s, device: int) -> list[PassRec]:
    cap = 6 * pmc_schedule_microbatches(s)
    buf = (Pass * cap)()
    _check(lib.pmc_schedule_device_order(s, device, buf, cap))
    return [_rec(p) for p in buf]


def pmc_schedule_global_order(s) -> list[PassRec]:
    cap = pmc_schedule_num_passes(s)
    buf = (Pass * cap)()
    _check(lib.pmc_schedule_global_order(s, buf, cap))
    return [_rec(p) for p in buf]


def pmc_schedule_account(s, unit_bytes: int, stats_bytes: int) -> list[tuple[int, int, int]]:
    d = pmc_schedule_devices(s)
    buf = (DevicePeak * d)()
    _check(lib.pmc_schedule_account(s, unit_bytes, stats_bytes, buf, d))
    return [(p.peak_live_units, p.peak_live_bytes, p.peak_tensor_bytes) for p in buf]


def pmc_schedule_makespan(s, t_f=1.0, t_b=1.0, t_w=1.0) -> float:
    out = C.c_double()
    _check(lib.pmc_schedule_makespan(s, t_f, t_b, t_w, C.byref(out)))
    return out.value


# ---- replay ----------------------------------------------------------------------------------

def pmc_replay_workspace_bytes(s, cfg: ChunkCfg) -> int:
    return lib.pmc_replay_workspace_bytes(s, C.byref(cfg))


def schedule_replay(ctx, s, chunks, x, dy_last, y_last=None, dx_first=None, flags: int = 0):
    """Returns (report dict, per-device list of (units, bytes, tensor_bytes))."""
    d = pmc_schedule_devices(s)
    rep = ReplayReport()
    peaks = (DevicePeak * d)()
    ch = (_vp * len(chunks))(*[c.value if isinstance(c, _vp) else c for c in chunks])
    _check(lib.schedule_replay(ctx, s, ch, _ptr_array(x), _ptr_array(dy_last),
                               _ptr_array(y_last) if y_last is not None else None,
                               _ptr_array(dx_first) if dx_first is not None else None,
                               flags, C.byref(rep), peaks, d))
    report = {f: getattr(rep, f) for f, _ in ReplayReport._fields_}
    return report, [(p.peak_live_units, p.peak_live_bytes, p.peak_tensor_bytes) for p in peaks]


# ---- tracing ---------------------------------------------------------------------------------

TRACE_OPS = ("gemm", "ln_fwd", "ln_bwd", "attn_fwd", "attn_bwd", "colsum", "copy")


def pmc_trace_begin(ctx, capacity: int = 4096) -> None:
    _check(lib.pmc_trace_begin(ctx, capacity))


def pmc_trace_end(ctx, capacity: int = 4096) -> list[dict]:
    buf = (TraceRec * capacity)()
    n = _i32()
    _check(lib.pmc_trace_end(ctx, buf, capacity, C.byref(n)))
    return [dict(op=TRACE_OPS[r.op], pass_=OPS[r.pass_], m=r.m, n=r.n, k=r.k, trans_a=bool(r.variant & 1),
                 trans_b=bool(r.variant & 2), epilogue=r.variant >> 2, ms=r.ms) for r in buf[:n.value]]


# ---- single operations -----------------------------------------------------------------------

def _dt(t) -> int:
    import torch
    return PMC_BF16 if t.dtype == torch.bfloat16 else PMC_F32


def pmc_gemm(ctx, a, b, c, trans_a=False, trans_b=False, epilogue=EPI_NONE, bias=None, resid=None, aux=None) -> None:
    """c[M,N] = op(a) . op(b) with the given epilogue; shapes are read from the tensors."""
    M, N = c.shape
    K = a.shape[0] if trans_a else a.shape[1]
    _check(lib.pmc_gemm(ctx, _dt(a), int(trans_a), int(trans_b), M, N, K, _ptr(a), a.stride(0), _ptr(b), b.stride(0),
                        _ptr(c), c.stride(0), epilogue, _ptr(bias), _ptr(resid), _ptr(aux)))


def pmc_gemm_grouped_wgrad(ctx, a_list, b_list, c) -> None:
    """c[M,N] (fp32) += sum_i a_i^T . b_i with a_i [K,M], b_i [K,N] bf16: one product over the pieces."""
    M, N = c.shape
    K = a_list[0].shape[0]
    _check(lib.pmc_gemm_grouped_wgrad(ctx, M, N, K, len(a_list), _ptr_array(a_list), a_list[0].stride(0),
                                      _ptr_array(b_list), b_list[0].stride(0), _ptr(c), c.stride(0)))


def pmc_layernorm_forward(ctx, x, gain, bias, eps, y, mean, rstd, x_copy=None) -> None:
    rows, h = x.shape
    _check(lib.pmc_layernorm_forward(ctx, _dt(x), rows, h, _ptr(x), _ptr(gain), _ptr(bias), eps, _ptr(y), _ptr(mean),
                                     _ptr(rstd), _ptr(x_copy)))


def pmc_layernorm_backward(ctx, dy, x, gain, mean, rstd, resid, dx, dgain, dbias) -> None:
    rows, h = x.shape
    _check(lib.pmc_layernorm_backward(ctx, _dt(x), rows, h, _ptr(dy), _ptr(x), _ptr(gain), _ptr(mean), _ptr(rstd),
                                      _ptr(resid), _ptr(dx), _ptr(dgain), _ptr(dbias)))


def pmc_layernorm_backward_static(ctx, dy, x, gain, mean, rstd, resid, dx, dgain, dbias) -> None:
    """pmc_layernorm_backward with the library's built-in scratch array (no workspace needed)."""
    rows, h = x.shape
    _check(lib.pmc_layernorm_backward_static(ctx, _dt(x), rows, h, _ptr(dy), _ptr(x), _ptr(gain), _ptr(mean), _ptr(rstd),
                                             _ptr(resid), _ptr(dx), _ptr(dgain), _ptr(dbias)))


def pmc_attention_forward(ctx, qkv, o, lse, batch, seq, heads, head_dim, causal=True) -> None:
    _check(lib.pmc_attention_forward(ctx, _dt(qkv), batch, seq, heads, head_dim, int(causal), _ptr(qkv), _ptr(o), _ptr(lse)))


def pmc_attention_backward(ctx, qkv, o, lse, d_o, dqkv, batch, seq, heads, head_dim, causal=True) -> None:
    _check(lib.pmc_attention_backward(ctx, _dt(qkv), batch, seq, heads, head_dim, int(causal), _ptr(qkv), _ptr(o),
                                      _ptr(lse), _ptr(d_o), _ptr(dqkv)))


def pmc_column_sum(ctx, a, out) -> None:
    rows, n = a.shape
    _check(lib.pmc_column_sum(ctx, _dt(a), rows, n, _ptr(a), a.stride(0), _ptr(out)))

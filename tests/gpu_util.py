"""Shared helpers of the GPU parity tests (marshalling and error measures only)."""
import os

import numpy as np
import torch

import synth
from oracle import layer as OL


def rel_l2(got, want) -> float:
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    denom = np.linalg.norm(want)
    return float(np.linalg.norm(got - want) / denom) if denom > 0 else float(np.linalg.norm(got))


def dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t.contiguous()


def host(t) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def tol(dtype) -> float:
    """spec tolerances: rel-L2 <= 2e-2 for bf16 storage, <= 1e-5 in fp32 mode."""
    return 2e-2 if dtype == "bf16" else 1e-5


# Element-wise and block-wise bounds that stand beside the whole-tensor norm.  A whole-tensor rel-L2
# of 2e-2 lets 4e-4 of a tensor's energy be garbage (a zeroed tile, a dropped slab of rows); these
# bounds do not.  With s = rms(want) of the whole tensor (or the `scale` the caller gives, for tensors
# that are zero by construction, such as the query gradient of a one-token sequence):
#   block:   every 32-row x 128-column block (128 elements of a vector) has
#            rms(got - want) over the block <= BLOCK[dtype] * max(rms(want) over the block, s)
#   element: |got - want| <= RTOL[dtype] * |want| + ATOL[dtype] * s
# bf16 results carry one rounding to bf16 of their own (2^-9 relative) on top of the roundings of
# every bf16 tensor upstream, which appear as noise with an ABSOLUTE level of a few 1e-3 s whatever
# the element's own size (so blocks and elements near zero are held to s, not to themselves), and
# with heavy tails in rows that LayerNorm's backward amplifies.  Measured on the GPU over all cases:
# whole-tensor up to 1.2e-2 (4 layers deep), worst block 1.3e-2 s, worst element 0.13 s + 0.03 |want|.
# A zeroed or stale 32 x 128 tile has a block error of about s (30 x the bound); a corrupted element is
# off by about s (4 x the bound).  fp32 mode: sums of up to a few thousand fp32 products, measured
# 7e-7 whole-tensor, worst block 8e-7 s, worst element 5e-6 s.
BLOCK = {"bf16": 3e-2, "f32": 2e-5}
RTOL = {"bf16": 5e-2, "f32": 1e-4}
ATOL = {"bf16": 0.25, "f32": 1e-4}
_REPORT = bool(os.environ.get("PMC_PARITY_REPORT"))


def closeness(got, want, dtype, atol_scale=1.0, scale=None):
    """(whole-tensor rel-L2, worst block / its bound, worst element / its bound) of got against want."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.ndim == 1:
        got, want = got[None, :], want[None, :]
    else:
        got, want = got.reshape(-1, got.shape[-1]), want.reshape(-1, want.shape[-1])
    err = got - want
    assert np.isfinite(err).all(), "non-finite values"
    rms = float(np.sqrt(np.mean(want * want)))
    s = float(scale) if scale is not None else rms
    assert s > 0, "reference tensor is identically zero: give a scale"
    whole = float(np.linalg.norm(err) / np.linalg.norm(want)) if rms > 1e-3 * s else float(np.linalg.norm(err) / (s * np.sqrt(err.size)))
    # element-wise
    bound = atol_scale * (RTOL[dtype] * np.abs(want) + ATOL[dtype] * s)
    elem = float(np.max(np.abs(err) / bound))
    # block-wise: pad to whole 32 x 128 blocks with zeros (zeros add nothing to either sum)
    r, c = err.shape
    br, bc = min(32, r), min(128, c)
    R, Cc = -(-r // br) * br, -(-c // bc) * bc

    def block_energy(a):
        sq = np.zeros((R, Cc))
        sq[:r, :c] = a * a
        return sq.reshape(R // br, br, Cc // bc, bc).sum(axis=(1, 3))

    e2, w2 = block_energy(err), block_energy(want)
    floor2 = s * s * br * bc
    block = float(np.sqrt(np.max(e2 / np.maximum(w2, floor2))))
    return whole, block / (atol_scale * BLOCK[dtype]), elem


def assert_close(got, want, dtype, name="", atol_scale=1.0, whole_tol=None, scale=None):
    """Element by element: whole-tensor rel-L2 within the benchmark spec's tolerance (relative to `scale`
    where the reference is zero by construction), every 32 x 128 block within BLOCK, every element
    within RTOL |want| + ATOL s; atol_scale widens the block and element bounds."""
    whole, block, elem = closeness(got, want, dtype, atol_scale, scale)
    if _REPORT:
        print(f"parity {name}: shape {np.shape(want)} whole {whole:.3e} block {block:.3f} elem {elem:.3f}", flush=True)
    limit = whole_tol if whole_tol is not None else tol(dtype)
    assert whole <= limit, f"{name}: whole-tensor rel-L2 {whole:.3e} > {limit:.1e}"
    assert block <= 1.0, f"{name}: worst 32x128 block at {block:.2f} of its bound"
    assert elem <= 1.0, f"{name}: worst element at {elem:.2f} of its bound"


def mat(key, shape, dtype, scale=1.0):
    return synth.matrix(key, shape, scale, bf16=(dtype == "bf16"))


def oracle_chunk(cfg, params, x, dy):
    """F, B, W of the oracle in fp64 on (bf16-representable) fp32 inputs."""
    p64 = OL.cast_params(params)
    y, saved = OL.chunk_forward(x.astype(np.float64), p64, cfg.heads, cfg.causal, cfg.ln_eps, cfg.microbatch)
    dx, stash, ln = OL.chunk_backward_input(dy.astype(np.float64), p64, saved, cfg.heads, cfg.microbatch)
    wg = OL.chunk_backward_weight(saved, stash)
    return y, dx, ln, wg


class tuned:
    """Sets process-wide tuning switches of the library for a with-block (or until reset()) and hands
    the choice back to the library afterwards."""
    NAMES = ("gemm_tile", "gemm_group", "gemm_wgrad", "attn_shape", "w_streams")

    def __init__(self, **switches):
        self.switches = switches

    def __enter__(self):
        import paper_2405_15362_amd as P
        for k, v in self.switches.items():
            P.pmc_tuning_set(k, -1 if v is None else int(v))
        return self

    def __exit__(self, *exc):
        tuned.reset()
        return False

    @staticmethod
    def reset():
        import paper_2405_15362_amd as P
        for k in tuned.NAMES:
            P.pmc_tuning_set(k, -1)

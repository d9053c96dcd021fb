"""Shared helpers of the GPU parity tests (marshalling and error norms only)."""
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


def mat(key, shape, dtype, scale=1.0):
    return synth.matrix(key, shape, scale, bf16=(dtype == "bf16"))


def oracle_chunk(cfg, params, x, dy):
    """F, B, W of the oracle in fp64 on (bf16-representable) fp32 inputs."""
    p64 = OL.cast_params(params)
    y, saved = OL.chunk_forward(x.astype(np.float64), p64, cfg.heads, cfg.causal, cfg.ln_eps, cfg.microbatch)
    dx, stash, ln = OL.chunk_backward_input(dy.astype(np.float64), p64, saved, cfg.heads, cfg.microbatch)
    wg = OL.chunk_backward_weight(saved, stash)
    return y, dx, ln, wg

"""Device-memory plumbing around the C ABI: torch owns parameters, gradient accumulators, the
activation pool and the workspace; the library borrows their pointers.  No arithmetic happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import (PARAMS_PER_LAYER, make_cfg, pmc_activation_bytes, pmc_chunk_bind, pmc_chunk_create,
               pmc_chunk_destroy, pmc_create, pmc_destroy, pmc_pass_workspace_bytes, pmc_pool_attach,
               pmc_workspace_attach)

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


def torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_device(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Host fp32 array -> contiguous GPU tensor in the storage type."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda").to(torch_dtype(dtype)).contiguous()


class Context:
    """A library context on torch's current stream with a pool of `slabs` units and a workspace."""

    def __init__(self, cfg, slabs: int, workspace_bytes: int | None = None):
        self.cfg = cfg
        self.ctx = pmc_create(torch.cuda.current_stream().cuda_stream or None)
        self.unit_bytes = pmc_activation_bytes(cfg)
        if self.unit_bytes == 0:
            raise ValueError("unsupported chunk configuration")
        slab = (self.unit_bytes + 255) // 256 * 256
        self.arena = torch.empty(slab * slabs, dtype=torch.uint8, device="cuda")
        pmc_pool_attach(self.ctx, self.arena, self.unit_bytes)
        ws = workspace_bytes if workspace_bytes is not None else pmc_pass_workspace_bytes(cfg)
        self.workspace = torch.empty(max(ws, 256), dtype=torch.uint8, device="cuda")
        pmc_workspace_attach(self.ctx, self.workspace)
        self.chunks = []

    def add_chunk(self, layer_params: list[dict], dtype: str):
        ch = Chunk(self, layer_params, dtype)
        self.chunks.append(ch)
        return ch

    def close(self):
        for ch in self.chunks:
            ch.close()
        self.chunks = []
        if self.ctx is not None:
            pmc_destroy(self.ctx)
            self.ctx = None


class Chunk:
    """One chunk: parameters (storage type) and fp32 gradient accumulators on the GPU, bound."""

    def __init__(self, context: Context, layer_params: list[dict], dtype: str):
        self.context = context
        self.params = [{k: to_device(p[k], dtype) for k in PARAM_NAMES} for p in layer_params]
        self.grads = [{k: torch.zeros(p[k].shape, dtype=torch.float32, device="cuda") for k in PARAM_NAMES}
                      for p in layer_params]
        self.handle = pmc_chunk_create(context.ctx, context.cfg)
        flat_p = [p[k] for p in self.params for k in PARAM_NAMES]
        flat_g = [g[k] for g in self.grads for k in PARAM_NAMES]
        assert len(flat_p) == PARAMS_PER_LAYER * len(layer_params)
        pmc_chunk_bind(self.handle, flat_p, flat_g)

    def zero_grads(self):
        for g in self.grads:
            for t in g.values():
                t.zero_()

    def grads_numpy(self):
        return [{k: v.cpu().numpy().astype(np.float64) for k, v in g.items()} for g in self.grads]

    def close(self):
        if self.handle is not None:
            pmc_chunk_destroy(self.handle)
            self.handle = None


def cfg_from_synth(c) -> "ChunkCfg":
    return make_cfg(c.layers, c.hidden, c.heads, c.ffn, c.seq, c.microbatch, c.dtype, c.causal, c.ln_eps)

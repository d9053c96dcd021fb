"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module holds no arithmetic of the method itself: it only draws random tensors with the
shapes and distributions of a GPT-like pipeline chunk (weights N(0, 0.02^2), LayerNorm gains
1 + N(0, 0.02^2), activations and upstream gradients N(0, 1)) and, for the bf16 storage mode,
rounds them to bf16-representable fp32 values so that both consumers start from identical numbers.

Every tensor gets its own PRNG stream, keyed by (config id, tensor name, chunk, layer/microbatch).
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass

import numpy as np

# Order of the per-layer parameter tensors across the C ABI and in the oracle.
PARAM_NAMES = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2",
)


@dataclass(frozen=True)
class ChunkCfg:
    """Shape of one pipeline chunk (a run of identical pre-LN transformer layers)."""
    layers: int
    hidden: int
    heads: int
    ffn: int
    seq: int
    microbatch: int = 1
    dtype: str = "bf16"      # "f32" or "bf16" (bf16 storage, fp32 accumulate)
    causal: bool = True
    ln_eps: float = 1e-5

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    @property
    def tokens(self) -> int:
        return self.seq * self.microbatch


# The five workload shapes the build is measured and parity-tested on.
CONFIGS = {
    "C1": ChunkCfg(layers=1, hidden=256, heads=4, ffn=1024, seq=128, dtype="f32"),
    "C2": ChunkCfg(layers=2, hidden=2048, heads=16, ffn=8192, seq=1024, dtype="bf16"),
    "C3": ChunkCfg(layers=4, hidden=4096, heads=32, ffn=16384, seq=2048, dtype="bf16"),
    "C4": ChunkCfg(layers=2, hidden=5120, heads=40, ffn=20480, seq=4096, dtype="bf16"),
    "C5": ChunkCfg(layers=2, hidden=4096, heads=32, ffn=16384, seq=2048, dtype="bf16"),
}


def param_shapes(cfg: ChunkCfg) -> dict[str, tuple[int, ...]]:
    h, f = cfg.hidden, cfg.ffn
    return {
        "ln1_g": (h,), "ln1_b": (h,),
        "w_qkv": (h, 3 * h), "b_qkv": (3 * h,),
        "w_o": (h, h), "b_o": (h,),
        "ln2_g": (h,), "ln2_b": (h,),
        "w_1": (h, f), "b_1": (f,),
        "w_2": (f, h), "b_2": (h,),
    }


def _rng(*key) -> np.random.Generator:
    digest = hashlib.sha256(repr(key).encode()).digest()
    seed = int.from_bytes(digest[:16], "little")
    return np.random.Generator(np.random.Philox(seed))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    bits = (bits + 0x7FFF + lsb) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(a.shape)


def _finish(a: np.ndarray, cfg: ChunkCfg) -> np.ndarray:
    a = a.astype(np.float32)
    return round_to_bf16(a) if cfg.dtype == "bf16" else a


def layer_params(cfg: ChunkCfg, config_id: str, chunk: int, layer: int) -> dict[str, np.ndarray]:
    """Parameters of one layer as fp32 arrays (bf16-representable in bf16 mode)."""
    out = {}
    for name, shape in param_shapes(cfg).items():
        g = _rng(config_id, "param", name, chunk, layer)
        v = g.standard_normal(shape, dtype=np.float32) * np.float32(0.02)
        if name in ("ln1_g", "ln2_g"):
            v = v + np.float32(1.0)
        out[name] = _finish(v, cfg)
    return out


def chunk_params(cfg: ChunkCfg, config_id: str, chunk: int = 0) -> list[dict[str, np.ndarray]]:
    return [layer_params(cfg, config_id, chunk, l) for l in range(cfg.layers)]


def chunk_input(cfg: ChunkCfg, config_id: str, microbatch: int = 0) -> np.ndarray:
    g = _rng(config_id, "x", microbatch)
    return _finish(g.standard_normal((cfg.tokens, cfg.hidden), dtype=np.float32), cfg)


def upstream_grad(cfg: ChunkCfg, config_id: str, microbatch: int = 0) -> np.ndarray:
    g = _rng(config_id, "dy", microbatch)
    return _finish(g.standard_normal((cfg.tokens, cfg.hidden), dtype=np.float32), cfg)


def matrix(key: tuple, shape: tuple[int, ...], scale: float = 1.0, bf16: bool = False) -> np.ndarray:
    """A plain N(0, scale^2) tensor for single-kernel tests."""
    v = _rng("matrix", *key).standard_normal(shape, dtype=np.float32) * np.float32(scale)
    return round_to_bf16(v) if bf16 else v

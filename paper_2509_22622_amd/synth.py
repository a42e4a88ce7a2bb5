"""Seeded synthetic inputs shared by the tests, the bench and the smoke check.

This module holds no arithmetic of the method (no RoPE, no key-set rule, no
softmax): it only draws numbers and encodes them as bfloat16 bit patterns.
Both the CPU oracle's callers and the HIP path's callers take their inputs
from here so that the two sides consume the same bits.

Recipe: i.i.d. N(0,1) drawn in float32, rounded to bfloat16 with
round-to-nearest-even, one independent Philox stream per
(master seed, config id, layer, chunk, tensor).  These stand in for the
activations of a trained Wan-1.3B-shaped model, which are not available.
"""
from __future__ import annotations

import dataclasses

import numpy as np

MASTER_SEED = 20250922
_TENSOR_ID = {"q": 0, "k": 1, "v": 2}


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one configuration (names follow the paper: chunk, window, sink)."""

    name: str
    cfg_id: int
    layers: int
    heads: int
    head_dim: int
    grid_h: int
    grid_w: int
    chunk_frames: int
    sink_frames: int
    window_frames: int
    n_chunks: int

    @property
    def tokens_per_frame(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def chunk_tokens(self) -> int:
        return self.chunk_frames * self.tokens_per_frame


# The five configurations of the benchmark definition.
TINY = Workload("tiny", 1, 1, 4, 64, 6, 10, 3, 3, 6, 8)
WAN_LAYER = Workload("wan1.3b-layer", 2, 1, 12, 128, 30, 52, 3, 3, 9, 6)
WAN_LOOP = Workload("wan1.3b-30layers", 3, 30, 12, 128, 30, 52, 3, 3, 9, 60)
LONG_WINDOW = Workload("long-window", 4, 1, 12, 128, 30, 52, 3, 0, 21, 9)
RECACHE = Workload("recache-prefill", 5, 30, 12, 128, 30, 52, 3, 3, 9, 5)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(cfg_id: int, layer: int, chunk: int, tensor: str, seed: int) -> np.random.Generator:
    key = (np.uint64(seed) << np.uint64(20)) ^ np.uint64(cfg_id)
    ctr = [np.uint64(layer), np.uint64(chunk), np.uint64(_TENSOR_ID[tensor]), np.uint64(0)]
    return np.random.Generator(np.random.Philox(key=[key, np.uint64(0x4C4C)], counter=ctr))


def normal_bf16(shape, cfg_id: int, layer: int, chunk: int, tensor: str,
                seed: int = MASTER_SEED, scale: float = 1.0) -> np.ndarray:
    """bf16 bit patterns of scale * N(0,1) for the given stream."""
    g = _rng(cfg_id, layer, chunk, tensor, seed)
    x = g.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        x = x * np.float32(scale)
    return f32_to_bf16_bits(x)


def chunk_qkv(w: Workload, layer: int, chunk: int, n_frames: int | None = None,
              seed: int = MASTER_SEED, q_scale: float = 1.0):
    """(q, k, v) bf16 bit patterns, each [n_frames*P, H, D], token-major."""
    n = w.chunk_frames if n_frames is None else n_frames
    shape = (n * w.tokens_per_frame, w.heads, w.head_dim)
    q = normal_bf16(shape, w.cfg_id, layer, chunk, "q", seed, q_scale)
    k = normal_bf16(shape, w.cfg_id, layer, chunk, "k", seed)
    v = normal_bf16(shape, w.cfg_id, layer, chunk, "v", seed)
    return q, k, v

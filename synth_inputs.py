"""Seeded synthetic Q/K/V streams with the shapes of the paper's workloads.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no attention, scoring, pruning or quantisation), so both
the CPU oracle's tests and the HIP path's tests may feed from it.

The paper measures on TUM-Dynamics / ScanNet sequences pushed through trained
StreamVGGT weights (Experiments, "Efficiency Analysis"); neither exists here,
so these streams stand in for them: per frame, 1 camera + 4 register tokens
followed by the patch tokens of a 518-pixel-max-edge image at patch size 14,
Q and V ~ N(0,1), and K ~ N(0,1) times a per-(head, channel) log-normal scale
so that a few key channels dominate (the channel-wise key outliers of the
paper's Fig. 3).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    """Shape parameters of one benchmark configuration."""

    name: str
    n_heads: int
    head_dim: int
    tokens_per_frame: int      # n = 1 + R + N, special tokens first
    n_special: int             # 1 camera + R register tokens
    pool_group: int            # g, query pooling size
    budget_tokens: int         # L_max
    frames: int
    n_layers: int
    n_streams: int
    k_bits: int
    k_group: int               # tokens per per-channel key group
    v_bits: int
    v_group: int               # channels per per-token value group
    dtype: str                 # "f32" or "bf16"
    seed: int


WORKLOADS = {
    # Tiny single layer, fp32 inputs, INT8/INT8.
    "tiny": Workload("tiny", 4, 64, 69, 5, 16, 256, 8, 1, 1, 8, 64, 8, 64, "f32", 0),
    # One VGGT-scale global-attention layer, 518x392 input, INT4/INT4.
    "vggt_layer": Workload("vggt_layer", 16, 64, 1041, 5, 16, 8192, 32, 1, 1, 4, 64, 4, 64, "bf16", 1),
    # 24-layer stack, 200 frames.
    "vggt_stack": Workload("vggt_stack", 16, 64, 1041, 5, 16, 16384, 200, 24, 1, 4, 64, 4, 64, "bf16", 2),
    # Long stream, 1000 frames.
    "vggt_long": Workload("vggt_long", 16, 64, 1041, 5, 16, 16384, 1000, 24, 1, 4, 64, 4, 64, "bf16", 3),
    # High-res, 4 streams, INT2 keys group 32.
    "vggt_hires": Workload("vggt_hires", 16, 64, 1374, 5, 16, 24576, 500, 24, 4, 2, 32, 4, 64, "bf16", 4),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to even).

    The result is still an fp32 array; every element has its low 16 bits zero.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def _rng(seed: int, stream: int, layer: int, frame: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream, layer, frame])))


def key_channel_scales(w: Workload, stream: int = 0, layer: int = 0) -> np.ndarray:
    """sigma[h, c] = exp(N(0,1)), drawn once per (seed, stream, layer)."""
    g = _rng(w.seed, stream, layer, 1 << 30)
    return np.exp(g.standard_normal((w.n_heads, w.head_dim))).astype(np.float32)


def frame_qkv(w: Workload, frame: int, stream: int = 0, layer: int = 0, sigma: np.ndarray | None = None):
    """Q, K, V of one frame, each fp32 [n, H, d] (bf16-representable when w.dtype == 'bf16')."""
    if sigma is None:
        sigma = key_channel_scales(w, stream, layer)
    g = _rng(w.seed, stream, layer, frame)
    shape = (w.tokens_per_frame, w.n_heads, w.head_dim)
    q = g.standard_normal(shape, dtype=np.float32)
    k = g.standard_normal(shape, dtype=np.float32) * sigma[None, :, :]
    v = g.standard_normal(shape, dtype=np.float32)
    if w.dtype == "bf16":
        q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
    return q, k.astype(np.float32), v

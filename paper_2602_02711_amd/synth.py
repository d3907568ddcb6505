"""Seeded synthetic inputs for the W4A16 / bf16 linear path.

This module serves both the CPU oracle's tests and the GPU path, and therefore holds none of
the method's arithmetic: it only draws numbers.  Weights are fp32 ``0.02 * N(0,1)`` (the usual
initialisation scale of an LLM's Linear layers), activations are ``N(0,1)`` stored as bf16 bit
patterns; both stand in for the checkpoints and prompts of the paper's Sec. 5.1 workloads,
which cost the same per shape whatever their values.  The shapes are those of a 7B-class
decoder: hidden 4096, 32 query and 8 key/value heads of 128, SwiGLU intermediate 14336.
"""
from __future__ import annotations

import numpy as np

GROUP = 128
BASE_SEED = 260_202_711

# (name, K, N) of the four per-layer Linear shapes; order is the order inside a decoder layer.
LAYER_SHAPES = (
    ("qkv", 4096, 6144),        # fused q (32x128) + k (8x128) + v (8x128)
    ("attn_out", 4096, 4096),
    ("gate_up", 4096, 28672),   # fused gate + up, 2 x 14336
    ("down", 14336, 4096),
)
# The sweep order used by the decode benchmark (smallest to largest weight stream).
SWEEP_SHAPES = (
    ("attn_out", 4096, 4096),
    ("qkv", 4096, 6144),
    ("gate_up", 4096, 28672),
    ("down", 14336, 4096),
)
SMALL_SHAPE = ("small", 1024, 1024)
LM_HEAD = ("lm_head", 4096, 128256)


def seed_for(config: int, shape_index: int, role: int, layer: int = 0) -> int:
    """role 0 = weights, 1 = activations."""
    return BASE_SEED + 1000 * config + 100 * layer + 10 * shape_index + role


def weights_f32(seed: int, N: int, K: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((N, K), dtype=np.float32)
    w *= np.float32(0.02)
    return w


def to_bf16_bits(values: np.ndarray) -> np.ndarray:
    """Storage conversion fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(values, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def activations_bf16(seed: int, M: int, K: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return to_bf16_bits(rng.standard_normal((M, K), dtype=np.float32))

"""Seeded tensor generators.  bf16 tensors are carried as uint16 bit patterns, f32 as float32.

Recipe: numpy.random.Generator(PCG64(seed)); weights are drawn once from the chain's seed in
list order; iteration t's external inputs from seed*1000 + t in list order.  A normal draw is
made in float32 and, for bf16, rounded to the nearest bf16 (ties to even) by bit arithmetic.
"""
from __future__ import annotations

from typing import List

import numpy as np

from .spec import ChainSpec, TensorSpec


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern, round to nearest, ties to even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def draw_tensor(t: TensorSpec, rng: np.random.Generator) -> np.ndarray:
    kind, mean, std = t.dist
    if kind != "normal":
        raise ValueError(f"unknown distribution {kind}")
    x = rng.standard_normal(t.numel, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    return f32_to_bf16_bits(x) if t.dtype == "bf16" else x


def make_weights(chain: ChainSpec) -> List[np.ndarray]:
    rng = np.random.Generator(np.random.PCG64(chain.seed))
    return [draw_tensor(t, rng) for t in chain.weights]


def make_inputs(chain: ChainSpec, t: int) -> List[np.ndarray]:
    rng = np.random.Generator(np.random.PCG64(chain.seed * 1000 + t))
    return [draw_tensor(s, rng) for s in chain.ext]

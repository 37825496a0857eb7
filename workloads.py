"""Seeded synthetic inputs and the BitNet-shaped layer sizes used by tests and bench.

This module holds none of the method's arithmetic: it only draws random arrays
with the shapes and value distributions the benchmark configurations state, so
that the CPU oracle and the GPU library see identical bytes.

Hidden sizes 2048 / 4096 / 7168 are the 1.3B / 6.7B / 30B rows of the paper's
model-size table (appendix); the paper does not state the FFN width, so the
conventional 4*d is used, and a fused QKV projection of 3*d.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_BASE = 231011453


@dataclass(frozen=True)
class Layer:
    name: str
    K: int  # fan-in
    N: int  # fan-out


@dataclass(frozen=True)
class Config:
    index: int
    name: str
    layers: tuple
    Ms: tuple
    w_std: float
    outlier_p: float = 0.0
    outlier_mul: float = 1.0
    per_tensor: bool = False


CONFIGS = (
    Config(0, "single-small", (Layer("lin", 256, 512),), (8,), 0.02),
    Config(1, "bitnet-1.3b-decode",
           (Layer("qkv", 2048, 6144), Layer("o", 2048, 2048),
            Layer("up", 2048, 8192), Layer("down", 8192, 2048)), (1, 4, 16), 0.02),
    Config(2, "bitnet-6.7b-prefill",
           (Layer("up", 4096, 16384), Layer("down", 16384, 4096)), (2048,), 0.02,
           outlier_p=0.001, outlier_mul=20.0),
    Config(3, "bitnet-30b",
           (Layer("qkv", 7168, 21504), Layer("up", 7168, 28672), Layer("down", 28672, 7168)),
           (64, 4096), 0.01),
    Config(4, "train-step-6.7b", (Layer("up", 4096, 16384),), (8192,), 0.02, per_tensor=True),
)


def seed_for(config_index: int, shape_index: int = 0, salt: int = 0) -> int:
    return SEED_BASE + 1000 * (config_index + 1) + shape_index + 100000 * salt


def make_weight(N: int, K: int, std: float, seed: int, mean: float = 0.0) -> np.ndarray:
    """fp32 latent weight [N,K] ~ N(mean, std^2)."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((N, K), dtype=np.float32)
    w *= np.float32(std)
    if mean != 0.0:
        w += np.float32(mean)
    return w


def make_activation(M: int, K: int, seed: int, outlier_p: float = 0.0,
                    outlier_mul: float = 1.0) -> np.ndarray:
    """fp32 activations [M,K] ~ N(0,1); a Bernoulli(outlier_p) subset is multiplied by
    outlier_mul before any normalisation (stress for the absmax scale)."""
    rng = np.random.default_rng(seed + 7)
    x = rng.standard_normal((M, K), dtype=np.float32)
    if outlier_p > 0.0:
        mask = rng.random((M, K), dtype=np.float32) < np.float32(outlier_p)
        x[mask] *= np.float32(outlier_mul)
    return x


def make_grad(M: int, N: int, seed: int, std: float = 1e-3) -> np.ndarray:
    """fp32 upstream gradient dY [M,N] ~ N(0, std^2)."""
    rng = np.random.default_rng(seed + 13)
    g = rng.standard_normal((M, N), dtype=np.float32)
    g *= np.float32(std)
    return g

"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds none of the method's arithmetic: it only draws tensors with
the shapes, value distributions and outlier structure of the workloads the
paper measures on (LLM linear-layer activations, weights and output
gradients), which need training data and are replaced by these stand-ins.

bf16 tensors are returned as numpy ``uint16`` arrays of bit patterns.
"""
from __future__ import annotations

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_f32(shape, std: float, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def normal_bf16(shape, std: float, seed: int) -> np.ndarray:
    return f32_to_bf16_bits(normal_f32(shape, std, seed))


def student_t_bf16(shape, nu: float, scale: float, seed: int) -> np.ndarray:
    """Heavy-tailed values: scale * Student-t(nu), rounded to bf16."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(-1)
    step = 1 << 22
    for lo in range(0, flat.size, step):
        hi = min(flat.size, lo + step)
        flat[lo:hi] = (rng.standard_t(nu, size=hi - lo) * scale).astype(np.float32)
    return f32_to_bf16_bits(out)


def activations_bf16(tokens: int, d_in: int, seed: int, outlier_frac: float = 0.005,
                     outlier_gain: float = 20.0) -> np.ndarray:
    """N(0,1) activations with a few outlier channels (columns) scaled up."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((tokens, d_in), dtype=np.float32)
    n_out = int(np.ceil(outlier_frac * d_in))
    cols = rng.choice(d_in, size=n_out, replace=False)
    x[:, cols] *= np.float32(outlier_gain)
    return f32_to_bf16_bits(x)


def linear_layer_bf16(tokens: int, d_in: int, d_out: int, seed: int):
    """(X, W, dY) of one linear layer: X N(0,1) with outlier channels, W N(0,0.02^2),
    dY N(0,(1e-3)^2), all bf16 bit patterns."""
    X = activations_bf16(tokens, d_in, seed * 3 + 0)
    W = normal_bf16((d_out, d_in), 0.02, seed * 3 + 1)
    dY = normal_bf16((tokens, d_out), 1e-3, seed * 3 + 2)
    return X, W, dY

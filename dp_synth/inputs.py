"""Seeded input generators (numpy, host side).

bf16 tensors are carried as uint16 bit patterns so that numpy (which has no bf16
type) can hold them exactly; each consumer converts them with its own code.
"""
from __future__ import annotations

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (round-to-nearest-even) and return the 16-bit patterns.

    Input formatting only: the synthetic tensors are *defined* as these rounded values.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = (u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    return r.astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly (used by harness code to feed torch)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(b.shape)


def normal_f32(shape, std: float, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def normal_bf16_bits(shape, std: float, seed: int) -> np.ndarray:
    return f32_to_bf16_bits(normal_f32(shape, std, seed))


def zipf_ids(B: int, T: int, V: int, s: float, seed: int) -> np.ndarray:
    """Token ids with p(rank r) proportional to r**-s over r = 1..V; id = r - 1. int32 [B, T]."""
    rng = np.random.default_rng(seed)
    w = np.arange(1, V + 1, dtype=np.float64) ** (-float(s))
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = rng.random(size=(B, T))
    ids = np.searchsorted(cdf, u, side="left")
    return np.minimum(ids, V - 1).astype(np.int32)


def position_ids(B: int, T: int) -> np.ndarray:
    return np.broadcast_to(np.arange(T, dtype=np.int32), (B, T)).copy()


def segment_ids(B: int, T: int) -> np.ndarray:
    """Token-type ids of a sentence pair: 0 for the first half of the sequence, 1 for the second. int32 [B, T]."""
    row = (np.arange(T, dtype=np.int32) >= (T + 1) // 2).astype(np.int32)
    return np.broadcast_to(row, (B, T)).copy()


def example_scales(B: int, lo: float, hi: float, seed: int) -> np.ndarray:
    """Per-example log-uniform scales in [lo, hi] (fp32): multiplying example i's output
    gradients by scale[i] makes the per-example norms straddle the clip norm."""
    rng = np.random.default_rng(seed)
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=B)).astype(np.float32)


def synthetic_sqnorms(B: int, C: float, seed: int) -> np.ndarray:
    """Positive fp32 values, log-uniform in [C^2/100, 100 C^2]: stand-in squared norms that put
    about half the examples on each side of the clip norm. Used where a test feeds the second
    pass directly, without running the first."""
    rng = np.random.default_rng(seed)
    e = rng.uniform(np.log(C * C / 100.0), np.log(C * C * 100.0), size=B)
    return np.exp(e).astype(np.float32)

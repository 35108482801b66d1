"""Seeded q, k, v, dout tensors in bf16 (carried as uint16 bit patterns).

Values are drawn as fp32 N(0,1) and rounded to nearest-even bf16.  numpy has no
bf16 type, so tensors travel as uint16 bit patterns; ``bf16_bits_to_f32`` widens
them exactly.  Nothing here is attention arithmetic.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

from .bags import BagSpec


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16). No NaN inputs expected."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _value_rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 1 + stream])))


def _normal_bf16(rng: np.random.Generator, shape, chunk_rows: int = 8192) -> np.ndarray:
    out = np.empty(shape, dtype=np.uint16)
    T = shape[0]
    for r0 in range(0, T, chunk_rows):
        r1 = min(T, r0 + chunk_rows)
        blk = rng.standard_normal(size=(r1 - r0,) + tuple(shape[1:]), dtype=np.float32)
        out[r0:r1] = f32_to_bf16_bits(blk)
    return out


def make_qkv_dout(bag: BagSpec, with_dout: bool = True) -> Dict[str, np.ndarray]:
    """bf16 bit patterns of q, k, v (and dout), each of shape (T, H, d), from the bag's seed.

    For a bag with ``k_outlier_prob`` > 0 every k entry is independently, with
    that probability, multiplied by ``k_outlier_scale`` before rounding.
    """
    T, H, d = bag.total_tokens, bag.H, bag.d
    shape = (T, H, d)
    out: Dict[str, np.ndarray] = {}
    out["q"] = _normal_bf16(_value_rng(bag.seed, 0), shape)
    if bag.k_outlier_prob > 0.0:
        rng = _value_rng(bag.seed, 1)
        rng_mask = _value_rng(bag.seed, 4)
        k = np.empty(shape, dtype=np.uint16)
        chunk = 8192
        for r0 in range(0, T, chunk):
            r1 = min(T, r0 + chunk)
            blk = rng.standard_normal(size=(r1 - r0, H, d), dtype=np.float32)
            mask = rng_mask.random(size=(r1 - r0, H, d), dtype=np.float32) < bag.k_outlier_prob
            blk[mask] *= np.float32(bag.k_outlier_scale)
            k[r0:r1] = f32_to_bf16_bits(blk)
        out["k"] = k
    else:
        out["k"] = _normal_bf16(_value_rng(bag.seed, 1), shape)
    out["v"] = _normal_bf16(_value_rng(bag.seed, 2), shape)
    if with_dout:
        out["dout"] = _normal_bf16(_value_rng(bag.seed, 3), shape)
    return out

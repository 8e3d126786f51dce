"""Seeded, counter-based random streams and bf16 helpers for the synthetic workloads.

Holds no arithmetic of the batching method: only random number streams and the
float32 <-> bfloat16 bit conversions that prepare *inputs*.  Both the CPU
oracle's tests and the HIP path's tests/bench draw their inputs from here, so the
two sides always see identical arrays.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 170702402


def _mix(h: int, v: int) -> int:
    """splitmix64-style avalanche of (h, v) -> 64-bit key word."""
    m = (1 << 64) - 1
    z = (h ^ (v + 0x9E3779B97F4A7C15 + ((h << 6) & m) + (h >> 2))) & m
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    return z ^ (z >> 31)


def stream(seed: int, *path: int) -> np.random.Generator:
    """Independent Philox stream named by (seed, path...).

    Philox is counter based: a stream depends only on its key, never on how many
    other streams were drawn before it, so any sub-array (one expert's weights,
    one example's feature map) can be regenerated alone.
    """
    h = 0x243F6A8885A308D3
    for v in path:
        h = _mix(h, int(v) & ((1 << 64) - 1))
    return np.random.Generator(np.random.Philox(key=[int(seed) & ((1 << 64) - 1), h]))


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bfloat16 bit patterns, round-to-nearest-even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float32 values (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array rounded to the nearest bfloat16-representable float32."""
    return bf16_to_f32(bf16_bits(a))

"""Seeded synthetic inputs for the AsyncMesh stage update.

Used by both the CPU oracle's tests and the GPU path's tests / benchmark so that the two see the
same numbers.  Holds none of the method's arithmetic: it only draws the starting weights and
the per-replica, per-step gradients with the value distributions of the training runs the
method was evaluated on (weights ~ N(0, 0.02^2) as in GPT-2 style initialisation, gradients
~ N(0, (1e-3)^2), every replica starting from the same point).
"""
from __future__ import annotations

import numpy as np

W_STD = 0.02
G_STD = 1e-3


def _rng(*key: int) -> np.random.Generator:
    return np.random.default_rng([int(k) & 0xFFFFFFFF for k in key])


def stage_weights(n: int, seed: int = 0) -> np.ndarray:
    """w^0, shared by every replica: n fp32 values ~ N(0, 0.02^2)."""
    return (_rng(seed, 0x57) .standard_normal(n, dtype=np.float32) * np.float32(W_STD)).astype(np.float32)


def replica_grads(n: int, replicas: int, t: int, seed: int = 0) -> list[np.ndarray]:
    """g_i^{t-1} for i < replicas: independent fp32 draws ~ N(0, (1e-3)^2) per replica and step."""
    return [(_rng(seed, 0x6A, t, i).standard_normal(n, dtype=np.float32) * np.float32(G_STD)).astype(np.float32)
            for i in range(replicas)]


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns (uint16), round-to-nearest-even; a storage conversion of the
    synthetic inputs, so that both sides are handed the very same bf16 gradients."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def tiled(pool: np.ndarray, n: int, offset: int = 0) -> np.ndarray:
    """n values read cyclically from pool starting at offset (how the large benchmark tensors are
    filled from a small host-generated pool)."""
    start = offset % pool.size
    reps = (start + n + pool.size - 1) // pool.size
    return np.tile(pool, reps)[start:start + n].copy()

"""Seeded synthetic-tensor generators shared by the CPU oracle tests and the GPU tests.

This module holds no operator arithmetic: it only produces reproducible input
tensors (as numpy arrays of exact bit patterns) so that the CPU oracle and the
HIP kernels are fed identical bytes.

Generator: a counter-based SplitMix64 stream (element i of a stream is the
SplitMix64 output function applied to ``seed + (i+1)*GAMMA``), mapped to a
uniform double in [0,1) from the top 53 bits, and to normals by Box-Muller.
Values are cast to fp32 and, where a workload asks for bf16, rounded once to
bf16 with round-to-nearest-even; bf16 tensors are carried as uint16 bit patterns.
"""
from __future__ import annotations

import numpy as np

GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1


def tensor_seed(config: int, tensor: int, set_index: int = 0) -> int:
    """Seed of tensor ``tensor`` of workload ``config``; ``set_index`` selects one of
    the rotated buffer sets a benchmark cycles through (0 = the parity-test set)."""
    return (0x9E3779B97F4A7C15 * (16 * config + tensor + 1) + 0xD1B54A32D192ED03 * set_index) & _MASK64


def splitmix64(seed: int, n: int, offset: int = 0) -> np.ndarray:
    """n consecutive outputs of the SplitMix64 stream started at ``seed``."""
    with np.errstate(over="ignore"):
        idx = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
        z = np.uint64(seed & _MASK64) + idx * GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, n: int, offset: int = 0) -> np.ndarray:
    """Uniform doubles in [0,1): top 53 bits of each SplitMix64 output times 2^-53."""
    return (splitmix64(seed, n, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform(seed: int, shape, lo: float, hi: float) -> np.ndarray:
    n = int(np.prod(shape))
    return (lo + (hi - lo) * uniform01(seed, n)).astype(np.float32).reshape(shape)


def normal(seed: int, shape, mean: float, var: float) -> np.ndarray:
    """N(mean, var) by Box-Muller on consecutive pairs of the uniform stream
    (``var`` is the variance, not the standard deviation)."""
    n = int(np.prod(shape))
    half = (n + 1) // 2
    u = uniform01(seed, 2 * half)
    u1, u2 = u[0::2], u[1::2]
    r = np.sqrt(-2.0 * np.log1p(-u1))          # 1-u1 in (0,1]: log never sees 0
    z = np.empty(2 * half, dtype=np.float64)
    z[0::2] = r * np.cos(2.0 * np.pi * u2)
    z[1::2] = r * np.sin(2.0 * np.pi * u2)
    return (mean + np.sqrt(var) * z[:n]).astype(np.float32).reshape(shape)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even. Finite inputs only."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)

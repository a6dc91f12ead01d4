"""Counter-based random numbers for weights, inputs and symbol draws.

Element ``i`` of stream ``seed`` is a pure function of (seed, i): a splitmix64
hash of the counter gives two 32-bit uniforms, Box-Muller in float64 turns them
into a standard normal.  No state is carried, so any consumer regenerates the
same values in any order.
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        x = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = x
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def _bits(seed: int, n: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        ctr = np.arange(n, dtype=np.uint64) + (np.uint64(seed) * np.uint64(0xD1342543DE82EF95))
    return _splitmix64(_splitmix64(ctr))


def uniform(seed: int, shape, lo=0.0, hi=1.0) -> np.ndarray:
    n = int(np.prod(shape)) if len(tuple(shape)) else 1
    b = _bits(seed, n)
    u = ((b >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    return (lo + (hi - lo) * u).reshape(shape)


def normal(seed: int, shape, mean=0.0, std=1.0) -> np.ndarray:
    n = int(np.prod(shape)) if len(tuple(shape)) else 1
    b = _bits(seed, n)
    u1 = ((b >> np.uint64(32)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
    u2 = ((b & np.uint64(0xFFFFFFFF)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (mean + std * z).reshape(shape)


def randint(seed: int, shape, lo: int, hi: int) -> np.ndarray:
    """Integers uniform on [lo, hi] (both ends included)."""
    n = int(np.prod(shape)) if len(tuple(shape)) else 1
    b = _bits(seed, n)
    span = np.uint64(hi - lo + 1)
    return (lo + (b % span).astype(np.int64)).reshape(shape)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float values to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)

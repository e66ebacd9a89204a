"""Counter-based integer hash used by every seeded input generator.

The generators never keep RNG state: a draw is a pure function of
``(seed, a, b, c)``.  That is what lets the host generator (numpy) and the
device generator (a HIP kernel) emit identical candidate bits without sharing
any code: both implement this one published recipe, the 64-bit finaliser of
SplitMix64 (Steele, Lea, Flood 2014), chained three times over the counters.

This module holds no arithmetic of the evaluated method.
"""
from __future__ import annotations

import numpy as np

MASK64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
MUL1 = 0xBF58476D1CE4E5B9
MUL2 = 0x94D049BB133111EB


def mix64(z: int) -> int:
    """SplitMix64 finaliser on a Python int (scalar path, graph generation)."""
    z &= MASK64
    z = ((z ^ (z >> 30)) * MUL1) & MASK64
    z = ((z ^ (z >> 27)) * MUL2) & MASK64
    return z ^ (z >> 31)


def hash3(seed: int, a: int, b: int, c: int) -> int:
    """h(seed, a, b, c): three chained finalisers, one per counter."""
    k = mix64(seed + GOLDEN * (a + 1))
    k = mix64(k + GOLDEN * (b + 1))
    return mix64(k + GOLDEN * (c + 1))


_G = np.uint64(GOLDEN)
_M1 = np.uint64(MUL1)
_M2 = np.uint64(MUL2)


def mix64_np(z: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def hash3_np(seed: int, a, b, c) -> np.ndarray:
    """Vector form of :func:`hash3`; ``a``, ``b``, ``c`` broadcast as uint64."""
    with np.errstate(over="ignore"):
        a = np.asarray(a, dtype=np.uint64)
        b = np.asarray(b, dtype=np.uint64)
        c = np.asarray(c, dtype=np.uint64)
        k = mix64_np(np.uint64(seed & MASK64) + _G * (a + np.uint64(1)))
        k = mix64_np(k + _G * (b + np.uint64(1)))
        return mix64_np(k + _G * (c + np.uint64(1)))


def uniform01(h: int) -> float:
    """Top 53 bits of a hash as a float in [0, 1)."""
    return (h >> 11) * (1.0 / (1 << 53))

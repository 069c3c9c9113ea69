"""Counter-based pseudo-random numbers for the synthetic workloads.

Every draw is a pure function of (seed, stream, index): the value at an index never
depends on how many other values were drawn, so the CPU checker and the GPU path are
handed bit-identical inputs regardless of chunking.  The mixer is the public
splitmix64 finaliser applied to a 64-bit counter.

This module holds no GCN arithmetic: it only produces raw uniforms, normals and
integers.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _base(seed: int, stream: int) -> np.uint64:
    # scalar pre-mix of (seed, stream) done with Python ints (exact, no overflow warnings)
    z = (seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    z ^= z >> 31
    return np.uint64(z)


def bits64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """uint64[count]: draws number start .. start+count-1 of the (seed, stream) sequence."""
    idx = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(_base(seed, stream) + (idx + np.uint64(1)) * _GOLDEN)


def uniform01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64[count] in [0, 1) from the top 53 bits."""
    return (bits64(seed, stream, start, count) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def randint(seed: int, stream: int, start: int, count: int, hi: int) -> np.ndarray:
    """int64[count] uniform in [0, hi) (multiply-shift on the top 32 bits; hi < 2**31)."""
    top = bits64(seed, stream, start, count) >> np.uint64(32)
    return ((top * np.uint64(hi)) >> np.uint64(32)).astype(np.int64)


def normal(seed: int, stream: int, count: int, chunk: int = 1 << 22) -> np.ndarray:
    """float32[count] ~ N(0,1) by Box-Muller: value 2k and 2k+1 come from uniforms 2k, 2k+1."""
    out = np.empty(count, dtype=np.float32)
    npairs = (count + 1) // 2
    for p0 in range(0, npairs, chunk):
        p1 = min(npairs, p0 + chunk)
        u = uniform01(seed, stream, 2 * p0, 2 * (p1 - p0))
        u1 = 1.0 - u[0::2]            # (0, 1]
        u2 = u[1::2]
        r = np.sqrt(-2.0 * np.log(u1))
        z = np.empty(2 * (p1 - p0), dtype=np.float64)
        z[0::2] = r * np.cos(2.0 * np.pi * u2)
        z[1::2] = r * np.sin(2.0 * np.pi * u2)
        lo, hi = 2 * p0, min(count, 2 * p1)
        out[lo:hi] = z[: hi - lo].astype(np.float32)
    return out


def permutation(seed: int, stream: int, n: int) -> np.ndarray:
    """int64[n]: a seeded permutation of 0..n-1 (stable argsort of 64-bit random keys)."""
    return np.argsort(bits64(seed, stream, 0, n), kind="stable").astype(np.int64)

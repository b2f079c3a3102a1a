"""Counter-based random numbers: SplitMix64 finaliser + Box-Muller.

Element i of stream (seed, stream) depends only on (seed, stream, i), so the
same buffers can be produced anywhere without shared state.
"""
from __future__ import annotations

import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_G = np.uint64(0x9E3779B97F4A7C15)


def _mix(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _bits(seed: int, stream: int, n: int, lane: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        base = _mix(np.array([(seed * 0x632BE59BD9B4E019 + stream * 0xD1342543DE82EF95
                               + lane * 0x2545F4914F6CDD1D) & 0xFFFFFFFFFFFFFFFF],
                             dtype=np.uint64))[0]
        idx = np.arange(1, n + 1, dtype=np.uint64)
        return _mix(base + idx * _G)


def uniform01(seed: int, stream: int, n: int, lane: int = 0) -> np.ndarray:
    """n doubles in (0, 1)."""
    b = _bits(seed, stream, n, lane)
    return ((b >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, n: int) -> np.ndarray:
    """n standard-normal doubles (Box-Muller on two independent lanes)."""
    u1 = uniform01(seed, stream, n, 0)
    u2 = uniform01(seed, stream, n, 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def uniform_int(seed: int, stream: int, n: int, hi: int) -> np.ndarray:
    """n int32 labels uniform in [0, hi)."""
    u = uniform01(seed, stream, n, 2)
    return np.minimum((u * hi).astype(np.int64), hi - 1).astype(np.int32)

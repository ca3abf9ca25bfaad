"""Counter-based pseudo-random numbers for the seeded synthetic workloads.

Everything here is input generation only: no pruning-scheme logic and no layer
arithmetic lives in this module.  The generator is a SplitMix64-style finaliser
applied to (seed, stream, counter), written out in NumPy uint64 arithmetic so
that the streams do not depend on the NumPy/PyTorch version.
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)
_S1 = np.uint64(0xD1342543DE82EF95)
_S2 = np.uint64(0xA24BAED4963EE407)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _C1
    z = (z ^ (z >> np.uint64(27))) * _C2
    return z ^ (z >> np.uint64(31))


def u64(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit words of stream `stream` of seed `seed`, counters offset..offset+n-1."""
    with np.errstate(over="ignore"):
        base = _mix(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) * _S1
                    + np.uint64(stream & 0xFFFFFFFFFFFFFFFF) * _S2 + _GAMMA)
        ctr = np.arange(offset, offset + n, dtype=np.uint64)
        return _mix(base + (ctr + np.uint64(1)) * _GAMMA)


def uniform01(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """Doubles in (0, 1): the top 53 bits, shifted off zero by half an ulp."""
    w = u64(seed, stream, n, offset) >> np.uint64(11)
    return (w.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, n: int, sigma: float = 1.0) -> np.ndarray:
    """n samples of N(0, sigma^2) as float64 (Box-Muller on two uniform streams)."""
    m = (n + 1) // 2
    u1 = uniform01(seed, 2 * stream, m)
    u2 = uniform01(seed, 2 * stream + 1, m)
    r = np.sqrt(-2.0 * np.log(u1))
    out = np.empty(2 * m, dtype=np.float64)
    out[0::2] = r * np.cos(2.0 * np.pi * u2)
    out[1::2] = r * np.sin(2.0 * np.pi * u2)
    return out[:n] * sigma

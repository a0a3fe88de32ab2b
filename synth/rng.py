"""Counter-based random numbers: splitmix64 finaliser over (seed, stream, index).

Element i of stream s under seed z is  mix64(mix64(z * K1 + s * K2) + i * GOLDEN),
so any slice can be produced independently and the result never depends on the
order in which tensors are generated.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_K1 = np.uint64(0xD1342543DE82EF95)
_K2 = np.uint64(0xA24BAED4963EE407)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


class Stream:
    """One named stream of 64-bit words under a seed."""

    def __init__(self, seed: int, stream: int):
        with np.errstate(over="ignore"):
            base = np.uint64(seed) * _K1 + np.uint64(stream) * _K2 + _GOLDEN
        self.key = _mix64(np.array([base], dtype=np.uint64))[0]

    def words(self, n: int, offset: int = 0) -> np.ndarray:
        idx = np.arange(offset, offset + n, dtype=np.uint64)
        with np.errstate(over="ignore"):
            return _mix64(self.key + (idx + np.uint64(1)) * _GOLDEN)


def _unit(words: np.ndarray) -> np.ndarray:
    """53-bit uniform in [0,1) as float64."""
    return (words >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform(seed: int, stream: int, shape, lo: float, hi: float) -> np.ndarray:
    """float32 array ~ U[lo, hi)."""
    n = int(np.prod(shape))
    u = _unit(Stream(seed, stream).words(n))
    return (lo + (hi - lo) * u).astype(np.float32).reshape(shape)


def normal(seed: int, stream: int, shape) -> np.ndarray:
    """float32 array ~ N(0,1) by Box-Muller on pairs of uniforms (float64 inside)."""
    n = int(np.prod(shape))
    m = (n + 1) // 2
    w = Stream(seed, stream).words(2 * m)
    u1 = 1.0 - _unit(w[0::2])          # (0,1]
    u2 = _unit(w[1::2])
    r = np.sqrt(-2.0 * np.log(u1))
    z = np.empty(2 * m, dtype=np.float64)
    z[0::2] = r * np.cos(2.0 * np.pi * u2)
    z[1::2] = r * np.sin(2.0 * np.pi * u2)
    return z[:n].astype(np.float32).reshape(shape)


def randint(seed: int, stream: int, shape, lo: int, hi: int) -> np.ndarray:
    """int32 array uniform on the integers lo..hi inclusive."""
    n = int(np.prod(shape))
    w = Stream(seed, stream).words(n)
    span = np.uint64(hi - lo + 1)
    return (lo + (w % span).astype(np.int64)).astype(np.int32).reshape(shape)

"""Counter-based random streams for the synthetic workloads.

Every draw is a pure function of (key, counter): SplitMix64 finalisation of
``key + (i + 1) * GOLDEN``.  Nothing here depends on a library's distribution
code, so the streams never drift between numpy versions.  The module holds no
arithmetic of the decoding method itself; it only makes inputs.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_TWO_M53 = 2.0 ** -53


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def make_key(*parts: int) -> np.uint64:
    """Fold a tuple of small integers into one 64-bit stream key."""
    with np.errstate(over="ignore"):
        k = np.uint64(0x243F6A8885A308D3)
        for p in parts:
            k = _mix(np.asarray(k + np.uint64(int(p) & 0xFFFFFFFFFFFFFFFF) * _GOLDEN + _GOLDEN,
                                dtype=np.uint64))
        return np.uint64(k)


def bits64(key: np.uint64, n: int, start: int = 0) -> np.ndarray:
    """n 64-bit words of stream `key`, counters start .. start+n-1."""
    with np.errstate(over="ignore"):
        i = np.arange(start + 1, start + n + 1, dtype=np.uint64)
        return _mix(np.uint64(key) + i * _GOLDEN)


def uniform(key: np.uint64, n: int, start: int = 0) -> np.ndarray:
    """float64 uniforms in [0, 1)."""
    return (bits64(key, n, start) >> np.uint64(11)).astype(np.float64) * _TWO_M53


def normal(key: np.uint64, n: int) -> np.ndarray:
    """float64 standard normals by Box-Muller (both branches used)."""
    h = (n + 1) // 2
    w = bits64(key, 2 * h)
    u1 = ((w[:h] >> np.uint64(11)).astype(np.float64) + 1.0) * _TWO_M53   # (0, 1]
    u2 = (w[h:] >> np.uint64(11)).astype(np.float64) * _TWO_M53           # [0, 1)
    r = np.sqrt(-2.0 * np.log(u1))
    t = 2.0 * np.pi * u2
    out = np.empty(2 * h, dtype=np.float64)
    out[:h] = r * np.cos(t)
    out[h:] = r * np.sin(t)
    return out[:n]


def randint(key: np.uint64, n: int, lo: int, hi: int) -> np.ndarray:
    """int64 draws uniform on lo..hi inclusive (modulo bias < 2^-40 for small ranges)."""
    span = np.uint64(hi - lo + 1)
    return (bits64(key, n) % span).astype(np.int64) + lo


def permutation(key: np.uint64, n: int) -> np.ndarray:
    """A permutation of 0..n-1: stable argsort of n random words."""
    return np.argsort(bits64(key, n), kind="stable").astype(np.int64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)

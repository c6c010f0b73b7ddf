"""Counter-based random numbers for the synthetic inputs.

The generator is the SplitMix64 sequence (Steele, Lea, Flood, "Fast splittable
pseudorandom number generators", OOPSLA 2014): the i-th output of a stream with
key ``k`` is ``mix64(k + (i + 1) * GAMMA)``.  Because output i depends only on
(k, i) it can be evaluated for whole index ranges at once, and any slice of a
stream can be regenerated without the rest.

This module holds no arithmetic of the training method; it only makes inputs.
"""
from __future__ import annotations

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK = (1 << 64) - 1


def _mix64_int(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def stream_key(seed: int, *tags: int) -> int:
    """Derive the 64-bit key of the stream named by (seed, tags...)."""
    k = _mix64_int(int(seed) + 0x9E3779B97F4A7C15)
    for t in tags:
        k = _mix64_int(k ^ _mix64_int(int(t) + 0x632BE59BD9B4E019))
    return k


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def u64(key: int, count: int, offset: int = 0, chunk: int = 1 << 24) -> np.ndarray:
    """Outputs offset .. offset+count-1 of the stream with the given key."""
    out = np.empty(count, dtype=np.uint64)
    k = np.uint64(key & _MASK)
    with np.errstate(over="ignore"):
        for lo in range(0, count, chunk):
            hi = min(count, lo + chunk)
            idx = np.arange(offset + lo + 1, offset + hi + 1, dtype=np.uint64)
            out[lo:hi] = _mix64(k + idx * _GAMMA)
    return out


def uniform(key: int, count: int, offset: int = 0) -> np.ndarray:
    """float64 uniform on [0, 1) with 53 random bits."""
    return (u64(key, count, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def normal(key: int, count: int, offset: int = 0) -> np.ndarray:
    """float64 standard normal by the Box-Muller transform.

    Output i uses stream outputs 2i and 2i+1, so slices are reproducible.
    """
    r = u64(key, 2 * count, 2 * offset)
    u1 = ((r[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / (1 << 53))  # (0, 1]
    u2 = (r[1::2] >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def below(key: int, count: int, bound: int, offset: int = 0) -> np.ndarray:
    """int64 values in [0, bound): 64-bit output reduced by multiply-shift.

    The bias is below bound / 2**64 and irrelevant for input generation.
    """
    r = u64(key, count, offset)
    hi = (r >> np.uint64(32)).astype(np.uint64)
    lo = (r & np.uint64(0xFFFFFFFF)).astype(np.uint64)
    b = np.uint64(bound)
    with np.errstate(over="ignore"):
        # floor(r * bound / 2**64) for bound < 2**32, from the two 32-bit halves
        t = (lo * b) >> np.uint64(32)
        v = (hi * b + t) >> np.uint64(32)
    return v.astype(np.int64)

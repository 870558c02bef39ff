"""Counter-based pseudo-random numbers for the synthetic workloads.

Every draw is a pure function of (seed, stream, index), so a value does not
depend on how many other values were drawn before it or on a library's RNG
version.  The same mixing function is written again in C in ``plangen.c``;
``tests/test_workloads.py`` checks that the two agree.

The mixer is the 64-bit finaliser published by Steele, Lea and Flood for
SplitMix (``z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; ...``).

This module holds no arithmetic of the scheduling method itself.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_STREAM_MUL = np.uint64(0xD1B54A32D192ED03)


def _mix(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def key(seed: int, stream: int) -> np.uint64:
    """Per-(seed, stream) key."""
    with np.errstate(over="ignore"):
        s = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + _GOLDEN
        k = _mix(s) ^ (np.uint64(stream & 0xFFFFFFFFFFFFFFFF) * _STREAM_MUL)
        return np.uint64(_mix(k + _GOLDEN))


def u64(seed: int, stream: int, index) -> np.ndarray:
    """64 random bits for each entry of ``index`` (any integer array or scalar)."""
    idx = np.asarray(index).astype(np.uint64)
    with np.errstate(over="ignore"):
        return _mix(key(seed, stream) + (idx + np.uint64(1)) * _GOLDEN)


def uniform01(seed: int, stream: int, index) -> np.ndarray:
    """float64 in [0, 1) with 53 random bits."""
    return (u64(seed, stream, index) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def randint(seed: int, stream: int, index, lo, hi) -> np.ndarray:
    """Integers in [lo, hi] (inclusive); ``lo``/``hi`` may be arrays.  Uses the
    plain modulo reduction (bias below 2^-32 for the ranges used here)."""
    lo = np.asarray(lo, dtype=np.int64)
    hi = np.asarray(hi, dtype=np.int64)
    span = (hi - lo + 1).astype(np.uint64)
    r = u64(seed, stream, index) % span
    return lo + r.astype(np.int64)

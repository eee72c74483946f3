"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Only random numbers live here -- nothing of the method (no packed offsets, no
contractions).  Values come from a counter-based generator: element ``t`` of
stream ``seed`` is a pure function of ``(seed, t)``, so any slice of any tensor
can be regenerated independently and both the CPU oracle and the GPU library
are handed the very same bytes.

Generator: the SplitMix64 output function (Steele, Lea, Flood 2014) applied to
``seed * 0x9E3779B97F4A7C15 + t``; the top 24 bits give ``u = k / 2**24``.

* ``uniform``  : ``2u - 1``  in [-1, 1), exactly representable in fp32.
* ``uniform64``: ``2 k53 / 2**53 - 1`` from the top 53 bits, an fp64 value with a full mantissa.
* ``normal``   : Box-Muller on ``u1 = (k+1)/2**24`` and a second draw ``u2``
                 (the mix of the first word), evaluated in fp64, rounded to fp32.
* ``small_int``: integers in [lo, hi] stored as fp32 (every partial sum of
                 products of such values is exact in fp32 for the sizes tested,
                 so results do not depend on summation order).

The paper's experiments use synthetic dense-valued tensors with a structural
mask at stated sizes (Section 6.1, Table 2); these streams stand in for them.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 24


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _words(seed: int, start: int, count: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        base = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) * _GOLDEN
        t = np.arange(start, start + count, dtype=np.uint64)
        return _mix(t + base + _GOLDEN)


def _fill(kind: str, seed: int, count: int, lo: int = 0, hi: int = 0) -> np.ndarray:
    out = np.empty(count, dtype=np.float32)
    for s in range(0, count, _CHUNK):
        c = min(_CHUNK, count - s)
        z = _words(seed, s, c)
        k = (z >> np.uint64(40)).astype(np.float64)
        if kind == "uniform":
            out[s:s + c] = (k * (2.0 / (1 << 24)) - 1.0).astype(np.float32)
        elif kind == "normal":
            with np.errstate(over="ignore"):
                z2 = _mix(z + _GOLDEN)
            u1 = (k + 1.0) / (1 << 24)
            u2 = (z2 >> np.uint64(40)).astype(np.float64) / (1 << 24)
            out[s:s + c] = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
        elif kind == "small_int":
            span = hi - lo + 1
            out[s:s + c] = ((z >> np.uint64(40)) % np.uint64(span)).astype(np.float32) + np.float32(lo)
        else:
            raise ValueError(kind)
    return out


def uniform64(seed: int, *shape: int) -> np.ndarray:
    """fp64 values uniform on [-1, 1) with a full 53-bit mantissa: ``2 k / 2**53 - 1`` from the top
    53 bits of the same stream (for the double-precision entry points)."""
    count = int(np.prod(shape, dtype=np.int64))
    out = np.empty(count, dtype=np.float64)
    for s in range(0, count, _CHUNK):
        c = min(_CHUNK, count - s)
        k = (_words(seed, s, c) >> np.uint64(11)).astype(np.float64)
        out[s:s + c] = k * (2.0 / (1 << 53)) - 1.0
    return out.reshape(shape)


def uniform(seed: int, *shape: int) -> np.ndarray:
    """fp32 values uniform on [-1, 1)."""
    return _fill("uniform", seed, int(np.prod(shape, dtype=np.int64))).reshape(shape)


def normal(seed: int, *shape: int) -> np.ndarray:
    """fp32 values ~ N(0, 1)."""
    return _fill("normal", seed, int(np.prod(shape, dtype=np.int64))).reshape(shape)


def small_int(seed: int, lo: int, hi: int, *shape: int) -> np.ndarray:
    """fp32 array of integers drawn from [lo, hi]."""
    return _fill("small_int", seed, int(np.prod(shape, dtype=np.int64)), lo, hi).reshape(shape)


def band_normal(seed: int, n: int, w: int, kind: str = "normal") -> np.ndarray:
    """(2w+1, n) block of diagonals: row d+w, slot i is the matrix entry (i, i+d).

    In-range slots are drawn from the stream; slots whose column i+d lies
    outside the matrix are set to +0 (the input recipe's padding rule).
    """
    if kind == "normal":
        D = normal(seed, 2 * w + 1, n)
    elif kind == "small_int":
        D = small_int(seed, -3, 3, 2 * w + 1, n)
    else:
        D = uniform(seed, 2 * w + 1, n)
    for d in range(-w, w + 1):
        if d < 0:
            D[d + w, : min(-d, n)] = 0.0
        elif d > 0:
            D[d + w, max(n - d, 0):] = 0.0
    return D

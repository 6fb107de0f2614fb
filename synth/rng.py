"""Counter-based random numbers for the synthetic workloads.

Every value is a pure function of (seed, stream, index), so any slice of any
tensor can be regenerated independently and the same inputs reach the CPU
checker and the GPU library.  The generator is SplitMix64's output mixer
(Steele, Lea, Flood 2014) applied to a counter; nothing here knows about
convolutions, patterns or pruning.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# stream numbers (one per kind of tensor, so tensors never share draws)
STREAM_INPUT = 0
STREAM_WEIGHT = 1
STREAM_BIAS = 2
STREAM_PATTERN = 3
STREAM_CONN = 4


def _mix(z: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser on uint64 arrays (wrap-around arithmetic)."""
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def bits64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """uint64 draws number start .. start+count-1 of (seed, stream)."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([np.uint64(seed) * _GOLDEN + np.uint64(stream + 1)], dtype=np.uint64))
        key = _mix(key ^ np.uint64(0xD1B54A32D192ED03))
        idx = np.arange(start, start + count, dtype=np.uint64)
        return _mix(key[0] + (idx + np.uint64(1)) * _GOLDEN)


def uniform01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 in [0, 1) with 24 random bits (so exact in fp32, and k/2**24)."""
    h = bits64(seed, stream, start, count)
    return (h >> np.uint64(40)).astype(np.float64) * (1.0 / (1 << 24))


def normal01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """Standard normal float64 by Box-Muller on two 53-bit uniforms per draw."""
    h = bits64(seed, stream, 2 * start, 2 * count)
    u1 = ((h[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / (1 << 53))   # (0, 1]
    u2 = (h[1::2] >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))           # [0, 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def chunked(fn, seed: int, stream: int, count: int, out_dtype, post=None, chunk: int = 1 << 22) -> np.ndarray:
    """Fill a long vector in chunks so the 64-bit temporaries stay small."""
    out = np.empty(count, dtype=out_dtype)
    for s in range(0, count, chunk):
        n = min(chunk, count - s)
        v = fn(seed, stream, s, n)
        if post is not None:
            v = post(v)
        out[s:s + n] = v
    return out


def choose_k(seed: int, stream: int, total: int, k: int) -> np.ndarray:
    """Indices of a uniformly random k-subset of range(total): the k smallest
    of `total` random keys (stable, so ties fall to the lower index)."""
    keys = bits64(seed, stream, 0, total)
    order = np.argsort(keys, kind="stable")
    return np.sort(order[:k])

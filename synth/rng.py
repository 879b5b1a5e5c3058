"""Counter-based integer random numbers for the synthetic input generators.

Every draw is a pure function of (seed, stream id, counter), so any array can be
regenerated anywhere, in any chunking, without generator state.  This module holds
no arithmetic of the GCN method: it only makes inputs (graphs, features, labels,
masks, initial weights) that are then handed, as plain arrays, both to the CPU
oracle and to the GPU library.
"""
from __future__ import annotations

import numpy as np

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)
_CHUNK = 1 << 24


def _finalise(z: np.ndarray) -> np.ndarray:
    """The 64-bit avalanche mixer of the SplitMix64 generator (Steele, Lea, Flood 2014)."""
    z = z + _GOLDEN
    z = (z ^ (z >> _U64(30))) * _M1
    z = (z ^ (z >> _U64(27))) * _M2
    return z ^ (z >> _U64(31))


def _key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        s = np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=_U64)
        t = np.array([stream & 0xFFFFFFFFFFFFFFFF], dtype=_U64)
        return _finalise(_finalise(s) ^ (t * _M2))[0]


def bits(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit words: word i is mix(key(seed, stream) + (offset + i) * odd constant)."""
    out = np.empty(n, dtype=_U64)
    k = _key(seed, stream)
    with np.errstate(over="ignore"):
        for lo in range(0, n, _CHUNK):
            hi = min(n, lo + _CHUNK)
            ctr = np.arange(offset + lo, offset + hi, dtype=_U64)
            out[lo:hi] = _finalise(k + ctr * _GOLDEN)
    return out


def uniform(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n doubles in [0, 1) from the top 53 bits of each word."""
    return (bits(seed, stream, n, offset) >> _U64(11)).astype(np.float64) * (1.0 / (1 << 53))


def integers(seed: int, stream: int, n: int, high: int, offset: int = 0) -> np.ndarray:
    """n integers in [0, high) (int64); high < 2**31 so the multiply-shift is exact enough."""
    assert 0 < high < (1 << 31)
    top = bits(seed, stream, n, offset) >> _U64(32)
    return ((top * _U64(high)) >> _U64(32)).astype(np.int64)


def normal_f32(seed: int, stream: int, n: int) -> np.ndarray:
    """n standard normals (float32) by Box-Muller on pairs of uniforms, generated in chunks."""
    out = np.empty(n, dtype=np.float32)
    half = (n + 1) // 2
    step = _CHUNK
    for lo in range(0, half, step):
        hi = min(half, lo + step)
        u1 = uniform(seed, stream, hi - lo, 2 * lo)
        u2 = uniform(seed, stream, hi - lo, 2 * lo + (hi - lo))
        # distinct counters per chunk: first (hi-lo) words feed u1, the next (hi-lo) feed u2
        r = np.sqrt(-2.0 * np.log1p(-u1))
        a = 2.0 * np.pi * u2
        z0 = (r * np.cos(a)).astype(np.float32)
        z1 = (r * np.sin(a)).astype(np.float32)
        n0 = min(n, 2 * hi) - 2 * lo
        blk = np.empty(2 * (hi - lo), dtype=np.float32)
        blk[0::2] = z0
        blk[1::2] = z1
        out[2 * lo:2 * lo + n0] = blk[:n0]
    return out


def permutation(seed: int, stream: int, n: int) -> np.ndarray:
    """A permutation of 0..n-1: argsort of n random words (ties broken by index)."""
    return np.argsort(bits(seed, stream, n), kind="stable").astype(np.int64)

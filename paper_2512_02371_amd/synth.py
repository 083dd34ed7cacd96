"""Seeded synthetic inputs for the five image stages.

This module only *draws numbers*: images, taps and weights with the value
distributions of the benchmark configurations.  It contains none of the
stages' arithmetic, and it is the only module that both the fp64 test oracle
and the HIP path's tests/benchmarks may share.

Every draw is a pure function of (seed, linear index): a counter-based
SplitMix64 hash, so any sub-range can be regenerated independently and the
same bits come out on every machine.

All fp16 data is returned as ``numpy.uint16`` bit patterns (IEEE binary16).
"""
from __future__ import annotations

import math

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser (Steele, Lea, Flood 2014) on a uint64 array."""
    with np.errstate(over="ignore"):
        z = z + _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def hash_u64(seed: int, start: int, count: int, stream: int = 0) -> np.ndarray:
    """64 hashed bits for linear indices start .. start+count-1 of (seed, stream)."""
    key = _mix(np.array([(seed * 0x1000193 + stream) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))
    idx = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(idx * np.uint64(0xD1342543DE82EF95) + key[0])


def _f16_bits(x: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(x.astype(np.float16)).view(np.uint16)


def uniform01_f16(seed: int, shape, chunk: int = 1 << 24) -> np.ndarray:
    """Uniform multiples of 2^-11 in [0, 1): exactly representable in fp16."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        h = hash_u64(seed, s, c) >> np.uint64(53)          # 11 bits
        out[s:s + c] = _f16_bits(h.astype(np.float64) / 2048.0)
    return out.reshape(shape)


def uniform_pm1_f16(seed: int, shape, chunk: int = 1 << 24) -> np.ndarray:
    """Uniform multiples of 2^-10 in [-1, 1): exactly representable in fp16."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        h = hash_u64(seed, s, c) >> np.uint64(53)
        out[s:s + c] = _f16_bits((h.astype(np.float64) - 1024.0) / 1024.0)
    return out.reshape(shape)


def binary01_f16(seed: int, shape) -> np.ndarray:
    """Values in {0, 1}: every partial sum of such an image is an integer."""
    n = int(np.prod(shape))
    h = hash_u64(seed, 0, n) >> np.uint64(63)
    return _f16_bits(h.astype(np.float64)).reshape(shape)


def normal_f16(seed: int, shape, std: float) -> np.ndarray:
    """N(0, std^2) by Box-Muller on two hashed uniforms, rounded once to fp16."""
    n = int(np.prod(shape))
    u1 = ((hash_u64(seed, 0, n, stream=1) >> np.uint64(11)).astype(np.float64) + 1.0) / 9007199254740993.0
    u2 = (hash_u64(seed, 0, n, stream=2) >> np.uint64(11)).astype(np.float64) / 9007199254740992.0
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    return _f16_bits(z * std).reshape(shape)


def random_taps_f16(seed: int, ntaps: int) -> np.ndarray:
    """ntaps uniform [0,1) draws, normalised to sum 1 in fp64, rounded once to fp16."""
    h = hash_u64(seed, 0, ntaps) >> np.uint64(11)
    t = (h.astype(np.float64) + 0.5) / 9007199254740992.0
    return _f16_bits(t / t.sum())


def random_kernel2d_f16(seed: int, kh: int, kw: int) -> np.ndarray:
    """kh x kw signed draws from (-1, 1), scaled to sum |k| = 1 in fp64, rounded once to fp16
    (a generic non-separable filter: no rank-1 structure, both signs)."""
    h = hash_u64(seed, 0, kh * kw) >> np.uint64(11)
    t = (h.astype(np.float64) + 0.5) / 4503599627370496.0 - 1.0
    return _f16_bits(t / np.abs(t).sum()).reshape(kh, kw)


def gaussian_taps_f16(ntaps: int, sigma: float) -> np.ndarray:
    """Sampled Gaussian centred on (ntaps-1)/2, normalised in fp64, rounded once to fp16."""
    r = np.arange(ntaps, dtype=np.float64) - (ntaps - 1) / 2.0
    g = np.exp(-(r * r) / (2.0 * sigma * sigma))
    return _f16_bits(g / g.sum())


def f16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Numpy's own half -> double conversion (used by tests, not by the oracle)."""
    return np.ascontiguousarray(bits).view(np.float16).astype(np.float64)


def f64_to_f16_bits(x: np.ndarray) -> np.ndarray:
    return _f16_bits(np.asarray(x, dtype=np.float64))


# The five benchmark configurations (shape, taps, anchors, seeds).
CONFIGS = {
    "fir1d": dict(H=256, W=256, ntaps=8, anchor=3, seed_img=1001, seed_taps=2001),
    "sepblur": dict(H=4096, W=4096, ntaps=16, anchor=7, sigma=3.0, seed_img=1002),
    "sat2d": dict(H=4096, W=4096, seed_img=1003),
    "conv3x3": dict(N=1, H=1024, W=1024, Cin=64, Cout=64, seed_img=1004, seed_w=2004),
    "pyr_level": dict(H=8192, W=8192, seed_img=1005),
}

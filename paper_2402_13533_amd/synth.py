"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the layer itself: it only draws numbers and
changes their storage format (fp32 -> bf16 bit patterns and back).  Both the HIP
library's callers and the CPU oracle's callers receive the *same bytes* from
here, so neither side's result depends on a library RNG version.

Generator: counter-based.  Element pair i of a tensor drawn with seed s comes
from splitmix64(mix(s) + i): the upper and lower 32 bits give two uniforms, one
Box-Muller transform in fp64 gives two standard normals, which are cast to fp32.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22

BASE_SEED = 20240213 * 1000


def tensor_seed(config: int, tensor_index: int) -> int:
    """Seed convention: one seed per (config, tensor)."""
    return BASE_SEED + 100 * config + tensor_index


def _splitmix64(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _seed_base(seed: int) -> np.uint64:
    s = np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _splitmix64(s + _GOLDEN)[0]


def uniform_bits(seed: int, n: int) -> np.ndarray:
    """n 64-bit words of the counter-based stream for `seed`."""
    base = _seed_base(seed)
    out = np.empty(n, dtype=np.uint64)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        ctr = np.arange(lo + 1, hi + 1, dtype=np.uint64)
        with np.errstate(over="ignore"):
            out[lo:hi] = _splitmix64(base + ctr * _GOLDEN)
    return out


def normal(seed: int, shape, std: float = 1.0) -> np.ndarray:
    """fp32 tensor of N(0, std^2) samples, deterministic in (seed, shape)."""
    shape = tuple(int(s) for s in np.atleast_1d(shape))
    n = int(np.prod(shape)) if shape else 1
    out = np.empty(n + (n & 1), dtype=np.float32)
    half = out.size // 2
    base = _seed_base(seed)
    for lo in range(0, half, _CHUNK):
        hi = min(half, lo + _CHUNK)
        ctr = np.arange(lo + 1, hi + 1, dtype=np.uint64)
        with np.errstate(over="ignore"):
            z = _splitmix64(base + ctr * _GOLDEN)
        u1 = ((z >> np.uint64(32)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
        u2 = ((z & np.uint64(0xFFFFFFFF)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
        rad = np.sqrt(-2.0 * np.log(u1)) * std
        ang = (2.0 * np.pi) * u2
        out[2 * lo:2 * hi:2] = rad * np.cos(ang)
        out[2 * lo + 1:2 * hi:2] = rad * np.sin(ang)
    return out[:n].reshape(shape)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    with np.errstate(over="ignore"):
        r = (u + rounding) >> np.uint32(16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    r = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> fp32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(seed: int, shape, std: float = 1.0) -> np.ndarray:
    """bf16 bit patterns (uint16) of N(0, std^2) samples."""
    return f32_to_bf16_bits(normal(seed, shape, std))

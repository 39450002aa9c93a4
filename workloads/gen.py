"""Seeded synthetic tensors for the five benchmark configurations.

This module serves both the CPU oracle's tests and the GPU path's tests and benchmark.  It holds
none of the method's arithmetic (no quantization, no scales, no layers): it only draws real-valued
or integer-valued tensors from a counter-based generator so that every consumer sees the same
numbers regardless of library versions.

Generator: splitmix64 applied to (seed, element index); uniform doubles from the top 53 bits;
normals by Box-Muller on two independent streams.  Everything is computed in fp64 and cast by
the caller.
"""
import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def bits(seed: int, count: int, stream: int = 0) -> np.ndarray:
    """count 64-bit words; word i of (seed, stream) depends on nothing but (seed, stream, i)."""
    with np.errstate(over="ignore"):
        base = _mix(np.uint64(seed) * _GOLD + np.uint64(stream + 1) * _M1)
        idx = np.arange(1, count + 1, dtype=np.uint64)
        return _mix(base + idx * _GOLD)


def uniform(seed: int, shape, lo: float = 0.0, hi: float = 1.0, stream: int = 0) -> np.ndarray:
    """fp64 uniform on [lo, hi)."""
    n = int(np.prod(shape))
    u = (bits(seed, n, stream) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)
    return (lo + (hi - lo) * u).reshape(shape)


def normal(seed: int, shape, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """fp64 normal(mean, std) by Box-Muller (one output per pair of uniforms)."""
    n = int(np.prod(shape))
    u1 = ((bits(seed, n, 0) >> np.uint64(11)).astype(np.float64) + 1.0) * (2.0 ** -53)  # (0, 1]
    u2 = (bits(seed, n, 1) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)          # [0, 1)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (mean + std * z).reshape(shape)


def integers(seed: int, shape, lo: int, hi: int) -> np.ndarray:
    """int64 uniform on [lo, hi] (inclusive)."""
    n = int(np.prod(shape))
    span = np.uint64(hi - lo + 1)
    v = (bits(seed, n, 0) >> np.uint64(16)) % span
    return (v.astype(np.int64) + lo).reshape(shape)


def permutation(seed: int, n: int) -> np.ndarray:
    """A seeded permutation of range(n) (argsort of n distinct-with-probability-1 words)."""
    return np.argsort(bits(seed, n, 2), kind="stable")

"""Seeded synthetic inputs shared by the oracle-side tests and the GPU harness.

Holds none of the method's arithmetic: a counter-based generator (splitmix64),
uniform / normal / small-integer matrices, and round-to-nearest-even storage in
fp32 / bf16 / fp16.  The same bit patterns are what the CPU oracle (after exact
widening to fp64) and the GPU library consume.

Storage dtypes are named "f32", "bf16", "f16".  A stored matrix is a numpy array
of float32 (f32), uint16 holding bfloat16 bits (bf16) or float16 (f16).
"""
from __future__ import annotations

import numpy as np

DTYPES = ("f32", "bf16", "f16")
_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def splitmix64(x: np.ndarray) -> np.ndarray:
    """The splitmix64 output function applied to each 64-bit counter."""
    with np.errstate(over="ignore"):
        z = (x + np.uint64(0x9E3779B97F4A7C15)) & _MASK
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK
        return z ^ (z >> np.uint64(31))


def _bits(seed: int, stream: int, count: int) -> np.ndarray:
    """count 64-bit words of stream `stream` under `seed` (pure function of its arguments)."""
    with np.errstate(over="ignore"):
        base = splitmix64(np.array([np.uint64(seed) * np.uint64(0x100000001B3) + np.uint64(stream)],
                                   dtype=np.uint64))[0]
        ctr = np.arange(count, dtype=np.uint64) + base
    return splitmix64(ctr)


def _unit(seed: int, stream: int, count: int) -> np.ndarray:
    """Uniform doubles in (0, 1): top 53 bits, offset by half a step so 0 never occurs."""
    return ((_bits(seed, stream, count) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def uniform(seed: int, stream: int, shape, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    n = int(np.prod(shape))
    return (lo + (hi - lo) * _unit(seed, stream, n)).reshape(shape)


def normal(seed: int, stream: int, shape, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """Box-Muller on pairs of uniforms; element 2t uses the cosine branch, 2t+1 the sine branch."""
    n = int(np.prod(shape))
    half = (n + 1) // 2
    u1 = _unit(seed, 2 * stream, half)
    u2 = _unit(seed, 2 * stream + 1, half)
    rad = np.sqrt(-2.0 * np.log(u1))
    out = np.empty(2 * half, np.float64)
    out[0::2] = rad * np.cos(2.0 * np.pi * u2)
    out[1::2] = rad * np.sin(2.0 * np.pi * u2)
    return (mean + std * out[:n]).reshape(shape)


def integers(seed: int, stream: int, shape, lo: int = -3, hi: int = 3) -> np.ndarray:
    """Integers uniform on [lo, hi] as int64 (exactly representable in every storage dtype here)."""
    n = int(np.prod(shape))
    span = np.uint64(hi - lo + 1)
    return ((_bits(seed, stream, n) >> np.uint64(16)) % span).astype(np.int64).reshape(shape) + lo


def store(values: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to the storage dtype, nearest-even."""
    if dtype == "f32":
        return np.asarray(values, np.float64).astype(np.float32)
    if dtype == "f16":
        return np.asarray(values, np.float64).astype(np.float32).astype(np.float16)
    if dtype == "bf16":
        f = np.ascontiguousarray(np.asarray(values, np.float64).astype(np.float32))
        u = f.view(np.uint32)
        bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        return ((u + bias) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


def widen(stored: np.ndarray, dtype: str) -> np.ndarray:
    """The exact fp64 value of every stored element."""
    if dtype == "bf16":
        return (stored.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return stored.astype(np.float64)


def matrices(kind_a: str, kind_b: str, M: int, N: int, K: int, dtype: str, seed: int):
    """(A_stored, B_stored) for a named distribution pair.

    kinds: "uniform" U[-1,1]; "normal" N(0,1); "weights" N(0,0.02^2); "int" integers in [-3,3].
    Stream 1 feeds A, stream 2 feeds B.
    """
    def one(kind, stream, shape):
        if kind == "uniform":
            return uniform(seed, stream, shape)
        if kind == "normal":
            return normal(seed, stream, shape)
        if kind == "weights":
            return normal(seed, stream, shape, 0.0, 0.02)
        if kind == "int":
            return integers(seed, stream, shape).astype(np.float64)
        raise ValueError(kind)
    return store(one(kind_a, 1, (M, K)), dtype), store(one(kind_b, 2, (K, N)), dtype)

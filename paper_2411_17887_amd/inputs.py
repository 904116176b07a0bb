"""Seeded synthetic inputs.  Holds none of the method's arithmetic.

Element i of every stream is a pure function of (seed, i): a SplitMix64 finaliser applied
to the counter ``seed + (i+1) * 0x9E3779B97F4A7C15``.  The same host buffer is handed to the
CPU oracle and uploaded to the GPU, so both sides see identical bits.  The paper has no
workloads or datasets; the distributions below are the ones the five benchmark
configurations name.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 241117887
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    """uint64 outputs for counters start .. start+count-1."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def _fill(n: int, dtype, fn) -> np.ndarray:
    out = np.empty(n, dtype=dtype)
    for a in range(0, n, _CHUNK):
        b = min(n, a + _CHUNK)
        out[a:b] = fn(a, b - a)
    return out


def int32_small(n: int, seed: int) -> np.ndarray:
    """int32 uniform in [-128, 127] (top 8 bits of the stream minus 128)."""
    return _fill(n, np.int32, lambda a, c: (splitmix64(seed, a, c) >> np.uint64(56)).astype(np.int32) - 128)


def int32_full(n: int, seed: int) -> np.ndarray:
    """int32 over the whole range (low 32 bits of the stream); sums wrap modulo 2^32."""
    return _fill(n, np.int32, lambda a, c: (splitmix64(seed, a, c) & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.int32))


def int8_full(n: int, seed: int) -> np.ndarray:
    """int8 over the whole range [-128, 127]."""
    return _fill(n, np.int8, lambda a, c: (splitmix64(seed, a, c) >> np.uint64(56)).astype(np.uint8).view(np.int8))


def mask_i8(n: int, seed: int) -> np.ndarray:
    """int8 in {0, 1} with P(1) = 1/2 (top bit of the stream): a stream-compaction mask."""
    return _fill(n, np.int8, lambda a, c: (splitmix64(seed, a, c) >> np.uint64(63)).astype(np.int8))


def _uniform24(seed: int, a: int, c: int) -> np.ndarray:
    return (splitmix64(seed, a, c) >> np.uint64(40)).astype(np.float32) * np.float32(2.0 ** -24)


def f16_uniform01(n: int, seed: int) -> np.ndarray:
    """float16 uniform in [0, 1): 24-bit uniform in fp32, rounded to nearest-even, kept below 1."""
    def fn(a, c):
        h = _uniform24(seed, a, c).astype(np.float16)
        h[h >= np.float16(1.0)] = np.float16(0.99951171875)   # largest half below 1
        return h
    return _fill(n, np.float16, fn)


def f32_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bfloat16 bit patterns (uint16).  No NaN/Inf handling needed here."""
    u = np.ascontiguousarray(v, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_uniform_pm1(n: int, seed: int) -> np.ndarray:
    """bfloat16 bit patterns (uint16) of values uniform in [-1, 1], rounded from fp32."""
    return _fill(n, np.uint16, lambda a, c: f32_to_bf16_bits(np.float32(2.0) * _uniform24(seed, a, c) - np.float32(1.0)))


def f32_normal(n: int, seed: int) -> np.ndarray:
    """float32 standard normal: Box-Muller in fp64 on two 53-bit uniforms per element."""
    def fn(a, c):
        z = splitmix64(seed, 2 * a, 2 * c)
        u1 = ((z[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53      # (0, 1]
        u2 = (z[1::2] >> np.uint64(11)).astype(np.float64) * 2.0 ** -53              # [0, 1)
        return (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    return _fill(n, np.float32, fn)


def tri_f32(n: int, seed: int) -> np.ndarray:
    """float32 values in {-1, 0, 1}: every partial sum is an integer below 2^24 in magnitude for
    n < 2^24, so fp32 summation is exact in any order."""
    return _fill(n, np.float32, lambda a, c: (splitmix64(seed, a, c) % np.uint64(3)).astype(np.float32) - np.float32(1.0))


def tri_f16(n: int, seed: int) -> np.ndarray:
    return tri_f32(n, seed).astype(np.float16)


def tri_bf16_bits(n: int, seed: int) -> np.ndarray:
    return f32_to_bf16_bits(tri_f32(n, seed))


# ------------------------------------------------------------ the five configurations
# name -> (call, kind, rows, cols, generator, gate)
CONFIGS = {
    "C1": dict(call="inclusive", kind="i32", rows=1, cols=4096, gen=int32_small, seed=BASE_SEED + 0, exact=True),
    "C2": dict(call="inclusive", kind="f16", rows=1, cols=1 << 24, gen=f16_uniform01, seed=BASE_SEED + 1, tol=1e-3),
    "C3": dict(call="exclusive", kind="i8", rows=1, cols=1 << 28, gen=mask_i8, seed=BASE_SEED + 2, exact=True),
    "C4": dict(call="inclusive", kind="f32", rows=1, cols=100_000_007, gen=f32_normal, seed=BASE_SEED + 3, tol=1e-5),
    "C5": dict(call="batched", kind="bf16", rows=4096, cols=65536, gen=bf16_uniform_pm1, seed=BASE_SEED + 4, tol=1e-3),
}


def make_config(name: str) -> np.ndarray:
    c = CONFIGS[name]
    return c["gen"](c["rows"] * c["cols"], c["seed"])

"""Seeded synthetic inputs for the fp16 reduction (numpy only, host side).

This module holds input generators and nothing else: no summation, no piece
of the reduction method.  Both the oracle-side tests and the GPU-side tests /
benchmark draw their inputs from here so that they see identical bits.

The paper's workloads are synthetic (normal(0,1) and uniform[0,1] arrays,
Sections 5.1, 5.4 and 6); the generators reproduce those distributions with a
counter-based PRNG so that any slice [lo, hi) of a stream can be produced on
its own and in parallel:

    u64(i) = mix(seed + (i + 1) * 0x9E3779B97F4A7C15)        (splitmix64 stream)
    uniform = (u64 >> 11) / 2^53  in [0, 1)
    normal  = Box-Muller on the uniforms of counters 2i and 2i+1

Values are rounded to binary16 with round-to-nearest-even (numpy's conversion);
a rounded-up endpoint of a half-open interval is clamped to the largest fp16
below it, and normals are clamped to +-65504.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 21

# One base seed, offset by the configuration number (configs 1..5).
BASE_SEED = 20010558500


def config_seed(config: int) -> int:
    return BASE_SEED + int(config)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _C1
    z = (z ^ (z >> np.uint64(27))) * _C2
    return z ^ (z >> np.uint64(31))


def u64_stream(seed: int, lo: int, hi: int) -> np.ndarray:
    """Counters lo..hi-1 of the splitmix64 stream of ``seed`` (uint64)."""
    with np.errstate(over="ignore"):
        i = np.arange(lo + 1, hi + 1, dtype=np.uint64)
        return _mix(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + i * GOLDEN)


def _unit(seed: int, lo: int, hi: int) -> np.ndarray:
    return (u64_stream(seed, lo, hi) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


_BELOW_ONE = np.float16(0.99951171875)          # 0x3BFF, largest fp16 < 1


def _uniform01(seed, lo, hi):
    h = _unit(seed, lo, hi).astype(np.float16)
    np.minimum(h, _BELOW_ONE, out=h)
    return h


def _uniform_pm1(seed, lo, hi):
    h = (2.0 * _unit(seed, lo, hi) - 1.0).astype(np.float16)
    np.minimum(h, _BELOW_ONE, out=h)
    return h


def _normal(seed, lo, hi):
    u = _unit(seed ^ 0x5851F42D4C957F2D, 2 * lo, 2 * hi)
    u1 = 1.0 - u[0::2]                           # (0, 1]: log is finite
    u2 = u[1::2]
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    np.clip(z, -65504.0, 65504.0, out=z)
    return z.astype(np.float16)


_KINDS = {"uniform01": _uniform01, "uniform_pm1": _uniform_pm1, "normal": _normal}


def generate(kind: str, n: int, seed: int, offset: int = 0, out: np.ndarray | None = None,
             threads: int | None = None) -> np.ndarray:
    """fp16 array of elements offset..offset+n-1 of stream (kind, seed)."""
    fn = _KINDS[kind]
    if out is None:
        out = np.empty(n, dtype=np.float16)
    if out.shape != (n,) or out.dtype != np.float16:
        raise ValueError("out must be a float16 array of length n")
    if n == 0:
        return out
    spans = [(s, min(s + _CHUNK, n)) for s in range(0, n, _CHUNK)]

    def work(span):
        a, b = span
        out[a:b] = fn(seed, offset + a, offset + b)

    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    if len(spans) == 1 or threads <= 1:
        for s in spans:
            work(s)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, spans))
    return out


def to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """float -> bfloat16 storage bits (uint16), round to nearest even; NaN stays NaN."""
    w = np.ascontiguousarray(v, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((w >> np.uint32(16)) & np.uint32(1))
    with np.errstate(over="ignore"):
        r = ((w + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(np.asarray(v, dtype=np.float32))
    if nan.any():
        r[nan] = np.uint16(0x7FC0)
    return r


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def generate_f32(kind: str, n: int, seed: int, offset: int = 0) -> np.ndarray:
    """float32 array of the same streams (values rounded to binary32 instead of binary16)."""
    out = np.empty(n, dtype=np.float32)
    for a in range(0, n, _CHUNK):
        b = min(a + _CHUNK, n)
        lo, hi = offset + a, offset + b
        if kind == "uniform01":
            out[a:b] = np.minimum(_unit(seed, lo, hi).astype(np.float32), np.float32(1.0 - 2.0 ** -24))
        elif kind == "uniform_pm1":
            out[a:b] = np.minimum((2.0 * _unit(seed, lo, hi) - 1.0).astype(np.float32), np.float32(1.0 - 2.0 ** -24))
        elif kind == "normal":
            u = _unit(seed ^ 0x5851F42D4C957F2D, 2 * lo, 2 * hi)
            out[a:b] = (np.sqrt(-2.0 * np.log(1.0 - u[0::2])) * np.cos(2.0 * np.pi * u[1::2])).astype(np.float32)
        else:
            raise KeyError(kind)
    return out


def generate_bf16(kind: str, n: int, seed: int, offset: int = 0) -> np.ndarray:
    """bfloat16 storage bits (uint16) of the same streams."""
    bits = to_bf16_bits(generate_f32(kind, n, seed, offset))
    if kind in ("uniform01", "uniform_pm1"):
        bits[bits == 0x3F80] = 0x3F7F          # a rounded-up 1.0 -> largest bfloat16 below 1
    return bits


# --- closed-form patterns (all values are small integers, hence fp16-exact) ---

def ones(n: int) -> np.ndarray:
    return np.ones(n, dtype=np.float16)


def constant(n: int, c: float) -> np.ndarray:
    h = np.float16(c)
    if float(h) != float(c):
        raise ValueError("constant %r is not fp16-exact" % (c,))
    return np.full(n, h, dtype=np.float16)


def periodic_ramp(n: int, period: int, step: float = 1.0) -> np.ndarray:
    """x_i = (i mod period) * step; fp16-exact for period <= 2048, step = 2^k."""
    if period < 1 or period > 2048:
        raise ValueError("period must be in 1..2048 for fp16-exact values")
    v = (np.arange(n, dtype=np.int64) % period).astype(np.float64) * step
    h = v.astype(np.float16)
    if n and not np.array_equal(h.astype(np.float64), v):
        raise ValueError("ramp values are not fp16-exact")
    return h


def alternating(n: int, c: float = 1.0) -> np.ndarray:
    """x_i = (-1)^i * c."""
    h = constant(n, c)
    h[1::2] = -h[1::2]
    return h


def one_hot(n: int, p: int, value: float = 1.0) -> np.ndarray:
    h = np.zeros(n, dtype=np.float16)
    h[p] = np.float16(value)
    return h


def prefix_indicator(n: int, k: int) -> np.ndarray:
    """x_i = 1 if i < k else 0."""
    h = np.zeros(n, dtype=np.float16)
    h[:k] = np.float16(1.0)
    return h


def small_integers(n: int, seed: int, lo: int = -8, hi: int = 8) -> np.ndarray:
    """Seeded integers in [lo, hi]: any summation order is exact in fp32 while
    n * max(|lo|, |hi|) <= 2^24."""
    if n == 0:
        return np.zeros(0, dtype=np.float16)
    span = np.uint64(hi - lo + 1)
    v = (u64_stream(seed, 0, n) % span).astype(np.int64) + lo
    return v.astype(np.float16)

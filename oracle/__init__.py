"""CPU oracle for the fp16 -> fp32 arithmetic reduction (test infrastructure).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library
and never imports it.

* ``sum_f16``           fp64 Kahan serial sum, the definition R(X) = sum x_i
                        (paper Section 4) -- the value GPU results are held to.
* ``sum_f16_naive``     uncompensated fp64 serial sum (the paper's own CPU
                        comparison, Section 5.4).
* ``sum_f16_blocked``   the same Kahan oracle over host threads (baseline timing).
* ``exact_sum_f16``     exact 128-bit integer sum in units of 2^-24 (a pin for
                        the oracle, independent decoder).
* ``mma_model``         fp64 model of the ones-matrix MMA encoding (Section 4.1,
                        4.3) used to pin the encoding identities.
* ``recurrence_model``  the recurrence variant with its binary16 partials (Section 5.1).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SOURCES = ("oracle_sum.c", "exact_check.c")
_CFLAGS = ("-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-pthread")

_lib = None


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc into ``oracle/liboracle.so``."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES]
    if not force and os.path.exists(_LIB_PATH):
        newest = max(os.path.getmtime(s) for s in srcs)
        if os.path.getmtime(_LIB_PATH) >= newest:
            return _LIB_PATH
    tmp = _LIB_PATH + ".tmp%d" % os.getpid()
    subprocess.run(["gcc", *_CFLAGS, "-o", tmp, *srcs, "-lm"], check=True)
    os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    dp = ctypes.POINTER(ctypes.c_double)
    lib.oracle_fp16_to_f64.argtypes = [ctypes.c_uint16]
    lib.oracle_fp16_to_f64.restype = ctypes.c_double
    lib.oracle_sum_f16.argtypes = [u16p, ctypes.c_size_t, dp, dp]
    lib.oracle_sum_f16.restype = None
    lib.oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
    lib.oracle_bf16_to_f64.restype = ctypes.c_double
    lib.oracle_f32_bits_to_f64.argtypes = [ctypes.c_uint32]
    lib.oracle_f32_bits_to_f64.restype = ctypes.c_double
    lib.oracle_sum_bf16.argtypes = [u16p, ctypes.c_size_t, dp, dp]
    lib.oracle_sum_bf16.restype = None
    lib.oracle_sum_f32.argtypes = [ctypes.POINTER(ctypes.c_uint32), ctypes.c_size_t, dp, dp]
    lib.oracle_sum_f32.restype = None
    lib.oracle_sum_f16_naive.argtypes = [u16p, ctypes.c_size_t, dp]
    lib.oracle_sum_f16_naive.restype = None
    lib.oracle_sum_f16_blocked.argtypes = [u16p, ctypes.c_size_t, ctypes.c_int, dp, dp]
    lib.oracle_sum_f16_blocked.restype = ctypes.c_int
    lib.exact_sum_f16.argtypes = [u16p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_uint64)]
    lib.exact_sum_f16.restype = ctypes.c_size_t
    _lib = lib
    return lib


def _bits(x) -> np.ndarray:
    """View an fp16 / uint16 1-D array as contiguous uint16 storage bits."""
    a = np.asarray(x)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("oracle expects float16 values or their uint16 bits, got %s" % a.dtype)
    if a.ndim != 1:
        raise ValueError("oracle expects a 1-D array")
    return np.ascontiguousarray(a)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def fp16_to_f64(bits: int) -> float:
    return float(_load().oracle_fp16_to_f64(ctypes.c_uint16(int(bits) & 0xFFFF)))


def sum_f16(x):
    """(sum, sum_abs) of fp16 array ``x`` as Python floats (binary64, Kahan)."""
    a = _bits(x)
    s, sa = ctypes.c_double(), ctypes.c_double()
    _load().oracle_sum_f16(_ptr(a), a.size, ctypes.byref(s), ctypes.byref(sa))
    return s.value, sa.value


def bf16_to_f64(bits: int) -> float:
    return float(_load().oracle_bf16_to_f64(ctypes.c_uint16(int(bits) & 0xFFFF)))


def f32_bits_to_f64(bits: int) -> float:
    return float(_load().oracle_f32_bits_to_f64(ctypes.c_uint32(int(bits) & 0xFFFFFFFF)))


def sum_bf16(x):
    """(sum, sum_abs) of bfloat16 values given as uint16 storage bits."""
    a = np.ascontiguousarray(np.asarray(x))
    if a.dtype != np.uint16 or a.ndim != 1:
        raise TypeError("sum_bf16 expects a 1-D uint16 array of bfloat16 bits")
    s, sa = ctypes.c_double(), ctypes.c_double()
    _load().oracle_sum_bf16(_ptr(a), a.size, ctypes.byref(s), ctypes.byref(sa))
    return s.value, sa.value


def sum_f32(x):
    """(sum, sum_abs) of binary32 values (float32 array or its uint32 bits)."""
    a = np.ascontiguousarray(np.asarray(x))
    if a.dtype == np.float32:
        a = a.view(np.uint32)
    if a.dtype != np.uint32 or a.ndim != 1:
        raise TypeError("sum_f32 expects a 1-D float32 / uint32 array")
    s, sa = ctypes.c_double(), ctypes.c_double()
    _load().oracle_sum_f32(a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), a.size,
                           ctypes.byref(s), ctypes.byref(sa))
    return s.value, sa.value


def sum_rows(x2d, dtype: str = "f16"):
    """Per-row (sum, sum_abs) arrays of a 2-D array: one oracle call per row."""
    fn = {"f16": sum_f16, "bf16": sum_bf16, "f32": sum_f32}[dtype]
    a = np.asarray(x2d)
    res = [fn(np.ascontiguousarray(a[r])) for r in range(a.shape[0])]
    return (np.array([r[0] for r in res], dtype=np.float64), np.array([r[1] for r in res], dtype=np.float64))


def sum_f16_naive(x) -> float:
    a = _bits(x)
    s = ctypes.c_double()
    _load().oracle_sum_f16_naive(_ptr(a), a.size, ctypes.byref(s))
    return s.value


def sum_f16_blocked(x, threads: int):
    """(sum, sum_abs, threads_used): the Kahan oracle over ``threads`` host threads."""
    a = _bits(x)
    s, sa = ctypes.c_double(), ctypes.c_double()
    used = _load().oracle_sum_f16_blocked(_ptr(a), a.size, int(threads),
                                          ctypes.byref(s), ctypes.byref(sa))
    if used < 0:
        raise MemoryError("oracle_sum_f16_blocked: allocation failed")
    return s.value, sa.value, max(1, used)


def exact_sum_f16(x):
    """Exact (sum, sum_abs) as ``fractions.Fraction`` plus the non-finite count."""
    a = _bits(x)
    out = (ctypes.c_uint64 * 4)()
    bad = _load().exact_sum_f16(_ptr(a), a.size, out)
    s = out[0] | (out[1] << 64)
    if s >= 1 << 127:
        s -= 1 << 128
    sa = out[2] | (out[3] << 64)
    return Fraction(s, 1 << 24), Fraction(sa, 1 << 24), int(bad)


def tolerance(sum_abs: float) -> float:
    """Acceptance bound for a GPU fp32 result: |gpu - sum| <= 1e-5 * sum |x_i|."""
    return 1e-5 * sum_abs

"""ctypes binding of ``libmfreduce.so``: argument marshalling only.

Every function has the name and argument order of its C declaration in
``include/mfreduce.h``; all arithmetic happens inside the library's HIP
kernels.  There is no CPU fallback: if the library has not been built,
loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmfreduce.so")

MFR_OK, MFR_ERR_INVALID_ARG, MFR_ERR_UNSUPPORTED, MFR_ERR_HIP, MFR_ERR_SCRATCH_LIMIT = 0, 1, 2, 3, 4
MFR_KERNEL_MFMA, MFR_KERNEL_SHFL, MFR_KERNEL_SPLIT = 0, 1, 2
MFR_GRID_AUTO, MFR_GRID_ONE_CHAIN = 0, -1
MFR_COMBINE_AUTO, MFR_COMBINE_SINGLE_LAUNCH, MFR_COMBINE_TWO_LAUNCHES = 0, 1, 2

MFR_DTYPE_F16, MFR_DTYPE_BF16, MFR_DTYPE_F32 = 0, 1, 2

EXPORTS = ("mfr_sum_f16", "mfr_sum_f16_tuned", "mfr_sum_f16_ex", "mfr_sum_f16_noalloc", "mfr_sum_f16_stamped", "mfr_wall_clock_khz", "mfr_sum_bf16", "mfr_sum_f32", "mfr_sum_ex",
           "mfr_sum_rows_ex", "mfr_sum_f16_rows", "mfr_sum_f16_recurrence", "mfr_sum_f16_f64", "mfr_sum_f16_f64_ex", "mfr_get_default_tuning", "mfr_grid_for", "mfr_plan_for",
           "mfr_plan_ex", "mfr_rows_plan", "mfr_rows_geometry", "mfr_release_scratch", "mfr_strerror", "mfr_last_hip_error", "mfr_version")


class mfr_tuning(ctypes.Structure):
    _fields_ = [("block_threads", ctypes.c_int), ("chain_R", ctypes.c_int),
                ("grid_blocks", ctypes.c_int), ("kernel", ctypes.c_int),
                ("chains_in_flight", ctypes.c_int), ("nontemporal", ctypes.c_int),
                ("combine", ctypes.c_int), ("split_permille", ctypes.c_int)]


class MfrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = mfr_strerror(status)
        if status == MFR_ERR_HIP:
            detail += " (%s)" % mfr_last_hip_error()
        super().__init__("%s: %s" % (where, detail))


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libmfreduce.so is not built: run `python -m paper_2001_05585_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    L.mfr_sum_f16.argtypes = [vp, sz, vp, vp]
    L.mfr_sum_f16.restype = ci
    L.mfr_sum_f16_tuned.argtypes = [vp, sz, vp, ci, ci, ci, ci, vp]
    L.mfr_sum_f16_tuned.restype = ci
    L.mfr_sum_f16_ex.argtypes = [vp, sz, vp, ctypes.POINTER(mfr_tuning), vp]
    L.mfr_sum_f16_ex.restype = ci
    L.mfr_sum_f16_noalloc.argtypes = [vp, sz, vp, ctypes.POINTER(mfr_tuning), vp]
    L.mfr_sum_f16_noalloc.restype = ci
    L.mfr_sum_f16_stamped.argtypes = [vp, sz, vp, ctypes.POINTER(mfr_tuning), vp, sz, vp]
    L.mfr_sum_f16_stamped.restype = ci
    L.mfr_wall_clock_khz.argtypes = [ctypes.POINTER(ci)]
    L.mfr_wall_clock_khz.restype = ci
    L.mfr_sum_bf16.argtypes = [vp, sz, vp, vp]
    L.mfr_sum_bf16.restype = ci
    L.mfr_sum_f32.argtypes = [vp, sz, vp, vp]
    L.mfr_sum_f32.restype = ci
    L.mfr_sum_ex.argtypes = [vp, ci, sz, vp, ctypes.POINTER(mfr_tuning), vp]
    L.mfr_sum_ex.restype = ci
    L.mfr_sum_rows_ex.argtypes = [vp, ci, sz, sz, sz, vp, ctypes.POINTER(mfr_tuning), vp]
    L.mfr_sum_rows_ex.restype = ci
    L.mfr_sum_f16_rows.argtypes = [vp, sz, sz, sz, vp, vp]
    L.mfr_sum_f16_rows.restype = ci
    L.mfr_sum_f16_f64.argtypes = [vp, sz, vp, vp]
    L.mfr_sum_f16_f64.restype = ci
    L.mfr_sum_f16_f64_ex.argtypes = [vp, sz, vp, ctypes.POINTER(mfr_tuning), vp]
    L.mfr_sum_f16_f64_ex.restype = ci
    L.mfr_sum_f16_recurrence.argtypes = [vp, sz, vp, ci, vp]
    L.mfr_sum_f16_recurrence.restype = ci
    L.mfr_plan_ex.argtypes = [sz, sz, ci, ctypes.POINTER(mfr_tuning), ctypes.POINTER(ctypes.c_ulonglong)]
    L.mfr_plan_ex.restype = ci
    L.mfr_rows_plan.argtypes = [sz, ci, sz, sz, sz, ci, ctypes.POINTER(ctypes.c_ulonglong)]
    L.mfr_rows_plan.restype = ci
    L.mfr_rows_geometry.argtypes = [sz, ci, sz, sz, sz, ctypes.POINTER(mfr_tuning), ci, ctypes.POINTER(ctypes.c_ulonglong)]
    L.mfr_rows_geometry.restype = ci
    ip = ctypes.POINTER(ci)
    L.mfr_get_default_tuning.argtypes = [ip, ip, ip]
    L.mfr_get_default_tuning.restype = ci
    L.mfr_grid_for.argtypes = [sz, sz, ctypes.POINTER(mfr_tuning)]
    L.mfr_grid_for.restype = ctypes.c_longlong
    L.mfr_plan_for.argtypes = [sz, sz, ctypes.POINTER(mfr_tuning), ctypes.POINTER(ctypes.c_ulonglong)]
    L.mfr_plan_for.restype = ci
    L.mfr_release_scratch.argtypes = [ctypes.c_void_p]
    L.mfr_release_scratch.restype = ci
    L.mfr_strerror.argtypes = [ci]
    L.mfr_strerror.restype = ctypes.c_char_p
    L.mfr_last_hip_error.argtypes = []
    L.mfr_last_hip_error.restype = ctypes.c_char_p
    L.mfr_version.argtypes = []
    L.mfr_version.restype = ci
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != MFR_OK:
        raise MfrError(status, where)


def mfr_sum_f16(x: int, n: int, out: int, stream: int = 0) -> None:
    """x, out: device addresses; stream: hipStream_t handle (0 = null stream)."""
    _check(lib().mfr_sum_f16(x, n, out, stream), "mfr_sum_f16")


def mfr_sum_f16_tuned(x: int, n: int, out: int, block_threads: int, chain_R: int,
                      grid_blocks: int = MFR_GRID_AUTO, kernel: int = MFR_KERNEL_MFMA,
                      stream: int = 0) -> None:
    _check(lib().mfr_sum_f16_tuned(x, n, out, block_threads, chain_R, grid_blocks, kernel, stream),
           "mfr_sum_f16_tuned")


def make_tuning(block_threads=0, chain_R=0, grid_blocks=0, kernel=0, chains_in_flight=0,
                nontemporal=0, combine=0, split_permille=0) -> mfr_tuning:
    return mfr_tuning(block_threads, chain_R, grid_blocks, kernel, chains_in_flight, nontemporal, combine,
                      split_permille)


def mfr_sum_f16_ex(x: int, n: int, out: int, t: mfr_tuning | None = None, stream: int = 0) -> None:
    tp = ctypes.byref(t) if t is not None else None
    _check(lib().mfr_sum_f16_ex(x, n, out, tp, stream), "mfr_sum_f16_ex")


def mfr_sum_f16_noalloc(x: int, n: int, out: int, t: mfr_tuning | None = None, stream: int = 0) -> None:
    tp = ctypes.byref(t) if t is not None else None
    _check(lib().mfr_sum_f16_noalloc(x, n, out, tp, stream), "mfr_sum_f16_noalloc")


def mfr_sum_f16_stamped(x: int, n: int, out: int, t: mfr_tuning | None, stamps: int, stamps_len: int, stream: int = 0) -> None:
    tp = ctypes.byref(t) if t is not None else None
    _check(lib().mfr_sum_f16_stamped(x, n, out, tp, stamps, stamps_len, stream), "mfr_sum_f16_stamped")


def mfr_wall_clock_khz() -> int:
    khz = ctypes.c_int()
    _check(lib().mfr_wall_clock_khz(ctypes.byref(khz)), "mfr_wall_clock_khz")
    return khz.value


def mfr_sum_bf16(x: int, n: int, out: int, stream: int = 0) -> None:
    _check(lib().mfr_sum_bf16(x, n, out, stream), "mfr_sum_bf16")


def mfr_sum_f32(x: int, n: int, out: int, stream: int = 0) -> None:
    _check(lib().mfr_sum_f32(x, n, out, stream), "mfr_sum_f32")


def mfr_sum_ex(x: int, dtype: int, n: int, out: int, t: mfr_tuning | None = None, stream: int = 0) -> None:
    tp = ctypes.byref(t) if t is not None else None
    _check(lib().mfr_sum_ex(x, dtype, n, out, tp, stream), "mfr_sum_ex")


def mfr_sum_rows_ex(x: int, dtype: int, rows: int, cols: int, row_stride: int, out: int,
                    t: mfr_tuning | None = None, stream: int = 0) -> None:
    tp = ctypes.byref(t) if t is not None else None
    _check(lib().mfr_sum_rows_ex(x, dtype, rows, cols, row_stride, out, tp, stream), "mfr_sum_rows_ex")


def mfr_sum_f16_rows(x: int, rows: int, cols: int, row_stride: int, out: int, stream: int = 0) -> None:
    _check(lib().mfr_sum_f16_rows(x, rows, cols, row_stride, out, stream), "mfr_sum_f16_rows")


def mfr_sum_f16_f64(x: int, n: int, out: int, stream: int = 0) -> None:
    _check(lib().mfr_sum_f16_f64(x, n, out, stream), "mfr_sum_f16_f64")


def mfr_sum_f16_f64_ex(x: int, n: int, out: int, t: mfr_tuning | None = None, stream: int = 0) -> None:
    tp = ctypes.byref(t) if t is not None else None
    _check(lib().mfr_sum_f16_f64_ex(x, n, out, tp, stream), "mfr_sum_f16_f64_ex")


def mfr_sum_f16_recurrence(x: int, n: int, out: int, chain_R: int, stream: int = 0) -> None:
    _check(lib().mfr_sum_f16_recurrence(x, n, out, chain_R, stream), "mfr_sum_f16_recurrence")


def mfr_plan_ex(n: int, x_addr: int, dtype: int, t: mfr_tuning | None = None):
    plan = (ctypes.c_ulonglong * 7)()
    tp = ctypes.byref(t) if t is not None else None
    _check(lib().mfr_plan_ex(n, x_addr, dtype, tp, plan), "mfr_plan_ex")
    return tuple(int(v) for v in plan)


def mfr_rows_plan(x_addr: int, dtype: int, rows: int, cols: int, row_stride: int, cus: int = 256):
    """None if the per-row kernels are chosen, else the 12 plan values of the many-rows kernel."""
    plan = (ctypes.c_ulonglong * 12)()
    st = int(lib().mfr_rows_plan(x_addr, dtype, rows, cols, row_stride, cus, plan))
    if st < 0:
        _check(-st, "mfr_rows_plan")
    return tuple(int(v) for v in plan) if st == 1 else None


def mfr_rows_geometry(x_addr: int, dtype: int, rows: int, cols: int, row_stride: int, t: mfr_tuning | None = None,
                      cus: int = 256):
    """None if the many-rows kernel is chosen, else the 8 geometry values of the per-row kernels."""
    plan = (ctypes.c_ulonglong * 8)()
    tp = ctypes.byref(t) if t is not None else None
    st = int(lib().mfr_rows_geometry(x_addr, dtype, rows, cols, row_stride, tp, cus, plan))
    if st < 0:
        _check(-st, "mfr_rows_geometry")
    return tuple(int(v) for v in plan) if st == 1 else None


def mfr_get_default_tuning():
    b, r, g = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().mfr_get_default_tuning(ctypes.byref(b), ctypes.byref(r), ctypes.byref(g)),
           "mfr_get_default_tuning")
    return b.value, r.value, g.value


def mfr_grid_for(n: int, x_addr: int, t: mfr_tuning | None = None) -> int:
    tp = ctypes.byref(t) if t is not None else None
    return int(lib().mfr_grid_for(n, x_addr, tp))


def mfr_plan_for(n: int, x_addr: int, t: mfr_tuning | None = None):
    """(head, slots, main0, chains, tile_slots, epi0, epi1)."""
    plan = (ctypes.c_ulonglong * 7)()
    tp = ctypes.byref(t) if t is not None else None
    _check(lib().mfr_plan_for(n, x_addr, tp, plan), "mfr_plan_for")
    return tuple(int(v) for v in plan)


def mfr_release_scratch(stream: int = 0) -> None:
    _check(lib().mfr_release_scratch(stream), "mfr_release_scratch")


def mfr_strerror(status: int) -> str:
    return lib().mfr_strerror(status).decode()


def mfr_last_hip_error() -> str:
    return lib().mfr_last_hip_error().decode()


def mfr_version() -> int:
    return int(lib().mfr_version())

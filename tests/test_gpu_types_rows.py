"""GPU parity for the other element types (bfloat16, binary32) and the batched
(rows) form, against the CPU oracle.  Bit-exact on integer-valued inputs whose
every partial sum is exact in fp32; |gpu - oracle| <= 1e-5 * sum |x_i| otherwise."""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2001_05585_amd import binding as B            # noqa: E402
from paper_2001_05585_amd import workloads as W          # noqa: E402
from gpu_util import Outputs, stream_handle              # noqa: E402

TOL = 1e-5
KERNELS = (B.MFR_KERNEL_MFMA, B.MFR_KERNEL_SHFL)
NAN16, NAN32 = 0x7FC0, 0x7FC00000


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; the HIP path has no fallback")
    B.lib()


class TypedInput:
    """Raw element bits on the GPU with NaN poison around them and an element shift."""

    def __init__(self, bits: np.ndarray, shift: int = 0):
        assert bits.dtype in (np.uint16, np.uint32)
        self.esize = bits.dtype.itemsize
        guard = 64
        poison = NAN16 if self.esize == 2 else NAN32
        buf = np.full(bits.size + 2 * guard + 8, poison, dtype=bits.dtype)
        self.start = guard + shift
        buf[self.start:self.start + bits.size] = bits
        self.tensor = torch.from_numpy(buf.view(np.int16 if self.esize == 2 else np.int32)).cuda()
        assert self.tensor.data_ptr() % 16 == 0
        self.ptr = self.tensor.data_ptr() + self.esize * self.start
        self.n = bits.size


def run(dtype, d, n, tunings):
    o = Outputs(len(tunings))
    for i, t in enumerate(tunings):
        B.mfr_sum_ex(d.ptr, dtype, n, o.ptr(i), t, stream_handle())
    return o.get()


def tunings_for_types():
    out = [None]
    for kernel in KERNELS:
        for block, R, grid in ((64, 1, 0), (256, 4, 0), (1024, 8, 0), (128, 3, 5), (256, 2, -1), (512, 5, 700)):
            out.append(B.make_tuning(block, R, grid, kernel))
    return out


def int_bits(dtype, n, seed):
    v = W.small_integers(n, seed).astype(np.float32)
    return (W.to_bf16_bits(v) if dtype == B.MFR_DTYPE_BF16 else v.view(np.uint32)), v.astype(np.float64)


@pytest.mark.parametrize("dtype", [B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32])
def test_every_small_n_bit_exact(dtype):
    per_slot = 8 if dtype == B.MFR_DTYPE_BF16 else 4
    bits, vals = int_bits(dtype, 2100, seed=61)
    want = np.concatenate([[0.0], np.cumsum(vals)])
    for shift in (0, 1, per_slot - 1):
        d = TypedInput(bits, shift)
        ts = [B.make_tuning(256, 1), B.make_tuning(64, 4, 2, B.MFR_KERNEL_SHFL), B.make_tuning(128, 2, 3)]
        o = Outputs(2101 * len(ts))
        for n in range(2101):
            for j, t in enumerate(ts):
                B.mfr_sum_ex(d.ptr, dtype, n, o.ptr(n * len(ts) + j), t, stream_handle())
        r = o.get().reshape(2101, len(ts))
        for j in range(len(ts)):
            wrong = np.nonzero(r[:, j] != want)[0]
            assert wrong.size == 0, (dtype, shift, j, wrong[:5], r[wrong[:5], j], want[wrong[:5]])


@pytest.mark.parametrize("dtype", [B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32])
def test_one_hot_every_position(dtype):
    per_tile = 512 if dtype == B.MFR_DTYPE_BF16 else 256
    t = B.make_tuning(64, 2, 2, B.MFR_KERNEL_MFMA, 1)
    n = 3 * (2 * 2 * per_tile) + 2 * per_tile + 5
    zero = np.zeros(n, dtype=np.uint16 if dtype == B.MFR_DTYPE_BF16 else np.uint32)
    one = 0x3F80 if dtype == B.MFR_DTYPE_BF16 else 0x3F800000
    d = TypedInput(zero, 3)
    o = Outputs(n)
    for p in range(n):
        d.tensor[d.start + p] = one
        B.mfr_sum_ex(d.ptr, dtype, n, o.ptr(p), t, stream_handle())
        d.tensor[d.start + p] = 0
    r = o.get()
    wrong = np.nonzero(r != 1.0)[0]
    assert wrong.size == 0, (dtype, wrong[:8], r[wrong[:8]])


@pytest.mark.parametrize("dtype", [B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32])
def test_integer_inputs_same_bits_in_every_geometry(dtype, oracle_lib):
    n = (1 << 18) + 5
    bits, vals = int_bits(dtype, n, seed=71)
    want = float(vals.sum())
    osum = oracle_lib.sum_bf16(bits)[0] if dtype == B.MFR_DTYPE_BF16 else oracle_lib.sum_f32(bits)[0]
    assert osum == want
    for shift in (0, 1, 3):
        d = TypedInput(bits, shift)
        r = run(dtype, d, n, tunings_for_types())
        assert np.all(r == want), (dtype, shift, r, want)


@pytest.mark.parametrize("dtype", [B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32])
@pytest.mark.parametrize("kind,n", [("uniform01", (1 << 22) + 7), ("normal", (1 << 22) + 7), ("uniform_pm1", 4_000_007),
                                    ("normal", 1000)])
def test_random_inputs_within_tolerance(dtype, kind, n, oracle_lib):
    if dtype == B.MFR_DTYPE_BF16:
        bits = W.generate_bf16(kind, n, 500 + n % 97)
        s, sa = oracle_lib.sum_bf16(bits)
    else:
        bits = W.generate_f32(kind, n, 500 + n % 97).view(np.uint32)
        s, sa = oracle_lib.sum_f32(bits)
    d = TypedInput(bits, 1)
    r = run(dtype, d, n, tunings_for_types()).astype(np.float64)
    err = np.abs(r - s) / sa
    assert err.max() <= TOL, (dtype, kind, n, err.max())


def test_typed_convenience_entries(oracle_lib):
    n = (1 << 20) + 3
    b = W.generate_bf16("uniform01", n, 9)
    f = W.generate_f32("normal", n, 9)
    db, df = TypedInput(b), TypedInput(f.view(np.uint32))
    o = Outputs(2)
    B.mfr_sum_bf16(db.ptr, n, o.ptr(0), stream_handle())
    B.mfr_sum_f32(df.ptr, n, o.ptr(1), stream_handle())
    r = o.get().astype(np.float64)
    sb, sab = oracle_lib.sum_bf16(b)
    sf, saf = oracle_lib.sum_f32(f)
    assert abs(r[0] - sb) <= TOL * sab and abs(r[1] - sf) <= TOL * saf


@pytest.mark.parametrize("dtype", [B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32])
def test_special_values(dtype):
    n = 100000
    one, pinf, ninf, nan = ((0x3F80, 0x7F80, 0xFF80, 0x7FC1) if dtype == B.MFR_DTYPE_BF16
                            else (0x3F800000, 0x7F800000, 0xFF800000, 0x7FC00001))
    base = np.full(n, one, dtype=np.uint16 if dtype == B.MFR_DTYPE_BF16 else np.uint32)
    for kernel in KERNELS:
        t = B.make_tuning(256, 2, 0, kernel)
        x = base.copy(); x[70001] = pinf
        assert float(run(dtype, TypedInput(x), n, [t])[0]) == math.inf
        x[5] = ninf
        assert math.isnan(float(run(dtype, TypedInput(x), n, [t])[0]))
        x = base.copy(); x[n - 1] = nan
        assert math.isnan(float(run(dtype, TypedInput(x), n, [t])[0]))


# ------------------------------------------------------------------ rows ---

def rows_call(dev_ptr, dtype, rows, cols, stride, tuning=None):
    o = Outputs(max(rows, 1) + 1)
    B.mfr_sum_rows_ex(dev_ptr, dtype, rows, cols, stride, o.ptr(0), tuning, stream_handle())
    r = o.get()
    assert r[rows] == Outputs.SENTINEL            # nothing written past out[rows)
    return r[:rows]


@pytest.mark.parametrize("rows,cols,stride", [(1, 5000, 5000), (7, 4096, 4096), (33, 1000, 1000), (64, 777, 784),
                                              (5, 100003, 100008), (300, 512, 512), (3, 1, 8), (1000, 37, 40),
                                              (9, 2049, 2051), (4, 65536 + 7, 65536 + 7),
                                              (150, 30011, 30016), (300, 9001, 9008), (31, 40000, 40000)])
def test_rows_integer_inputs_bit_exact(rows, cols, stride, oracle_lib):
    flat = W.small_integers(rows * stride + 16, seed=rows * 1000 + cols)
    for shift in (0, 3):
        d = TypedInput(flat.view(np.uint16), shift)
        x2d = np.stack([flat[r * stride:r * stride + cols] for r in range(rows)])
        want, _ = oracle_lib.sum_rows(x2d)
        for t in (None, B.make_tuning(64, 2, 0, B.MFR_KERNEL_SHFL), B.make_tuning(256, 1, 3), B.make_tuning(128, 4, 2, 0, 0, 0, 2)):
            got = rows_call(d.ptr, B.MFR_DTYPE_F16, rows, cols, stride, t)
            assert np.array_equal(got.astype(np.float64), want), (rows, cols, stride, shift, got[:4], want[:4])


@pytest.mark.parametrize("cols", [5, 37, 512, 1000, 3000, 4095])
def test_many_short_rows_with_padded_stride(cols, oracle_lib):
    # library defaults + many short rows: the many-rows kernel, rows 16-byte aligned or shifted by 3 elements
    rows = 2051
    stride = (cols + 7) // 8 * 8 + 8
    flat = W.small_integers(rows * stride + 16, seed=cols)
    x2d = np.stack([flat[r * stride:r * stride + cols] for r in range(rows)])
    want, _ = oracle_lib.sum_rows(x2d)
    for shift in (0, 3):
        d = TypedInput(flat.view(np.uint16), shift)
        got = rows_call(d.ptr, B.MFR_DTYPE_F16, rows, cols, stride)
        assert np.array_equal(got.astype(np.float64), want), (cols, shift, got[:4], want[:4])
    f = W.generate_f32("normal", rows * stride, 1234 + cols)
    s, sa = oracle_lib.sum_rows(f.reshape(rows, stride)[:, :cols], "f32")
    df = TypedInput(f.view(np.uint32), 0)          # keep the device buffer alive across the call
    got = rows_call(df.ptr, B.MFR_DTYPE_F32, rows, cols, stride).astype(np.float64)
    assert (np.abs(got - s) <= TOL * sa).all()


@pytest.mark.parametrize("cols", [1, 5, 31, 32, 33, 37, 64, 65, 100, 128, 129, 256, 700, 767])
def test_many_short_rows_library_default(cols, oracle_lib):
    # library defaults, >= 4096 rows of a 16-bit type: the accumulator columns of a chain shared out among rows
    rows = 5003
    stride = (cols + 7) // 8 * 8 + (8 if cols % 16 else 0)
    flat = W.small_integers(rows * stride + 16, seed=cols + 1)
    x2d = np.stack([flat[r * stride:r * stride + cols] for r in range(rows)])
    want, _ = oracle_lib.sum_rows(x2d)
    d = TypedInput(flat.view(np.uint16), 0)
    got = rows_call(d.ptr, B.MFR_DTYPE_F16, rows, cols, stride)
    assert np.array_equal(got.astype(np.float64), want), (cols, np.nonzero(got != want)[0][:5])
    # bfloat16, random values
    f = W.generate_f32("normal", rows * stride, 99 + cols)
    b = W.to_bf16_bits(f)
    s, sa = oracle_lib.sum_rows(b.reshape(rows, stride)[:, :cols], "bf16")
    db = TypedInput(b, 0)                          # keep the device buffer alive across the call
    got = rows_call(db.ptr, B.MFR_DTYPE_BF16, rows, cols, stride).astype(np.float64)
    assert (np.abs(got - s) <= TOL * sa + 1e-30).all()
    # special values stay in their own row
    y = flat.view(np.uint16).copy()
    y[7 * stride + cols - 1] = 0x7C00
    y[4000 * stride] = 0x7E00
    dy = TypedInput(y, 0)
    got = rows_call(dy.ptr, B.MFR_DTYPE_F16, rows, cols, stride).astype(np.float64)
    assert got[7] == math.inf and math.isnan(got[4000])
    keep = np.ones(rows, dtype=bool); keep[[7, 4000]] = False
    assert np.array_equal(got[keep], want[keep])


def test_rows_random_inputs_and_types(oracle_lib):
    rows, cols = 48, 50000
    stride = cols + 8
    x = W.generate("normal", rows * stride, 77)
    d = TypedInput(x.view(np.uint16), 0)
    x2d = x.reshape(rows, stride)[:, :cols]
    s, sa = oracle_lib.sum_rows(x2d)
    got = rows_call(d.ptr, B.MFR_DTYPE_F16, rows, cols, stride).astype(np.float64)
    assert (np.abs(got - s) / sa).max() <= TOL
    # each row equals what a single call computes for that row, bit for bit, when the geometry is the same
    t = B.make_tuning(256, 4, 6)
    got = rows_call(d.ptr, B.MFR_DTYPE_F16, rows, cols, stride, t)
    o = Outputs(rows)
    for r in range(rows):
        B.mfr_sum_f16_ex(d.ptr + 2 * r * stride, cols, o.ptr(r), t, stream_handle())
    assert np.array_equal(got.view(np.uint32), o.get().view(np.uint32))
    f = W.generate_f32("uniform_pm1", rows * stride, 78)
    df = TypedInput(f.view(np.uint32), 0)
    s, sa = oracle_lib.sum_rows(f.reshape(rows, stride)[:, :cols], "f32")
    got = rows_call(df.ptr, B.MFR_DTYPE_F32, rows, cols, stride).astype(np.float64)
    assert (np.abs(got - s) / sa).max() <= TOL


def test_rows_degenerate_and_many_rows(oracle_lib):
    d = TypedInput(W.ones(70000 * 8).view(np.uint16))
    assert rows_call(d.ptr, B.MFR_DTYPE_F16, 0, 10, 10).size == 0
    assert np.all(rows_call(d.ptr, B.MFR_DTYPE_F16, 5, 0, 8) == 0.0)
    got = rows_call(d.ptr, B.MFR_DTYPE_F16, 70000, 8, 8)          # more rows than one launch holds
    assert np.all(got == 8.0)
    o = Outputs(4)
    B.mfr_sum_f16_rows(d.ptr, 3, 1000, 1024, o.ptr(0), stream_handle())
    r = o.get()
    assert np.all(r[:3] == 1000.0) and r[3] == Outputs.SENTINEL

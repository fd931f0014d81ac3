"""GPU parity at the full sizes of the five configurations, in the launch
configuration bench.py times (default tuning) and in the swept geometries.

Acceptance: |gpu - oracle| <= 1e-5 * sum |x_i| (oracle = fp64 Kahan sum; for
n >= 2^26 the same oracle over host threads, which the CPU tests pin to the
exact integer sum)."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2001_05585_amd import binding as B            # noqa: E402
from paper_2001_05585_amd import workloads as W          # noqa: E402
from gpu_util import Outputs, stream_handle              # noqa: E402
from test_golden import golden_rows                      # noqa: E402

TOL = 1e-5
THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; the HIP path has no fallback")
    B.lib()


def golden(cfg, n):
    for c, _, m, s, sa in golden_rows():
        if c == cfg and m == n:
            return s, sa
    return None


def oracle_of(oracle_lib, x):
    if x.size <= 1 << 24:
        return oracle_lib.sum_f16(x)
    s, sa, _ = oracle_lib.sum_f16_blocked(x, THREADS)
    return s, sa


def upload(x):
    t = torch.from_numpy(x.view(np.int16)).cuda()
    assert t.data_ptr() % 16 == 0
    return t


def run_all(dev, n, tunings, offset_elems=0):
    o = Outputs(len(tunings))
    for i, t in enumerate(tunings):
        B.mfr_sum_f16_ex(dev.data_ptr() + 2 * offset_elems, n, o.ptr(i), t, stream_handle())
    return o.get().astype(np.float64)


def test_config2_every_block_R_cell_at_2p26(oracle_lib):
    n = 1 << 26
    x = W.generate("uniform01", n, W.config_seed(2))
    s, sa = oracle_of(oracle_lib, x)
    assert (s, sa) == golden(2, n) or abs(s - golden(2, n)[0]) <= 1e-9 * sa
    dev = upload(x)
    tunings = [B.make_tuning(block, R, grid) for block in (32, 64, 128, 256, 512, 1024)
               for R in range(1, 9) for grid in (B.MFR_GRID_AUTO, B.MFR_GRID_ONE_CHAIN)]
    r = run_all(dev, n, tunings)
    err = np.abs(r - s) / sa
    print("config 2: max |err|/sum|x| over %d cells = %.3g" % (len(tunings), err.max()))
    assert err.max() <= TOL


def test_config3_normal_2p28_headline(oracle_lib):
    n = 1 << 28
    x = W.generate("normal", n, W.config_seed(3))
    s, sa = oracle_of(oracle_lib, x)
    gs, gsa = golden(3, n)
    assert abs(s - gs) <= 1e-12 * sa and abs(sa - gsa) <= 1e-12 * sa
    dev = upload(x)
    tunings = [None, B.make_tuning(kernel=B.MFR_KERNEL_SHFL), B.make_tuning(128, 4, B.MFR_GRID_ONE_CHAIN),
               B.make_tuning(256, 1), B.make_tuning(1024, 8, 4096)]
    # the split variant of Section 5.3 at the fractions `bench.py --sweep split` times
    tunings += [B.make_tuning(256, 4, 0, B.MFR_KERNEL_SPLIT, 2, 0, 0, f) for f in (0, 100, 500, 900, 1000)]
    r = run_all(dev, n, tunings)
    err = np.abs(r - s)
    print("config 3: gpu=%.6f oracle=%.6f |err|/sum|x|=%.3g |err|/|sum|=%.3g" % (r[0], s, err[0] / sa, err[0] / abs(s)))
    assert (err / sa).max() <= TOL
    # misaligned view of the same buffer (a slice starting at element 1)
    s1, sa1 = oracle_of(oracle_lib, x[1:])
    r1 = run_all(dev, n - 1, [None, B.make_tuning(kernel=B.MFR_KERNEL_SHFL)], offset_elems=1)
    assert (np.abs(r1 - s1) / sa1).max() <= TOL


def test_rows_at_the_sweep_sizes_sampled_rows(oracle_lib):
    """The batched entry on 512 MiB of rows, library defaults (the shapes `bench.py --sweep rows` times):
    sampled rows against the oracle, one by one."""
    total = 1 << 28
    x = W.generate("normal", total, W.config_seed(3))
    dev = upload(x)
    rng = np.random.default_rng(31)
    out = torch.empty((1 << 23) + 1, dtype=torch.float32, device="cuda")
    shapes = [(32, 32, 0), (64, 64, 0), (256, 256, 1), (1024, 1024, 0), (1001, 1001, 0), (2304, 2304, 0), (4096, 4096, 0),
              (4096, 4096, 1), (5001, 5001, 0), (8192, 8192, 0), (100, 104, 0), (50000, 50001, 0), (16777209, 16777209, 0),
              (1 << 27, 1 << 27, 0)]
    for cols, stride, shift in shapes:
        rows = (total - shift - cols) // stride + 1
        out.fill_(float("nan"))
        B.mfr_sum_rows_ex(dev.data_ptr() + 2 * shift, B.MFR_DTYPE_F16, rows, cols, stride, out.data_ptr(), None, stream_handle())
        torch.cuda.synchronize()
        got = out[:rows].cpu().numpy().astype(np.float64)
        assert not np.isnan(got).any(), (cols, stride, shift)
        assert bool(torch.isnan(out[rows]).item())                       # nothing written past the rows
        pick = np.unique(np.concatenate([[0, 1, rows - 2, rows - 1], rng.integers(0, rows, 60)]))
        pick = pick[(pick >= 0) & (pick < rows)]
        for r in pick:
            seg = x[shift + r * stride: shift + r * stride + cols]
            s, sa = oracle_of(oracle_lib, seg)
            assert abs(got[r] - s) <= TOL * sa, (cols, stride, shift, int(r), got[r], s)
        # all rows together: the row sums add up to the sum of the elements they cover
        if stride == cols:
            s, sa = oracle_of(oracle_lib, x[shift: shift + rows * cols])
            assert abs(got.sum() - s) <= TOL * sa, (cols, stride, shift)


@pytest.mark.parametrize("dtype,kind,n", [(B.MFR_DTYPE_BF16, "normal", 1 << 28), (B.MFR_DTYPE_F32, "uniform_pm1", (1 << 27) + 3)])
def test_other_element_types_at_512MiB(oracle_lib, dtype, kind, n):
    """bfloat16 and binary32 input at the size `bench.py --sweep types` times, library defaults and the
    conventional kernel, against the oracle of the same type."""
    if dtype == B.MFR_DTYPE_BF16:
        x = W.generate_bf16(kind, n, W.config_seed(3))
        s, sa = oracle_lib.sum_bf16(x)
        dev, esize = torch.from_numpy(x.view(np.int16)).cuda(), 2
    else:
        x = W.generate_f32(kind, n, W.config_seed(4))
        s, sa = oracle_lib.sum_f32(x)
        dev, esize = torch.from_numpy(x).cuda(), 4
    tunings = [None, B.make_tuning(kernel=B.MFR_KERNEL_SHFL), B.make_tuning(512, 2, 1000)]
    o = Outputs(2 * len(tunings))
    for i, t in enumerate(tunings):
        B.mfr_sum_ex(dev.data_ptr(), dtype, n, o.ptr(2 * i), t, stream_handle())
        B.mfr_sum_ex(dev.data_ptr() + esize, dtype, n - 1, o.ptr(2 * i + 1), t, stream_handle())     # a slice from element 1
    r = o.get().astype(np.float64)
    first = float(oracle_lib.bf16_to_f64(int(x[0]))) if dtype == B.MFR_DTYPE_BF16 else float(x[0])
    assert (np.abs(r[0::2] - s) / sa).max() <= TOL, (r, s)
    assert (np.abs(r[1::2] - (s - first)) / sa).max() <= TOL + 1e-12, (r, s, first)


@pytest.mark.parametrize("n", [400_000_000, 400_000_007])
def test_config4_uniform_pm1_400M(oracle_lib, n):
    x = W.generate("uniform_pm1", n, W.config_seed(4))
    s, sa = oracle_of(oracle_lib, x)
    gs, gsa = golden(4, n)
    assert abs(s - gs) <= 1e-12 * sa and abs(sa - gsa) <= 1e-12 * sa
    dev = upload(x)
    r = run_all(dev, n, [None, B.make_tuning(kernel=B.MFR_KERNEL_SHFL), B.make_tuning(64, 2, 3000)])
    err = np.abs(r - s) / sa
    print("config 4 (n=%d): max |err|/sum|x| = %.3g" % (n, err.max()))
    assert err.max() <= TOL


def test_config5_size_sweep_up_to_2p30(oracle_lib):
    nmax = (1 << 30) + 7
    x = W.generate("uniform01", nmax, W.config_seed(5))
    dev = upload(x)
    sizes = [m for k in range(16, 31) for m in (1 << k, (1 << k) + 7)]
    tunings = [None, B.make_tuning(kernel=B.MFR_KERNEL_SHFL)]
    worst = 0.0
    for n in sizes:
        s, sa = oracle_of(oracle_lib, x[:n])
        g = golden(5, n)
        if g is not None:
            assert abs(s - g[0]) <= 1e-12 * sa
        r = run_all(dev, n, tunings)
        err = (np.abs(r - s) / sa).max()
        worst = max(worst, err)
        assert err <= TOL, (n, r, s)
        assert np.all(np.isfinite(r))
    print("config 5: worst |err|/sum|x| over %d sizes x 2 kernels = %.3g" % (len(sizes), worst))


def test_more_than_2p32_elements(oracle_lib):
    """64-bit sizes: n = 2^32 + 2^20 + 7 all-ones (8 GiB on the device, filled there).  The binary64
    mode must return n exactly; the fp32 modes must be within tolerance of n; a one-hot near the
    end must be found."""
    n = (1 << 32) + (1 << 20) + 7
    free, _ = torch.cuda.mem_get_info()
    if free < 2 * n + (1 << 30):
        pytest.skip("not enough device memory for an 8 GiB input")
    x = torch.ones(n + 8, dtype=torch.float16, device="cuda")
    ptr = x.data_ptr() + 2            # misaligned start
    o = Outputs(3)
    o64 = torch.zeros(1, dtype=torch.float64, device="cuda")
    B.mfr_sum_f16(ptr, n, o.ptr(0), stream_handle())
    B.mfr_sum_f16_ex(ptr, n, o.ptr(1), B.make_tuning(kernel=B.MFR_KERNEL_SHFL), stream_handle())
    B.mfr_sum_f16_ex(ptr, n, o.ptr(2), B.make_tuning(512, 2, 5000), stream_handle())
    B.mfr_sum_f16_f64(ptr, n, o64.data_ptr(), stream_handle())
    r = o.get().astype(np.float64)
    assert float(o64[0]) == float(n)
    assert np.all(np.abs(r - n) <= TOL * n), r
    x.zero_()
    x[n - 3] = 1.0                    # element n - 4 of the call's range
    B.mfr_sum_f16(ptr, n, o.ptr(0), stream_handle())
    B.mfr_sum_f16(ptr, n - 4, o.ptr(1), stream_handle())
    r = o.get()
    assert r[0] == 1.0 and r[1] == 0.0

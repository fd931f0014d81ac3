"""Seeded random sweep of sizes, alignments, geometries, kernels, element types and entry points on
integer-valued inputs, where every summation order is exact: the GPU must return the exact sum."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2001_05585_amd import binding as B            # noqa: E402
from paper_2001_05585_amd import workloads as W          # noqa: E402
from gpu_util import Outputs, stream_handle              # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; the HIP path has no fallback")
    B.lib()


def random_tuning(rng, dtype):
    kernel = int(rng.choice([0, 1, 2] if dtype == B.MFR_DTYPE_F16 else [0, 1]))
    blocks = [64, 128, 256, 512, 1024] + ([32] if dtype == B.MFR_DTYPE_F16 and kernel != 2 else [])
    R = int(rng.integers(1, 9))
    us = [u for u in (1, 2, 3, 4, 6, 8) if u * R <= 16]
    grid = int(rng.choice([0, -1, 1, 2, 3, 17, 100, 513, 3000]))
    return B.make_tuning(int(rng.choice(blocks)), R, grid, kernel, int(rng.choice(us)), int(rng.integers(0, 3)),
                         int(rng.integers(0, 3)), int(rng.integers(0, 1001)) if kernel == 2 else 0)


def test_random_geometries_on_exact_inputs():
    """Expected values come from numpy's binary64 prefix sums of small integers: every partial sum is an
    integer below 2^24, exact in binary64 and binary32 alike, so it is the number the oracle returns too."""
    rng = np.random.default_rng(20010558)
    pool = W.small_integers((1 << 21) + 64, seed=12, lo=-6, hi=6)
    pool64 = pool.astype(np.float64)
    csum = np.concatenate([[0.0], np.cumsum(pool64)])
    dev = {
        B.MFR_DTYPE_F16: torch.from_numpy(pool.view(np.int16)).cuda(),
        B.MFR_DTYPE_BF16: torch.from_numpy(W.to_bf16_bits(pool.astype(np.float32)).view(np.int16)).cuda(),
        B.MFR_DTYPE_F32: torch.from_numpy(pool.astype(np.float32)).cuda(),
    }
    cases = []
    for _ in range(600):
        dtype = int(rng.choice([0, 0, 1, 2]))
        n = int(rng.choice([rng.integers(0, 70), rng.integers(0, 5000), rng.integers(0, 1 << 21)]))
        start = int(rng.integers(0, 64))
        cases.append((dtype, n, start, random_tuning(rng, dtype)))
    o = Outputs(len(cases))
    for i, (dtype, n, start, t) in enumerate(cases):
        esize = 4 if dtype == B.MFR_DTYPE_F32 else 2
        B.mfr_sum_ex(dev[dtype].data_ptr() + esize * start, dtype, n, o.ptr(i), t, stream_handle())
    r = o.get().astype(np.float64)
    want = np.array([csum[start + n] - csum[start] for (_, n, start, _) in cases])
    bad = np.nonzero(r != want)[0]
    assert bad.size == 0, [(cases[i][0], cases[i][1], cases[i][2], cases[i][3].block_threads, cases[i][3].chain_R,
                            cases[i][3].grid_blocks, cases[i][3].kernel, r[i], want[i]) for i in bad[:5]]


def test_random_row_shapes_on_exact_inputs():
    """As above: integer-valued rows, numpy's binary64 row sums are the exact sums."""
    rng = np.random.default_rng(5585)
    pool = W.small_integers((1 << 22) + 4096, seed=13, lo=-3, hi=3)
    dev = torch.from_numpy(pool.view(np.int16)).cuda()
    pool64 = pool.astype(np.float64)
    csum = np.concatenate([[0.0], np.cumsum(pool64)])
    for _ in range(60):
        cols = int(rng.choice([rng.integers(1, 40), rng.integers(1, 3000), rng.integers(1, 40000)]))
        stride = cols + int(rng.choice([0, 1, 3, 8, 16])) if rng.random() < 0.5 else (cols + 7) // 8 * 8
        rows = int(min(rng.choice([1, 2, 9, 100, 1500, 6000]), ((1 << 22) - 64) // stride))
        start = int(rng.choice([0, 0, 8, rng.integers(0, 16)]))
        use_default = rng.random() < 0.6
        t = None if use_default else random_tuning(rng, B.MFR_DTYPE_F16)
        if t is not None and t.kernel == 2:
            t.kernel, t.split_permille = 0, 0
        o = Outputs(rows + 1)
        B.mfr_sum_rows_ex(dev.data_ptr() + 2 * start, B.MFR_DTYPE_F16, rows, cols, stride, o.ptr(0), t, stream_handle())
        r = o.get().astype(np.float64)
        want = np.array([csum[start + k * stride + cols] - csum[start + k * stride] for k in range(rows)])
        assert r[rows] == Outputs.SENTINEL
        assert np.array_equal(r[:rows], want), (rows, cols, stride, start, use_default, np.nonzero(r[:rows] != want)[0][:5])


def test_denormal_inputs_fp32_and_bf16(oracle_lib):
    # subnormal inputs of the wider types are honoured by the matrix path and by the conventional path
    n = 1 << 20
    f = np.full(n, 2.0 ** -140, dtype=np.float32)                 # subnormal binary32
    b = np.full(n, 0x0001, dtype=np.uint16)                        # smallest subnormal bfloat16 (2^-133)
    for dtype, host, want in ((B.MFR_DTYPE_F32, torch.from_numpy(f), n * 2.0 ** -140),
                              (B.MFR_DTYPE_BF16, torch.from_numpy(b.view(np.int16)), n * 2.0 ** -133)):
        d = host.cuda()
        o = Outputs(2)
        B.mfr_sum_ex(d.data_ptr(), dtype, n, o.ptr(0), B.make_tuning(kernel=B.MFR_KERNEL_MFMA), stream_handle())
        B.mfr_sum_ex(d.data_ptr(), dtype, n, o.ptr(1), B.make_tuning(kernel=B.MFR_KERNEL_SHFL), stream_handle())
        r = o.get().astype(np.float64)
        print("subnormal inputs dtype=%d: mfma=%r shfl=%r exact=%r" % (dtype, float(r[0]), float(r[1]), want))
        for v in r:
            assert abs(v - want) <= 1e-5 * want                   # honoured by both paths (not flushed)

"""The entry point that allocates nothing (scratch in a fixed device array) against the entry
point it is a variant of, mfr_sum_f16_ex: same kernels and geometry, so the results must be the
same bits; and against the CPU oracle within the usual tolerance.  Two calls in a row share the
array, the second with a smaller input, then more calls of alternating sizes and grids."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2001_05585_amd import binding as B            # noqa: E402
from paper_2001_05585_amd import workloads as W          # noqa: E402
from gpu_util import DeviceInput, Outputs, stream_handle  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; the HIP path has no fallback")
    B.lib()


def both(d, n, tuning):
    o = Outputs(2)
    B.mfr_sum_f16_noalloc(d.ptr, n, o.ptr(0), tuning, stream_handle())
    B.mfr_sum_f16_ex(d.ptr, n, o.ptr(1), tuning, stream_handle())
    r = o.get()
    return r[0], r[1]


def test_two_calls_in_a_row_the_second_smaller(oracle_lib):
    big = W.generate("uniform_pm1", (1 << 23) + 77, 991)
    small = W.generate("normal", (1 << 19) + 5, 992)
    d_big, d_small = DeviceInput(big, 3), DeviceInput(small, 1)
    o = Outputs(4)
    s = stream_handle()
    B.mfr_sum_f16_noalloc(d_big.ptr, big.size, o.ptr(0), None, s)        # first call
    B.mfr_sum_f16_noalloc(d_small.ptr, small.size, o.ptr(1), None, s)    # second call, smaller input
    B.mfr_sum_f16_ex(d_big.ptr, big.size, o.ptr(2), None, s)
    B.mfr_sum_f16_ex(d_small.ptr, small.size, o.ptr(3), None, s)
    r = o.get()
    assert r[0] == r[2] and r[1] == r[3], r
    for got, x in ((r[0], big), (r[1], small)):
        want, sum_abs = oracle_lib.sum_f16(x)
        assert abs(float(got) - want) <= 1e-5 * sum_abs


def test_same_bits_as_the_allocating_entry_point_over_sizes_and_grids():
    x = W.small_integers((1 << 22) + 999, seed=12, lo=-3, hi=3)
    y = W.generate("normal", (1 << 22) + 999, 13)
    dx, dy = DeviceInput(x, 2), DeviceInput(y)
    tunings = [None, B.make_tuning(256, 1), B.make_tuning(64, 2, 2048), B.make_tuning(128, 4, 8192, 1),
               B.make_tuning(1024, 1, 7, 0, 2, 0, B.MFR_COMBINE_TWO_LAUNCHES), B.make_tuning(64, 1, 5000, 0, 1, 0, B.MFR_COMBINE_SINGLE_LAUNCH),
               B.make_tuning(32, 8, 300), B.make_tuning(256, 3, 2, 2, 2, 0, 0, 400)]
    sizes = [x.size, 1 << 20, 70000, 49152, 513, 1, 0, (1 << 21) + 3, 2000, x.size]
    for n in sizes:                      # large and small inputs alternate on the same array
        for t in tunings:
            a, b = both(dx, n, t)
            assert a == b == float(x[:n].astype(np.float64).sum()), (n, t and (t.block_threads, t.chain_R, t.grid_blocks))
            a, b = both(dy, n, t)
            assert a == b, (n, t and (t.block_threads, t.chain_R, t.grid_blocks))


def test_grids_beyond_the_fixed_scratch_are_refused():
    d = DeviceInput(W.ones(1 << 22))
    o = Outputs(1)
    L = B.lib()
    s = stream_handle()
    t = B.make_tuning(64, 1, 8193)
    assert L.mfr_sum_f16_noalloc(d.ptr, d.n, o.ptr(0), t, s) == B.MFR_ERR_SCRATCH_LIMIT
    t = B.make_tuning(64, 1, B.MFR_GRID_ONE_CHAIN)             # one chain per wave: 8192 blocks of one wave -> fits
    assert L.mfr_sum_f16_noalloc(d.ptr, 8192 * 512, o.ptr(0), t, s) == B.MFR_OK
    assert L.mfr_sum_f16_noalloc(d.ptr, 8193 * 512, o.ptr(0), t, s) == B.MFR_ERR_SCRATCH_LIMIT
    assert o.get()[0] == 8192 * 512.0                          # the refused call enqueued nothing
    assert "scratch" in B.mfr_strerror(B.MFR_ERR_SCRATCH_LIMIT)
    assert L.mfr_sum_f16_noalloc(None, 5, o.ptr(0), None, s) == B.MFR_ERR_INVALID_ARG
    assert L.mfr_sum_f16_noalloc(d.ptr, 5, None, None, s) == B.MFR_ERR_INVALID_ARG
    assert L.mfr_sum_f16_noalloc(d.ptr + 1, 5, o.ptr(0), None, s) == B.MFR_ERR_INVALID_ARG


def test_can_be_captured_without_a_warm_up_call_on_the_stream():
    """Nothing is allocated, so unlike mfr_sum_f16_ex the very first call on a stream can be captured."""
    n = (1 << 21) + 9
    x = W.small_integers(n, seed=77, lo=-2, hi=2)
    want = float(x.astype(np.float64).sum())
    d = DeviceInput(x, 2)
    out = Outputs(1)
    B.mfr_sum_f16_noalloc(d.ptr, 16, out.ptr(0), None, stream_handle())      # loads the code object, looks the array up
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        B.mfr_sum_f16_noalloc(d.ptr, n, out.ptr(0), None, s.cuda_stream)
    for rep in range(4):
        out.tensor.fill_(-1.0)
        torch.cuda.synchronize()
        g.replay()
        assert out.get()[0] == want, rep
        # eager work between the replays
        B.mfr_sum_f16_noalloc(d.ptr, 70000, out.ptr(0), None, stream_handle())
        assert out.get()[0] == float(x[:70000].astype(np.float64).sum())

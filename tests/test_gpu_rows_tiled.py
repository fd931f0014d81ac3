"""GPU parity of the many-rows kernel (accumulator columns shared out among rows)
against the CPU oracle, through mfr_sum_rows_ex with library defaults.

Integer-valued inputs (every partial sum exact in fp32): bit-exact.  Random
inputs: |gpu - oracle| <= 1e-5 * sum |x_i| per row.  The gaps between rows and
the bytes around the array hold NaN, so that a value read from outside a row
and not masked shows up in that row's sum."""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2001_05585_amd import binding as B            # noqa: E402
from paper_2001_05585_amd import workloads as W          # noqa: E402
from gpu_util import Outputs, stream_handle              # noqa: E402

TOL = 1e-5
F16, BF16, F32 = B.MFR_DTYPE_F16, B.MFR_DTYPE_BF16, B.MFR_DTYPE_F32
NAN = {F16: 0x7E00, BF16: 0x7FC0, F32: 0x7FC00000}
STORAGE = {F16: np.uint16, BF16: np.uint16, F32: np.uint32}


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; the HIP path has no fallback")
    B.lib()


def cus():
    return torch.cuda.get_device_properties(0).multi_processor_count


def encode(dtype, values):
    """float32 values -> storage bits of the element type (values are exactly representable)."""
    v = np.asarray(values, dtype=np.float32)
    if dtype == F16:
        return v.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        return W.to_bf16_bits(v)
    return v.view(np.uint32)


class RowsInput:
    """rows x cols values laid out with a stride, NaN in the gaps and around the array, shifted by
    `shift` elements from a 16-byte boundary."""

    def __init__(self, dtype, bits2d, stride, shift):
        rows, cols = bits2d.shape
        st = STORAGE[dtype]
        guard = 64
        span = (rows - 1) * stride + cols
        buf = np.full(span + 2 * guard + 16, NAN[dtype], dtype=st)
        start = guard + shift
        idx = (np.arange(rows)[:, None] * stride + np.arange(cols)[None, :]).ravel() + start
        buf[idx] = bits2d.ravel()
        self.tensor = torch.from_numpy(buf.view(np.int16 if st == np.uint16 else np.int32)).cuda()
        assert self.tensor.data_ptr() % 16 == 0
        self.ptr = self.tensor.data_ptr() + buf.itemsize * start


def call(dtype, inp, rows, cols, stride, tuning=None):
    o = Outputs(rows + 1)
    B.mfr_sum_rows_ex(inp.ptr, dtype, rows, cols, stride, o.ptr(0), tuning, stream_handle())
    r = o.get()
    assert r[rows] == Outputs.SENTINEL            # nothing written past out[rows)
    return r[:rows]


def expect_plan(dtype, inp, rows, cols, stride, **want):
    plan = B.mfr_rows_plan(inp.ptr, dtype, rows, cols, stride, cus())
    assert plan is not None, "the many-rows kernel should be chosen for this shape"
    names = dict(P=0, D=1, GF=2, all_plain=9)
    for k, v in want.items():
        assert plan[names[k]] == v, (k, plan)
    return plan


# (rows, cols, stride, shift) chosen to reach every kernel shape, masked and unmasked
INT_CASES = [
    (4096, 32, 32, 0), (4099, 64, 64, 0), (4100, 128, 128, 0), (2050, 256, 256, 0), (2048, 512, 512, 0),
    (2048, 1024, 1024, 0), (2049, 2048, 2048, 4), (600, 2048, 2048, 0),             # unmasked steps only
    (5003, 1, 1, 0), (5003, 1, 1, 1), (5003, 7, 7, 3), (5003, 31, 33, 0), (5003, 33, 40, 0), (4001, 64, 64, 1),
    (4001, 65, 72, 0), (4001, 100, 100, 0), (4001, 129, 131, 5), (3000, 255, 256, 0), (3000, 300, 304, 7),
    (2500, 500, 500, 2), (2100, 1001, 1001, 0), (2100, 1536, 1544, 4), (2049, 3000, 3002, 0),
    (700, 2500, 2504, 0), (513, 3501, 3504, 6),                                      # long rows from 512 rows on
    (2048, 384, 384, 0), (2048, 640, 648, 0), (2050, 768, 768, 4), (3000, 600, 600, 0), (2048, 350, 353, 1),
    (2048, 300, 300, 0), (2049, 192, 192, 0),                                        # rows over 512 bytes in narrower shapes
    (2048, 257, 257, 0), (2048, 514, 514, 0), (2048, 1030, 1030, 0), (2048, 260, 260, 0),   # whole steps and a few bytes
    (1100, 257, 257, 1), (1100, 129, 129, 0), (1027, 515, 515, 0),
    # 16-bit rows 2 bytes off a 4-byte boundary, all of them or every other one: read from one element earlier
    (4096, 1, 1, 0), (4096, 32, 32, 1), (4096, 64, 64, 1), (4096, 128, 128, 1), (4096, 160, 160, 1), (4096, 256, 256, 1),
    (700, 256, 256, 1), (2048, 1024, 1024, 1), (2048, 288, 288, 1), (2048, 512, 512, 1), (2048, 1025, 1025, 0),
    (2048, 513, 513, 0), (2048, 150, 150, 3), (3000, 97, 97, 0), (1031, 1500, 1500, 5), (4096, 16, 16, 7),
    # rests of up to 128 and 256 bytes after the whole steps: tail tiles with two and four columns per row
    (2051, 289, 290, 0), (2051, 288, 288, 1), (2051, 321, 322, 0), (2051, 320, 320, 1), (2051, 545, 546, 0), (2051, 544, 544, 1),
    (2051, 577, 578, 0), (2051, 576, 576, 1), (2051, 1057, 1058, 0), (2051, 1056, 1056, 1), (2051, 1089, 1090, 0),
    (2051, 1088, 1088, 1), (1029, 600, 600, 0), (1029, 1150, 1150, 0), (1029, 1600, 1600, 0), (2051, 350, 350, 0),
    (2051, 384, 384, 1),
    # rows of two to four 1 KiB steps that end in a masked step or in tail tiles: the instances with the steps written out
    (1030, 1229, 1230, 0), (1030, 1664, 1664, 1), (1030, 1537, 1538, 0), (1030, 1536, 1536, 1), (1030, 1568, 1568, 1),
    (1030, 1601, 1602, 0), (1030, 1600, 1600, 1), (1030, 640, 640, 1), (1030, 1152, 1152, 1), (1031, 2052, 2052, 0),
    (1029, 2100, 2100, 0), (1027, 2150, 2150, 0), (1100, 900, 900, 0), (1100, 1750, 1750, 0),
]

# few rows whose 16-byte phases differ: the per-row kernels, every block doing the slot arithmetic of its own row
MIXED_PHASE_CASES = [(33, 1001, 1001, 0), (100, 37, 39, 1), (1000, 5, 5, 0), (40, 20000, 20001, 0), (7, 100003, 100003, 0),
                     (300, 9001, 9003, 3), (2, 1 << 20 | 1, (1 << 20) + 5, 0), (150, 1, 3, 0)]


@pytest.mark.parametrize("dtype", [F16, BF16, F32])
@pytest.mark.parametrize("rows,cols,stride,shift", INT_CASES)
def test_integer_rows_bit_exact(dtype, rows, cols, stride, shift, oracle_lib):
    """Expected values are numpy's binary64 row sums of small integers: every row sum is an integer far
    below 2^24, so numpy's sum, the oracle's and any other correct sum are the same number (the first
    row is also checked against the oracle itself)."""
    vals = W.small_integers(rows * cols, seed=rows * 31 + cols, lo=-4, hi=4).astype(np.float32).reshape(rows, cols)
    inp = RowsInput(dtype, encode(dtype, vals).reshape(rows, cols), stride, shift)
    expect_plan(dtype, inp, rows, cols, stride)
    want = vals.astype(np.float64).sum(axis=1)
    assert want[0] == oracle_lib.sum_f32(np.ascontiguousarray(vals[0]))[0]
    got = call(dtype, inp, rows, cols, stride).astype(np.float64)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, (rows, cols, stride, shift, bad[:5], got[bad[:5]], want[bad[:5]])


# many 16-bit rows of 4 KiB or more that start 2 bytes off a 4-byte boundary, and rows of 16 KiB or more:
# the per-row kernels again (aligned slots whatever the phase), one block per row
LONG_ROWS_PER_ROW_CASES = [(2049, 3000, 3001, 0), (513, 4001, 4003, 6), (2049, 4096, 4096, 1), (1500, 2048, 2048, 3),
                           (66000, 2048, 2049, 0), (1100, 8192, 8192, 0), (1100, 9001, 9001, 0),
                           # enough rows of 16 KiB and more that the launch limits the blocks resident per CU
                           # (whole rounds of six 128-thread or three 256-thread blocks per CU)
                           (3072, 8192, 8192, 0), (1536, 20000, 20000, 0), (3100, 8192, 8192, 0),
                           # one to two rows per SIMD, rows of 64 KiB and more: a one-wave block per row with 6, 4 or 3 KiB in flight
                           (1100, 40000, 40000, 0), (1300, 33000, 33001, 0), (1800, 33000, 33001, 1)]


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("rows,cols,stride,shift", LONG_ROWS_PER_ROW_CASES)
def test_many_long_rows_through_the_per_row_kernels_bit_exact(dtype, rows, cols, stride, shift):
    vals = W.small_integers(rows * cols, seed=rows * 13 + cols, lo=-4, hi=4).astype(np.float32).reshape(rows, cols)
    inp = RowsInput(dtype, encode(dtype, vals).reshape(rows, cols), stride, shift)
    assert B.mfr_rows_plan(inp.ptr, dtype, rows, cols, stride, cus()) is None
    want = vals.astype(np.float64).sum(axis=1)
    got = call(dtype, inp, rows, cols, stride).astype(np.float64)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, (rows, cols, stride, shift, bad[:5], got[bad[:5]], want[bad[:5]])


@pytest.mark.parametrize("dtype", [F16, F32])
@pytest.mark.parametrize("rows,cols,shift", [(8, (1 << 20) + 5, 0), (9, 300001, 3), (6, 70000, 1), (300, 150001, 0),
                                             (40, 1 << 19, 0), (700, 65544, 0),
                                             # a few rows more than half the SIMDs: two one-wave blocks per row
                                             (520, 66001, 0), (620, 40000, 2),
                                             # one to two rows per SIMD: a one-wave block per row
                                             (1400, 40000, 0)])
def test_few_long_rows_count_every_position_once(dtype, rows, cols, shift):
    """Few long rows with library defaults start at different chains of their row (a step per row that depends on
    the pitch) and wrap round: distinct powers of two at the ends of the row, around every sixteenth of it and at
    random places (zero elsewhere) must add up to 2^K - 1 in every row, whichever chain the row started at."""
    K = 16 if dtype == F16 else 24
    rng = np.random.default_rng(cols + rows)
    marks = [0, 1, 7, 8, cols - 1, cols - 2, cols - 9]
    for k in range(1, 16):
        marks += [k * cols // 16 - 1, k * cols // 16, k * cols // 16 + 8]
    marks += [int(v) for v in rng.integers(0, cols, 200)]
    marks = np.unique(np.array(marks))
    stride = cols + (3 if shift else 0)
    vals = np.zeros((rows, cols), dtype=np.float32)
    for trial in range(4):
        vals[:] = 0
        for r in range(rows):
            pos = rng.choice(marks, K, replace=False) if trial else marks[(np.arange(K) * 3 + r + trial) % marks.size]
            pos = np.unique(pos)
            vals[r, pos] = 2.0 ** rng.permutation(K)[:pos.size]
        want = vals.astype(np.float64).sum(axis=1)
        inp = RowsInput(dtype, encode(dtype, vals).reshape(rows, cols), stride, shift)
        assert B.mfr_rows_plan(inp.ptr, dtype, rows, cols, stride, cus()) is None
        got = call(dtype, inp, rows, cols, stride).astype(np.float64)
        bad = np.nonzero(got != want)[0]
        assert bad.size == 0, (rows, cols, shift, trial, bad[:5], got[bad[:5]], want[bad[:5]])


@pytest.mark.parametrize("dtype", [F16, BF16, F32])
@pytest.mark.parametrize("rows,cols,stride,shift", MIXED_PHASE_CASES)
def test_few_rows_of_differing_phase_bit_exact(dtype, rows, cols, stride, shift):
    vals = W.small_integers(rows * cols, seed=rows * 17 + cols, lo=-4, hi=4).astype(np.float32).reshape(rows, cols)
    inp = RowsInput(dtype, encode(dtype, vals).reshape(rows, cols), stride, shift)
    assert B.mfr_rows_plan(inp.ptr, dtype, rows, cols, stride, cus()) is None
    want = vals.astype(np.float64).sum(axis=1)
    tunings = [None, B.make_tuning(256, 2), B.make_tuning(64, 8, 0, B.MFR_KERNEL_SHFL, 1), B.make_tuning(128, 1, 3, 0, 4, 2)]
    if dtype == F16:
        tunings.append(B.make_tuning(32, 4))
        # split kernel: the chains of a row that starts off a boundary can be one fewer than the host planned
        tunings += [B.make_tuning(256, 2, 0, B.MFR_KERNEL_SPLIT, 0, 0, 0, f) for f in (0, 500, 1000)]
        tunings.append(B.make_tuning(64, 1, 1, B.MFR_KERNEL_SPLIT, 1, 0, 0, 999))
    for t in tunings:
        got = call(dtype, inp, rows, cols, stride, t).astype(np.float64)
        bad = np.nonzero(got != want)[0]
        assert bad.size == 0, (rows, cols, stride, shift, t and (t.block_threads, t.chain_R), bad[:5], got[bad[:5]], want[bad[:5]])


def test_shapes_reach_every_kernel_shape():
    """The bit-exact cases above go through every instance of the many-rows kernel that the library can choose:
    (P, D, GF, unmasked, flags: tail tiles, shifted rows, log2 of the tail tile's columns per row, steps written
    out).  The set of instances is found by asking for the plans of row lengths up to 8200 elements."""
    def instance(plan):
        written_out = plan[0] == 16 and plan[1] == 1 and plan[4] in (2, 3, 4) and \
            ((plan[11] & 1 and plan[2] == 4) or (not plan[11] & 1 and not plan[9]))
        written_out = written_out or (plan[0] == 16 and plan[1] == 4 and plan[4] in (2, 3) and not plan[9])
        return (plan[0], plan[1], plan[2], plan[9], plan[11], plan[4] if written_out else 0)

    seen, reachable = set(), set()
    for dtype in (F16, F32):
        esize = 2 if dtype != F32 else 4
        for rows, cols, stride, shift in INT_CASES:
            plan = B.mfr_rows_plan((1 << 20) + shift * esize, dtype, rows, cols, stride, 256)
            assert plan is not None
            seen.add(instance(plan))
        for rows in (600, 1030):
            for cols in list(range(1, 2700)) + list(range(2700, 8200, 7)):
                for first, gap in ((0, 0), (1, 0), (0, 1), (0, 8)):
                    plan = B.mfr_rows_plan((1 << 20) + first * esize, dtype, rows, cols, cols + gap, 256)
                    if plan is not None:
                        reachable.add(instance(plan))
    assert len(reachable) == 59
    assert seen == reachable, (sorted(reachable - seen), sorted(seen - reachable))


@pytest.mark.parametrize("dtype,kind", [(F16, "normal"), (F16, "uniform01"), (BF16, "normal"), (F32, "uniform_pm1")])
@pytest.mark.parametrize("rows,cols,stride,shift", [(4096, 64, 64, 0), (3001, 100, 104, 1), (2048, 1024, 1024, 0),
                                                    (2051, 777, 777, 0), (600, 3000, 3000, 2)])
def test_random_rows_within_tolerance(dtype, kind, rows, cols, stride, shift, oracle_lib):
    seed = 7000 + rows + cols
    if dtype == F16:
        bits = W.generate(kind, rows * cols, seed).view(np.uint16)
    elif dtype == BF16:
        bits = W.generate_bf16(kind, rows * cols, seed)
    else:
        bits = W.generate_f32(kind, rows * cols, seed).view(np.uint32)
    bits2d = bits.reshape(rows, cols)
    inp = RowsInput(dtype, bits2d, stride, shift)
    expect_plan(dtype, inp, rows, cols, stride)
    s, sa = oracle_lib.sum_rows(bits2d if dtype != F16 else bits2d.view(np.float16), {F16: "f16", BF16: "bf16", F32: "f32"}[dtype])
    got = call(dtype, inp, rows, cols, stride).astype(np.float64)
    assert (np.abs(got - s) <= TOL * sa).all(), np.max(np.abs(got - s) / sa)
    # the per-row kernels (explicit tuning) agree to the same bound
    if (stride * bits.itemsize) % 16 == 0:
        got2 = call(dtype, inp, rows, cols, stride, B.make_tuning(256, 2)).astype(np.float64)
        assert (np.abs(got2 - s) <= TOL * sa).all()


def test_special_values_stay_in_their_row():
    rows, cols, stride = 4100, 96, 100
    vals = np.ones((rows, cols), dtype=np.float32)
    bits = encode(F16, vals).reshape(rows, cols).copy()
    bits[7, cols - 1] = 0x7C00          # +Inf
    bits[8, 0] = 0xFC00                 # -Inf
    bits[4000, 5] = 0x7E00              # NaN
    bits[4099, 0] = 0x7C00; bits[4099, 1] = 0xFC00
    inp = RowsInput(F16, bits, stride, 3)
    got = call(F16, inp, rows, cols, stride).astype(np.float64)
    assert got[7] == math.inf and got[8] == -math.inf and math.isnan(got[4000]) and math.isnan(got[4099])
    keep = np.ones(rows, dtype=bool); keep[[7, 8, 4000, 4099]] = False
    assert np.all(got[keep] == cols)
    # contiguous rows of an odd number of 16-bit elements: every other row is read from the element before it,
    # which is the last element of the row above
    for rows, cols in ((2100, 257), (2100, 129), (3000, 33), (1100, 1025), (2100, 301)):
        bits = encode(F16, np.ones((rows, cols), dtype=np.float32)).reshape(rows, cols).copy()
        bits[10, cols - 1] = 0x7C00       # +Inf just before row 11
        bits[21, cols - 1] = 0x7E00       # NaN just before row 22
        bits[31, 0] = 0xFC00              # -Inf as a shifted row's first element
        bits[rows - 2, cols - 1] = 0x7E00
        inp = RowsInput(F16, bits, cols, 0)
        got = call(F16, inp, rows, cols, cols).astype(np.float64)
        assert got[10] == math.inf and math.isnan(got[21]) and got[31] == -math.inf and math.isnan(got[rows - 2])
        keep = np.ones(rows, dtype=bool); keep[[10, 21, 31, rows - 2]] = False
        assert np.all(got[keep] == cols), (rows, cols, np.nonzero(got[keep] != cols)[0][:5])


def test_sparse_diagonals_every_column_position():
    # a few nonzero values per row among zeros: diagonals that start at rows around the first, a middle
    # and the last iteration and run through every column, each diagonal with its own power of two
    rows, cols, stride = 2600, 75, 77
    bases = (0, 1, 15, 16, 127, 128, 1300, 2470, 2524, 2599)
    for dtype, shift in ((F16, 5), (F16, 0), (F32, 1)):
        vals = np.zeros((rows, cols), dtype=np.float32)
        for i, r0 in enumerate(bases):
            k = np.arange(cols)
            vals[(r0 + k) % rows, k] += 2.0 ** i
        inp = RowsInput(dtype, encode(dtype, vals).reshape(rows, cols), stride, shift)
        got = call(dtype, inp, rows, cols, stride).astype(np.float64)
        want = vals.astype(np.float64).sum(axis=1)
        assert np.array_equal(got, want), (dtype, shift, np.nonzero(got != want)[0][:5])


def test_same_result_at_every_alignment():
    rows, cols = 2304, 200
    vals = W.small_integers(rows * cols, seed=99, lo=-4, hi=4).astype(np.float32).reshape(rows, cols)
    want = vals.astype(np.float64).sum(axis=1)
    for dtype in (F16, F32):
        per_slot = 8 if dtype == F16 else 4
        for shift in range(per_slot):
            for stride in (cols, cols + 1, cols + per_slot):
                inp = RowsInput(dtype, encode(dtype, vals).reshape(rows, cols), stride, shift)
                got = call(dtype, inp, rows, cols, stride).astype(np.float64)
                assert np.array_equal(got, want), (dtype, shift, stride)


def test_more_rows_than_a_grid_dimension_and_tiny_rows():
    rows = 70001
    for cols, stride in ((8, 8), (3, 3), (1, 2)):
        vals = W.small_integers(rows * cols, seed=cols, lo=-4, hi=4).astype(np.float32).reshape(rows, cols)
        inp = RowsInput(F16, encode(F16, vals).reshape(rows, cols), stride, 0)
        got = call(F16, inp, rows, cols, stride).astype(np.float64)
        assert np.array_equal(got, vals.astype(np.float64).sum(axis=1)), (cols, stride)


def test_repeat_calls_are_bit_identical_and_streams_do_not_interfere():
    rows, cols, stride = 6000, 333, 340
    bits = W.generate("normal", rows * cols, 4242).view(np.uint16).reshape(rows, cols)
    inp = RowsInput(F16, bits, stride, 2)
    first = call(F16, inp, rows, cols, stride).view(np.uint32).copy()
    for _ in range(30):
        assert np.array_equal(call(F16, inp, rows, cols, stride).view(np.uint32), first)
    # two streams at once, each with its own output
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    o1, o2 = Outputs(rows), Outputs(rows)
    torch.cuda.synchronize()
    for _ in range(10):
        B.mfr_sum_rows_ex(inp.ptr, F16, rows, cols, stride, o1.ptr(0), None, s1.cuda_stream)
        B.mfr_sum_rows_ex(inp.ptr, F16, rows, cols, stride, o2.ptr(0), None, s2.cuda_stream)
    torch.cuda.synchronize()
    assert np.array_equal(o1.get().view(np.uint32), first) and np.array_equal(o2.get().view(np.uint32), first)


def test_batched_calls_can_be_captured_in_a_hip_graph():
    # the many-rows kernel uses no scratch; the per-row kernels use the stream's scratch, which exists after
    # one eager call: both kinds of call only launch kernels and can be captured and replayed
    shapes = [(3000, 200, 208, 0), (40, 50000, 50001, 1), (1200, 9000, 9000, 0)]
    s = torch.cuda.Stream()
    inputs, outs, wants = [], [], []
    for rows, cols, stride, shift in shapes:
        vals = W.small_integers(rows * cols, seed=rows + cols, lo=-3, hi=3).astype(np.float32).reshape(rows, cols)
        inputs.append(RowsInput(F16, encode(F16, vals).reshape(rows, cols), stride, shift))
        outs.append(Outputs(rows + 1))
        wants.append(vals.astype(np.float64).sum(axis=1))

    def issue():
        for (rows, cols, stride, _), inp, o in zip(shapes, inputs, outs):
            B.mfr_sum_rows_ex(inp.ptr, F16, rows, cols, stride, o.ptr(0), None, s.cuda_stream)
    with torch.cuda.stream(s):
        issue()                                        # eager: allocates the stream's scratch
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        issue()
    for rep in range(4):
        for o in outs:
            o.tensor.fill_(Outputs.SENTINEL)           # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        for (rows, _, _, _), o, want in zip(shapes, outs, wants):
            r = o.get()
            assert r[rows] == Outputs.SENTINEL
            assert np.array_equal(r[:rows].astype(np.float64), want), (rep, rows)


def test_last_rows_whose_final_slot_would_pass_the_array_are_summed_by_extra_blocks(oracle_lib):
    """Contiguous rows whose last 16-byte slot would reach past the array's end are left out of the tiles and
    summed by extra blocks of the same launch from element-wide loads; their sums and the rows before them are
    exact, and nothing past the array is read (RowsInput puts NaN there)."""
    with_last_rows = 0
    for dtype in (F16, BF16, F32):
        for rows, cols, shift in ((3000, 33, 0), (3000, 1, 3), (2048, 257, 0), (1500, 515, 1), (1200, 1021, 0), (1030, 2047, 0),
                                  (600, 2050, 0), (1027, 7, 5), (2049, 100, 1), (1100, 1201, 0)):
            rng = np.random.default_rng(rows + cols)
            vals = rng.integers(-3, 4, size=(rows, cols)).astype(np.float32)
            vals[-1, -1] = 3.0                                   # the very last element of the array counts
            inp = RowsInput(dtype, encode(dtype, vals).reshape(rows, cols), cols, shift)
            plan = B.mfr_rows_plan(inp.ptr, dtype, rows, cols, cols, cus())
            assert plan is not None, (dtype, rows, cols)
            with_last_rows += plan[8] < rows
            got = call(dtype, inp, rows, cols, cols)
            assert np.array_equal(got.astype(np.float64), vals.astype(np.float64).sum(axis=1)), (dtype, rows, cols, shift)
    assert with_last_rows >= 28          # all of them but a binary32 shape or two whose rows are whole slots
    # special values in such a row stay in it
    rows, cols = 2050, 33
    bits = encode(F16, np.ones((rows, cols), dtype=np.float32)).reshape(rows, cols).copy()
    bits[rows - 1, cols - 1] = 0x7C00
    bits[rows - 2, 0] = 0x7E00
    inp = RowsInput(F16, bits, cols, 0)
    assert B.mfr_rows_plan(inp.ptr, F16, rows, cols, cols, cus())[8] < rows
    got = call(F16, inp, rows, cols, cols).astype(np.float64)
    assert got[rows - 1] == math.inf and math.isnan(got[rows - 2]) and np.all(got[: rows - 2] == cols)


def test_alternating_inputs_never_see_the_previous_calls_partials_per_row_kernels():
    """The per-row kernels of a batched call share one scratch array (gridDim.x partials per row) and
    ticket counters per row across calls: two inputs with different exact row sums alternate on one stream."""
    rows, cols = 24, (1 << 17) + 40
    a = RowsInput(F16, encode(F16, np.ones((rows, cols), np.float32)).reshape(rows, cols), cols, 0)
    b = RowsInput(F16, encode(F16, np.full((rows, cols), 3.0, np.float32)).reshape(rows, cols), cols + 8, 1)
    for block, R, grid, combine in ((256, 3, 0, 1), (64, 2, 40, 1), (128, 1, 9, 2), (64, 1, 700, 1)):
        t = B.make_tuning(block, R, grid, 0, 0, 0, combine)
        calls = 400
        o = Outputs(rows * calls)
        for i in range(calls):
            if i % 2 == 0:
                B.mfr_sum_rows_ex(a.ptr, F16, rows, cols, cols, o.ptr(rows * i), t, stream_handle())
            else:
                B.mfr_sum_rows_ex(b.ptr, F16, rows, cols, cols + 8, o.ptr(rows * i), t, stream_handle())
        r = o.get().reshape(calls, rows)
        assert np.all(r[0::2] == float(cols)) and np.all(r[1::2] == 3.0 * cols), (block, R, grid, combine)

"""GPU parity: the HIP path (through the C ABI) against the CPU oracle.

Bit-exact wherever every summation order gives the same fp32 (integer-valued
inputs with sum |x_i| <= 2^24); otherwise |gpu - oracle| <= 1e-5 * sum |x_i|.
"""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2001_05585_amd import binding as B            # noqa: E402
from paper_2001_05585_amd import workloads as W          # noqa: E402
from gpu_util import DeviceInput, Outputs, gpu_sum, stream_handle   # noqa: E402

TOL = 1e-5
BLOCKS = (32, 64, 128, 256, 512, 1024)
KERNELS = (B.MFR_KERNEL_MFMA, B.MFR_KERNEL_SHFL)


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; the HIP path has no fallback")
    B.lib()


def within_tolerance(g, s, sa):
    return abs(float(g) - s) <= TOL * sa


def all_tunings(grids=(0, -1, 3)):
    i = 0
    for kernel in KERNELS:
        for block in BLOCKS:
            for R in range(1, 9):
                for grid in grids:
                    i += 1
                    yield B.make_tuning(block, R, grid, kernel, combine=i % 3)


def describe(t):
    return "kernel=%d block=%d R=%d grid=%d U=%d nt=%d combine=%d" % (
        t.kernel, t.block_threads, t.chain_R, t.grid_blocks, t.chains_in_flight, t.nontemporal, t.combine)


# ------------------------------------------------------------ config 1 ---

def test_config1_uniform_2p20_block256_R1(oracle_lib):
    x = W.generate("uniform01", 1 << 20, W.config_seed(1))
    s, sa = oracle_lib.sum_f16(x)
    g = gpu_sum(x, B.make_tuning(256, 1))
    assert within_tolerance(g, s, sa), (g, s)
    d = DeviceInput(x)
    o = Outputs(2)
    B.mfr_sum_f16_tuned(d.ptr, d.n, o.ptr(0), 256, 1, 0, B.MFR_KERNEL_MFMA, stream_handle())
    B.mfr_sum_f16(d.ptr, d.n, o.ptr(1), stream_handle())
    r = o.get()
    assert within_tolerance(r[0], s, sa) and within_tolerance(r[1], s, sa)
    assert np.float32(r[0]) == g


# ------------------------------------------- closed forms, bit-exact ---

def test_all_ones_2p24_is_exact_in_every_cell():
    x = W.ones(1 << 24)
    d = DeviceInput(x)
    tunings = list(all_tunings(grids=(0, -1)))
    o = Outputs(len(tunings))
    for i, t in enumerate(tunings):
        B.mfr_sum_f16_ex(d.ptr, d.n, o.ptr(i), t, stream_handle())
    r = o.get()
    bad = [describe(t) + " -> %r" % r[i] for i, t in enumerate(tunings) if r[i] != 16777216.0]
    assert not bad, bad[:10]


@pytest.mark.parametrize("kernel", KERNELS)
def test_closed_forms_exact(kernel, oracle_lib):
    cases = []
    for n in (1, 7, 8, 9, 511, 512, 513, 4096, 65536 + 7, (1 << 20) + 7):
        cases.append((W.ones(n), float(n)))
        cases.append((W.constant(n, -3.0), -3.0 * n))
        cases.append((W.constant(n, 0.25), 0.25 * n))
        cases.append((W.alternating(n, 5.0), 5.0 if n % 2 else 0.0))
        q, r = divmod(n, 4)
        cases.append((W.periodic_ramp(n, 4), float(q * 6 + r * (r - 1) // 2)))
    n = 16384
    cases.append((W.periodic_ramp(n, 2048), float(8 * 2048 * 2047 // 2)))
    cases.append((W.periodic_ramp(2048, 2048, 0.5), 2048 * 2047 / 4))
    cases.append((np.concatenate([W.constant(70000, 3.0), W.constant(70000, -3.0), W.constant(5, 0.5)]), 2.5))
    for x, want in cases:
        assert oracle_lib.sum_f16(x)[0] == want          # the oracle agrees with the closed form
        for t in (B.make_tuning(256, 1, 0, kernel), B.make_tuning(64, 4, 5, kernel),
                  B.make_tuning(32, 3, -1, kernel), B.make_tuning(1024, 8, 0, kernel)):
            g = gpu_sum(x, t, shift=3)
            assert float(g) == want, (x.size, describe(t), g, want)


# ----------------------------------------------- one-hot sweep (every slot) ---

@pytest.mark.parametrize("kernel,block,R,grid,U", [
    (B.MFR_KERNEL_MFMA, 64, 2, 2, 1), (B.MFR_KERNEL_MFMA, 128, 1, 2, 2),
    (B.MFR_KERNEL_MFMA, 32, 2, 3, 1), (B.MFR_KERNEL_SHFL, 64, 2, 2, 1),
    (B.MFR_KERNEL_MFMA, 64, 4, 1, 4),
])
@pytest.mark.parametrize("shift", [0, 5])
def test_one_hot_every_position(kernel, block, R, grid, U, shift):
    t = B.make_tuning(block, R, grid, kernel, U)
    waves = max(1, block // 64)
    tile = 256 if block == 32 else 512
    grid_tile = grid * waves * R * U * tile
    n = 3 * grid_tile + 2 * tile + 7
    d = DeviceInput(np.zeros(n, dtype=np.float16), shift)
    positions = list(range(0, n))
    o = Outputs(len(positions))
    one = 0x3C00
    for i, p in enumerate(positions):
        d.set(p, one)
        B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), t, stream_handle())
        d.set(p, 0)
    r = o.get()
    wrong = np.nonzero(r != 1.0)[0]
    assert wrong.size == 0, (describe(t), [(int(positions[i]), float(r[i])) for i in wrong[:8]])


def test_prefix_indicator_around_boundaries():
    t = B.make_tuning(128, 2, 3)
    n = 40000
    ks = sorted(set([0, 1, 7, 8, 9, n] + [b + e for b in (512, 1024, 2048, 3 * 2 * 2 * 512, 6144 * 2) for e in (-1, 0, 1)]))
    for kernel in KERNELS:
        t.kernel = kernel
        for k in ks:
            g = gpu_sum(W.prefix_indicator(n, k), t, shift=1)
            assert float(g) == float(k), (kernel, k, g)


# ------------------------------------ brute force on every small n ---

@pytest.mark.parametrize("kernel", KERNELS)
def test_every_n_up_to_2100_bit_exact(kernel, oracle_lib):
    full = W.small_integers(2100, seed=21)
    for shift in (0, 1, 7):
        d = DeviceInput(full, shift)
        tunings = [B.make_tuning(256, 1, 0, kernel), B.make_tuning(64, 4, 2, kernel), B.make_tuning(32, 2, 0, kernel)]
        o = Outputs(2101 * len(tunings))
        for n in range(2101):
            for j, t in enumerate(tunings):
                B.mfr_sum_f16_ex(d.ptr, n, o.ptr(n * len(tunings) + j), t, stream_handle())
        r = o.get().reshape(2101, len(tunings))
        vals = full.astype(np.float64)
        want = np.concatenate([[0.0], np.cumsum(vals)])
        assert oracle_lib.sum_f16(full)[0] == want[-1]
        for j in range(len(tunings)):
            wrong = np.nonzero(r[:, j] != want)[0]
            assert wrong.size == 0, (kernel, shift, j, wrong[:5], r[wrong[:5], j], want[wrong[:5]])


# ---------------------------------------------------------- invariances ---

def test_integer_inputs_same_bits_for_every_geometry_and_shift(oracle_lib):
    n = (1 << 18) + 7
    x = W.small_integers(n, seed=31)
    want = oracle_lib.sum_f16(x)[0]
    for shift in range(8):
        d = DeviceInput(x, shift)
        tunings = list(all_tunings(grids=(0, 3) if shift else (0, -1, 3)))
        if shift not in (0, 3):
            tunings = tunings[::7]
        o = Outputs(len(tunings))
        for i, t in enumerate(tunings):
            B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), t, stream_handle())
        r = o.get()
        bad = [describe(t) + " -> %r" % r[i] for i, t in enumerate(tunings) if r[i] != want]
        assert not bad, (shift, want, bad[:10])
    # permutation and split additivity
    perm = np.random.default_rng(5).permutation(n)
    assert float(gpu_sum(x[perm])) == want
    a = 100003
    assert float(gpu_sum(x[:a])) + float(gpu_sum(x[a:])) == want


def test_in_flight_and_nontemporal_variants_agree():
    n = (1 << 20) + 1234
    x = W.small_integers(n, seed=41)
    want = float(x.astype(np.float64).sum())
    d = DeviceInput(x, 2)
    tunings = []
    for kernel in KERNELS:
        for R in range(1, 9):
            for U in (1, 2, 3, 4, 6, 8):
                if R * U <= 16:
                    for nt in (1, 2):
                        tunings.append(B.make_tuning(256, R, 0, kernel, U, nt))
    o = Outputs(len(tunings))
    for i, t in enumerate(tunings):
        B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), t, stream_handle())
    r = o.get()
    assert all(v == want for v in r), [(describe(t), r[i]) for i, t in enumerate(tunings) if r[i] != want][:8]


# ------------------------------------------------ random inputs, tolerance ---

@pytest.mark.parametrize("kind,cfg,n", [("uniform01", 2, (1 << 22) + 7), ("normal", 3, (1 << 22) + 7),
                                        ("uniform_pm1", 4, 4_000_007), ("uniform01", 5, (1 << 16) + 7),
                                        ("normal", 3, 1000), ("uniform01", 5, 1 << 16)])
def test_random_inputs_within_tolerance(kind, cfg, n, oracle_lib):
    x = W.generate(kind, n, W.config_seed(cfg))
    s, sa = oracle_lib.sum_f16(x)
    d = DeviceInput(x, 0)
    tunings = [None] + list(all_tunings(grids=(0, -1)))[::5]
    o = Outputs(len(tunings))
    for i, t in enumerate(tunings):
        B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), t, stream_handle())
    r = o.get()
    errs = np.abs(r.astype(np.float64) - s) / sa
    assert errs.max() <= TOL, (kind, n, errs.max())
    # fp32 partials cannot overflow where fp16 partials would (sum > 65504)
    assert np.all(np.isfinite(r))


def test_both_combine_modes_agree(oracle_lib):
    n = (1 << 23) + 77
    x = W.generate("uniform_pm1", n, 123)
    s, sa = oracle_lib.sum_f16(x)
    d = DeviceInput(x, 4)
    tunings = [B.make_tuning(block, R, grid, 0, 0, 0, combine)
               for block in (64, 256, 1024) for R in (1, 4) for grid in (0, 2, 777, 5000, -1)
               for combine in (B.MFR_COMBINE_SINGLE_LAUNCH, B.MFR_COMBINE_TWO_LAUNCHES)]
    o = Outputs(len(tunings))
    for i, t in enumerate(tunings):
        B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), t, stream_handle())
    r = o.get()
    assert np.abs(r.astype(np.float64) - s).max() <= TOL * sa
    # the two modes add the same fp32 partials in binary64: same fp32 result up to one rounding
    pairs = r.reshape(-1, 2)
    assert np.all(np.abs(pairs[:, 0] - pairs[:, 1]) <= np.spacing(np.abs(pairs[:, 0]).astype(np.float32)))


# ------------------------------------------------ split variant (Section 5.3) ---

def split_tunings():
    for f in (0, 1, 250, 500, 873, 999, 1000):
        for block, R, grid, U in ((256, 4, 0, 2), (64, 1, 7, 1), (512, 2, 0, 4), (128, 8, -1, 1), (1024, 3, 2, 2)):
            yield B.make_tuning(block, R, grid, B.MFR_KERNEL_SPLIT, U, 0, 0, f)


def test_split_variant_integer_inputs_bit_exact(oracle_lib):
    for n in (1, 511, 5000, (1 << 18) + 7, (1 << 21) + 12345):
        x = W.small_integers(n, seed=900 + n % 13, lo=-4, hi=4)
        want = oracle_lib.sum_f16(x)[0]
        for shift in (0, 5):
            d = DeviceInput(x, shift)
            ts = list(split_tunings())
            o = Outputs(len(ts))
            for i, t in enumerate(ts):
                B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), t, stream_handle())
            r = o.get()
            bad = [(describe(t), t.split_permille, r[i]) for i, t in enumerate(ts) if r[i] != want]
            assert not bad, (n, shift, want, bad[:6])


def test_split_variant_one_hot_and_random(oracle_lib):
    t = B.make_tuning(128, 2, 2, B.MFR_KERNEL_SPLIT, 1, 0, 0, 400)
    n = 3 * (2 * 2 * 2 * 512) + 1024 + 7
    d = DeviceInput(np.zeros(n, dtype=np.float16), 2)
    o = Outputs(n)
    for p in range(n):
        d.set(p, 0x3C00)
        B.mfr_sum_f16_ex(d.ptr, n, o.ptr(p), t, stream_handle())
        d.set(p, 0)
    r = o.get()
    assert np.all(r == 1.0), np.nonzero(r != 1.0)[0][:8]
    n = (1 << 23) + 3
    x = W.generate("normal", n, 4242)
    s, sa = oracle_lib.sum_f16(x)
    d = DeviceInput(x)
    ts = list(split_tunings())
    o = Outputs(len(ts))
    for i, tt in enumerate(ts):
        B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), tt, stream_handle())
    r = o.get().astype(np.float64)
    assert (np.abs(r - s) / sa).max() <= TOL


def test_repeat_calls_are_bit_identical():
    x = W.generate("normal", (1 << 22) + 3, 77)
    d = DeviceInput(x, 1)
    for t in (None, B.make_tuning(64, 1, -1), B.make_tuning(1024, 2, 0, B.MFR_KERNEL_SHFL),
              B.make_tuning(128, 2, 4000, 0, 0, 0, B.MFR_COMBINE_SINGLE_LAUNCH),
              B.make_tuning(128, 2, 4000, 0, 0, 0, B.MFR_COMBINE_TWO_LAUNCHES)):
        o = Outputs(300)
        for i in range(300):
            B.mfr_sum_f16_ex(d.ptr, d.n, o.ptr(i), t, stream_handle())
        r = o.get()
        assert np.all(r.view(np.uint32) == r.view(np.uint32)[0])


def test_two_streams_overlap(oracle_lib):
    xa = W.generate("uniform01", (1 << 22) + 5, 81)
    xb = W.generate("uniform_pm1", (1 << 21) + 9, 82)
    da, db = DeviceInput(xa), DeviceInput(xb, 3)
    oa, ob = Outputs(50), Outputs(50)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for i in range(50):
        B.mfr_sum_f16(da.ptr, da.n, oa.ptr(i), s1.cuda_stream)
        B.mfr_sum_f16(db.ptr, db.n, ob.ptr(i), s2.cuda_stream)
    ra, rb = oa.get(), ob.get()
    sa_, saa = oracle_lib.sum_f16(xa)
    sb_, sba = oracle_lib.sum_f16(xb)
    assert np.all(ra == ra[0]) and np.all(rb == rb[0])
    assert within_tolerance(ra[0], sa_, saa) and within_tolerance(rb[0], sb_, sba)


def test_release_scratch_and_use_the_stream_again():
    n = (1 << 22) + 77
    d = DeviceInput(W.ones(n), 1)
    o = Outputs(6)
    s1 = torch.cuda.Stream()
    B.mfr_release_scratch(s1.cuda_stream)                 # nothing held yet: fine
    B.mfr_sum_f16_ex(d.ptr, n, o.ptr(0), B.make_tuning(64, 1, 65536), s1.cuda_stream)     # a large scratch
    B.mfr_sum_f16_recurrence(d.ptr, n, o.ptr(1), 2, s1.cuda_stream)
    B.mfr_release_scratch(s1.cuda_stream)                 # synchronises the stream first
    B.mfr_sum_f16(d.ptr, n, o.ptr(2), s1.cuda_stream)     # allocates again
    B.mfr_sum_f16_ex(d.ptr, n, o.ptr(3), B.make_tuning(64, 1, 65536), s1.cuda_stream)
    B.mfr_release_scratch(s1.cuda_stream)
    B.mfr_release_scratch(s1.cuda_stream)
    B.mfr_sum_f16(d.ptr, n, o.ptr(4), stream_handle())    # other streams are not affected
    B.mfr_sum_f16(d.ptr, n, o.ptr(5), s1.cuda_stream)
    s1.synchronize()
    assert np.all(o.get()[[0, 2, 3, 4, 5]] == float(n))   # (the recurrence variant's fp16 partials overflow here)


def test_alternating_inputs_never_see_the_previous_calls_partials():
    # the scratch of a stream is reused by every call: a partial left over from the previous call must
    # never be read.  Two inputs with different exact sums alternate on one stream.
    n = (1 << 22) + 640
    a, b = DeviceInput(W.ones(n)), DeviceInput(W.constant(n, 3.0), 1)
    for block, R, grid in ((256, 4, 256), (128, 2, 700), (64, 1, 2048), (64, 1, 8192)):
        for combine in (B.MFR_COMBINE_SINGLE_LAUNCH, B.MFR_COMBINE_TWO_LAUNCHES):
            t = B.make_tuning(block, R, grid, 0, 0, 0, combine)
            o = Outputs(1500)
            for i in range(1500):
                d = a if i % 2 == 0 else b
                B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), t, stream_handle())
            r = o.get()
            assert np.all(r[0::2] == float(n)) and np.all(r[1::2] == 3.0 * n), (block, R, grid, combine)


@pytest.mark.parametrize("kernel", [B.MFR_KERNEL_MFMA, B.MFR_KERNEL_SHFL])
def test_tiny_explicit_grids_on_long_real_inputs_stay_in_tolerance(kernel, oracle_lib):
    """One to three blocks on 2^24 and more values: a wave then runs thousands of chains.  Their fp32
    results are added in binary64, so the error does not grow with that count; uniform [0,1) inputs are
    the hard case for a running sum (every addition rounds, all in the same direction class)."""
    for n, kind in ((1 << 24, "uniform01"), ((1 << 25) + 77, "uniform01"), (1 << 24, "normal")):
        x = W.generate(kind, n, 4242 + n % 13)
        s, sa = oracle_lib.sum_f16(x)
        d = DeviceInput(x, 3)
        cells = [(64, 1, 1, 1), (256, 3, 1, 0), (64, 8, 2, 0), (1024, 2, 3, 0), (128, 5, 1, 0)]
        o = Outputs(len(cells))
        for i, (block, R, grid, U) in enumerate(cells):
            B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), B.make_tuning(block, R, grid, kernel, U), stream_handle())
        r = o.get().astype(np.float64)
        worst = float(np.max(np.abs(r - s))) / sa
        print("grid 1-3, kernel %d, %s n=%d: worst |err|/sum|x| = %.3g" % (kernel, kind, n, worst))
        assert worst <= TOL, (kernel, kind, n, r, s)
        assert worst <= 2e-6      # far inside the gate: (32 R + 8 R + 6) 2^-24 at most, in practice 1e-8


def test_host_threads_sharing_one_stream_while_the_scratch_grows(oracle_lib):
    """Several host threads enqueue on the same stream, with grids that keep outgrowing the stream's
    scratch, half of them with the two-launch combine.  A buffer that is outgrown stays allocated
    (work enqueued earlier still uses it) and the launches of one call are enqueued under the stream's
    launch mutex (no other call's kernel gets between a sum kernel and its combine kernel), so every
    result is right whatever the interleaving."""
    import threading
    n = (1 << 20) + 24
    x = W.small_integers(n, seed=5, lo=-2, hi=2)
    want = float(x.astype(np.float64).sum())
    d = DeviceInput(x)
    s = torch.cuda.Stream()
    B.mfr_release_scratch(s.cuda_stream)
    grids = [3, 9, 40, 300, 1500, 5000, 9000, 20000, 40000, 65536]
    threads, per_thread = 4, len(grids) * 6
    o = Outputs(threads * per_thread)
    errors = []

    def work(tid):
        try:
            for j in range(per_thread):
                grid = grids[(j + tid) % len(grids)]
                t = B.make_tuning(64, 1, grid, 0, 1, 0, B.MFR_COMBINE_SINGLE_LAUNCH if j % 2 else B.MFR_COMBINE_AUTO)
                B.mfr_sum_f16_ex(d.ptr, n, o.ptr(tid * per_thread + j), t, s.cuda_stream)
        except Exception as e:      # noqa: BLE001
            errors.append(e)

    ts = [threading.Thread(target=work, args=(i,)) for i in range(threads)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    s.synchronize()
    assert not errors, errors
    r = o.get()
    assert np.all(r == want), [(int(i), float(r[i])) for i in np.nonzero(r != want)[0][:10]]
    B.mfr_release_scratch(s.cuda_stream)


def test_an_mfma_adds_a_column_with_one_rounding(oracle_lib):
    """What the tolerance argument rests on, measured: one column of a tile holds 1.0 followed by 31
    values of 2^-24, each exactly half a unit in the last place of 1.0f.  Thirty-two sequential fp32
    additions would leave 1.0 (every addition is a tie that rounds back to even); the matrix unit adds
    the column's products and the accumulator with a single rounding, so the result is the correctly
    rounded sum, for one tile and for a chain of eight (255 such values).  A chain of R MFMAs therefore
    rounds R times per column, not 32 R times."""
    tiny = np.float16(2.0 ** -24)
    for R in (1, 2, 3, 8):
        # column 0 of a tile = the slots of lanes 0, 16, 32, 48: values 8 l .. 8 l + 7
        col0 = [512 * r + 8 * lane + j for r in range(R) for lane in (0, 16, 32, 48) for j in range(8)]
        x = np.zeros(512 * R, dtype=np.float16)
        x[col0] = tiny
        x[col0[0]] = 1.0
        s, sa = oracle_lib.sum_f16(x)
        assert s == 1.0 + (32 * R - 1) * 2.0 ** -24
        got = gpu_sum(x, B.make_tuning(64, R, 1, B.MFR_KERNEL_MFMA, 1))
        assert float(got) == float(np.float32(s)) != 1.0, (R, float(got), s)
        # the large value last in its column: the same
        x[col0[0]], x[col0[-1]] = tiny, 1.0
        got = gpu_sum(x, B.make_tuning(64, R, 1, B.MFR_KERNEL_MFMA, 1))
        assert float(got) == float(np.float32(s)), (R, float(got), s)


def test_single_launch_combine_with_65536_blocks():
    n = 1 << 25
    d = DeviceInput(W.ones(n))
    o = Outputs(6)
    for i, (grid, combine) in enumerate(((65536, 1), (65536, 2), (65535, 1), (40000, 1), (513, 1), (65537, 1))):
        B.mfr_sum_f16_ex(d.ptr, n, o.ptr(i), B.make_tuning(64, 1, grid, 0, 1, 0, combine), stream_handle())
    assert np.all(o.get() == float(n))


def test_calls_can_be_captured_in_a_hip_graph_once_scratch_exists(oracle_lib):
    # After one warm-up call on a stream (which allocates that stream's scratch) a call only launches
    # kernels, so it can be captured; the ticket counters reset themselves, so the graph can be replayed.
    n = (1 << 21) + 9
    xs = [W.generate("uniform_pm1", n, 700 + i) for i in range(3)]
    want = [oracle_lib.sum_f16(x) for x in xs]
    buf = DeviceInput(xs[0], 2)
    out = Outputs(2)
    s = torch.cuda.Stream()
    tuned = B.make_tuning(128, 2, 600, 0, 0, 0, B.MFR_COMBINE_SINGLE_LAUNCH)
    with torch.cuda.stream(s):
        B.mfr_sum_f16(buf.ptr, n, out.ptr(0), s.cuda_stream)
        B.mfr_sum_f16_ex(buf.ptr, n, out.ptr(1), tuned, s.cuda_stream)
    torch.cuda.synchronize()
    eager = out.get().copy()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        B.mfr_sum_f16(buf.ptr, n, out.ptr(0), s.cuda_stream)
        B.mfr_sum_f16_ex(buf.ptr, n, out.ptr(1), tuned, s.cuda_stream)
    for rep in range(6):
        i = rep % 3
        bits = torch.from_numpy(np.ascontiguousarray(xs[i]).view(np.int16)).cuda()
        buf.tensor[buf.start:buf.start + n] = bits           # eager work between replays
        out.tensor.fill_(Outputs.SENTINEL)
        torch.cuda.synchronize()
        g.replay()
        r = out.get()
        sref, saref = want[i]
        assert abs(float(r[0]) - sref) <= TOL * saref and abs(float(r[1]) - sref) <= TOL * saref, (rep, r, sref)
        if i == 0:
            assert np.array_equal(r, eager)


def test_host_threads_on_their_own_streams(oracle_lib):
    import threading
    inputs = [W.generate("uniform_pm1", (1 << 20) + 17 * k, 200 + k) for k in range(4)]
    devs = [DeviceInput(x, k) for k, x in enumerate(inputs)]
    outs = [Outputs(40) for _ in inputs]
    streams = [torch.cuda.Stream() for _ in inputs]
    errors = []

    def work(k):
        try:
            for i in range(40):
                t = None if i % 2 else B.make_tuning(128, 2, 300 + k)      # exercises scratch growth too
                B.mfr_sum_f16_ex(devs[k].ptr, devs[k].n, outs[k].ptr(i), t, streams[k].cuda_stream)
        except Exception as e:                                             # pragma: no cover
            errors.append(e)

    torch.cuda.synchronize()
    threads = [threading.Thread(target=work, args=(k,)) for k in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    for k, x in enumerate(inputs):
        s, sa = oracle_lib.sum_f16(x)
        r = outs[k].get().astype(np.float64)
        assert np.all(np.abs(r - s) <= TOL * sa)
        assert np.all(r[0::2] == r[0]) and np.all(r[1::2] == r[1])


# ----------------------------------------------------- degenerate cases ---

def test_n_zero_writes_zero():
    d = DeviceInput(W.ones(16))
    o = Outputs(3)
    B.mfr_sum_f16(d.ptr, 0, o.ptr(0), stream_handle())
    B.mfr_sum_f16_tuned(d.ptr, 0, o.ptr(1), 64, 3, -1, B.MFR_KERNEL_SHFL, stream_handle())
    B.lib().mfr_sum_f16(None, 0, o.ptr(2), None)
    r = o.get()
    assert np.all(r == 0.0)


def test_special_values_propagate():
    n = 100000
    for kernel in KERNELS:
        t = B.make_tuning(256, 2, 0, kernel)
        for pos in (0, 511, 70001, n - 1):
            x = W.ones(n).view(np.uint16).copy()
            x[pos] = 0x7C00
            assert float(gpu_sum(x, t)) == math.inf
            x[(pos + 777) % n] = 0xFC00
            assert math.isnan(float(gpu_sum(x, t)))
            x = W.ones(n).view(np.uint16).copy()
            x[pos] = 0x7E01
            assert math.isnan(float(gpu_sum(x, t)))


def test_largest_finite_values_do_not_overflow_fp32():
    n = 1 << 16
    x = W.constant(n, 65504.0)
    for kernel in KERNELS:
        g = gpu_sum(x, B.make_tuning(256, 4, 0, kernel))
        assert float(g) == 65504.0 * n


def test_subnormal_inputs_are_within_tolerance(oracle_lib):
    # 2^24 copies of the smallest subnormal: exactly 1.0 if the hardware honours
    # fp16 subnormals, 0.0 if it flushes them; both facts are reported, the
    # conventional kernel (v_cvt_f32_f16) must honour them.
    x = np.full(1 << 24, 1, dtype=np.uint16)
    g_shfl = float(gpu_sum(x, B.make_tuning(256, 4, 0, B.MFR_KERNEL_SHFL)))
    g_mfma = float(gpu_sum(x, B.make_tuning(256, 4, 0, B.MFR_KERNEL_MFMA)))
    print("subnormal sum: mfma=%r shfl=%r (oracle 1.0)" % (g_mfma, g_shfl))
    assert g_mfma in (0.0, 1.0) and g_shfl in (0.0, 1.0)
    assert g_mfma == 1.0, "MFMA path flushes fp16 subnormals"


def test_odd_pointer_is_rejected():
    d = DeviceInput(W.ones(64))
    o = Outputs(1)
    assert B.lib().mfr_sum_f16(d.ptr + 1, 8, o.ptr(0), None) == B.MFR_ERR_INVALID_ARG


def test_environment_override_reaches_the_default_entry():
    # MFR_BLOCK / MFR_R are read once per process: run in a fresh interpreter
    import os
    import subprocess
    import sys
    code = (
        "import numpy as np, torch\n"
        "from paper_2001_05585_amd import binding as B, workloads as W\n"
        "x = torch.from_numpy(W.generate('normal', (1 << 22) + 5, 11).view(np.int16)).cuda()\n"
        "o = torch.zeros(2, dtype=torch.float32, device='cuda')\n"
        "s = torch.cuda.current_stream().cuda_stream\n"
        "B.mfr_sum_f16(x.data_ptr(), x.numel(), o.data_ptr(), s)\n"
        "B.mfr_sum_f16_ex(x.data_ptr(), x.numel(), o.data_ptr() + 4, B.make_tuning(64, 2), s)\n"
        "torch.cuda.synchronize()\n"
        "r = o.cpu().numpy().view(np.uint32)\n"
        "print(B.mfr_get_default_tuning(), int(r[0]), int(r[1]), B.mfr_grid_for(x.numel(), x.data_ptr(), None))\n")
    env = dict(os.environ, MFR_BLOCK="64", MFR_R="2")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], env=env, cwd=root, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    fields = r.stdout.strip().splitlines()[-1]
    assert fields.startswith("(64, 2, 0)"), fields
    bits_default, bits_explicit, grid = [int(v) for v in fields.split(")")[1].split()]
    assert bits_default == bits_explicit            # the default entry ran the overridden geometry
    assert grid == 4 * torch.cuda.get_device_properties(0).multi_processor_count   # 64-thread blocks: four per CU


def test_stamped_call_gives_the_same_sum_and_ordered_stamps(oracle_lib):
    """The diagnostic entry runs the same kernels: same bits as mfr_sum_f16_ex, and per block
    start <= chains consumed <= handed over, with exactly one block storing the result, last of all."""
    x = W.generate("uniform_pm1", (1 << 22) + 3, 321)
    d = DeviceInput(x, 1)
    for t in (None, B.make_tuning(256, 3, 40), B.make_tuning(64, 1, 700, B.MFR_KERNEL_SHFL), B.make_tuning(256, 2, 1)):
        grid = B.mfr_grid_for(d.n, d.ptr, t)
        stamps = torch.zeros(4 * grid, dtype=torch.int64, device="cuda")
        o = Outputs(2)
        B.mfr_sum_f16_stamped(d.ptr, d.n, o.ptr(0), t, stamps.data_ptr(), 4 * grid, stream_handle())
        B.mfr_sum_f16_ex(d.ptr, d.n, o.ptr(1), t, stream_handle())
        r = o.get()
        assert r[0] == r[1]
        st = stamps.cpu().numpy().reshape(grid, 4)
        assert np.all(st[:, 0] > 0) and np.all(st[:, 0] <= st[:, 1]) and np.all(st[:, 1] <= st[:, 2])
        storing = np.nonzero(st[:, 3])[0]
        assert storing.tolist() == [grid - 1] and st[grid - 1, 3] >= st[:, 2].max()
    assert B.lib().mfr_sum_f16_stamped(d.ptr, d.n, o.ptr(0), None, stamps.data_ptr(), 3, stream_handle()) == B.MFR_ERR_INVALID_ARG
    assert B.lib().mfr_sum_f16_stamped(d.ptr, d.n, o.ptr(0), None, None, 1 << 20, stream_handle()) == B.MFR_ERR_INVALID_ARG
    assert 1000 <= B.mfr_wall_clock_khz() <= 10_000_000

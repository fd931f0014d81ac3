"""GPU parity of the recurrence variant (Section 5.1) against its CPU model
(oracle/recurrence_model.py) and against the fp64 oracle.

* Bit-exact on the model's hand-derived pins (tests/test_recurrence_model.py)
  and on integer inputs of moderate size: there every binary32 sum inside an
  MMA is exact whatever the order the hardware adds in, while the two binary16
  roundings of every group are anything but trivial, so GPU and model must
  agree in every bit, level by level.
* On random real inputs the model rounds once per MMA where the hardware may
  round partial sums inside one, so a value may round the other way in a rare
  tie: both must lie within the binary16 rounding bound of the fp64 oracle,
  and overflow to Inf on the same inputs.
"""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import recurrence_model as RM                  # noqa: E402
from paper_2001_05585_amd import binding as B             # noqa: E402
from paper_2001_05585_amd import workloads as W           # noqa: E402
from gpu_util import DeviceInput, Outputs, stream_handle   # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; the HIP path has no fallback")
    B.lib()


def gpu_recurrence(x, R, shift=0, n=None):
    d = DeviceInput(x, shift)
    o = Outputs(1)
    B.mfr_sum_f16_recurrence(d.ptr, d.n if n is None else n, o.ptr(0), R, stream_handle())
    return float(o.get()[0])


@pytest.mark.parametrize("R", range(1, 9))
def test_exact_cases_match_model_bit_for_bit(R, oracle_lib):
    for n in (1, 2, 8, 511, 512, 513, 2048, 512 * R, 512 * R + 1, 3 * 512 * R + 77):
        x = W.small_integers(n, seed=7 * n + R, lo=-1, hi=1)
        for shift in (0, 3):
            want = float(RM.recurrence(x, R, head=shift))
            got = gpu_recurrence(x, R, shift)
            assert got == want, (R, n, shift, got, want)
            if np.abs(x.astype(np.float64)).sum() <= 2048:
                assert got == oracle_lib.sum_f16(x)[0]
    assert gpu_recurrence(W.ones(2048), R) == 2048.0
    assert gpu_recurrence(W.alternating(300001, 2.0), R) == 2.0
    assert gpu_recurrence(W.ones(16), R, n=0) == 0.0


def planted(n, entries):
    x = np.zeros(n, dtype=np.float16)
    for index, value in entries:
        x[index] = value
    return x


def test_hand_derived_rounding_cases():
    """The cases of tests/test_recurrence_model.py whose values are worked out by hand there."""
    x = planted(512, [(8 * c, 1024.0) for c in range(15)] + [(8 * c + 1, 1.5) for c in range(15)] + [(120, -8000.0)])
    assert gpu_recurrence(x, 1) == 7392.0                      # the copy of C into the fp16 operand rounds
    assert gpu_recurrence(W.ones(2049), 5) == 2048.0           # the fp16 store rounds
    assert gpu_recurrence(W.ones(2051), 5) == 2052.0
    assert gpu_recurrence(planted(512, [(0, 2048.0), (1, 1.0), (2, 2.0 ** -20)]), 1) == 2048.0      # C is binary32
    assert gpu_recurrence(planted(1024, [(0, 2048.0), (1, 1.0), (512, 2.0 ** -20)]), 2) == 2048.0
    assert gpu_recurrence(planted(512, [(0, 2048.0), (8, 1.0), (16, 2.0 ** -20)]), 1) == 2048.0
    assert gpu_recurrence(planted(512, [(0, 40000.0), (1, 40000.0), (8, -60000.0)]), 1) == math.inf
    assert gpu_recurrence(planted(512, [(0, 40000.0), (16, 40000.0), (8, -60000.0)]), 1) == 20000.0
    x = planted(3 * 512, [(512 * g, 2048.0) for g in range(3)] + [(512 * g + 8, 1.0) for g in range(3)])
    assert gpu_recurrence(x, 1) == 6144.0                      # two levels, each rounds
    x = planted(9 * 512, [(512 * g, 2050.0) for g in range(3)] + [(512 * 8, -6000.0)])
    assert gpu_recurrence(x, 1) == 152.0                       # the level-2 copy decides (exact sum 150)
    x = planted(16, [(0, 2048.0), (1, 1.0), (8, -2048.0)])
    assert gpu_recurrence(x, 1, shift=0) == 0.0 and gpu_recurrence(x, 1, shift=7) == 1.0


@pytest.mark.parametrize("R", range(1, 9))
def test_integer_inputs_with_nontrivial_fp16_roundings_match_model_bit_for_bit(R):
    """Random integers (up to +-300 for short inputs, less for long ones so that totals stay in range):
    column sums and group totals reach thousands (spacing 2 to 32 in binary16, so the copy and the store
    round in most groups at one level or another) yet stay far below 2^24, so every binary32 sum is exact
    in any order and the model's result is the only correct one."""
    rounded = cases = 0
    for n, seed in ((512 * R, 1), (512 * R * 5 + 13, 2), (70001, 3), (512 * R * 512 * R + 999 if R <= 2 else 300007, 4),
                    ((1 << 21) + 77, 5)):
        hi = max(2, min(300, int(20000 * 1.7 / n ** 0.5)))
        x = W.small_integers(n, seed=seed * 31 + R, lo=-hi, hi=hi)
        for shift in (0, 1, 6):
            want = float(RM.recurrence(x, R, head=shift))
            got = gpu_recurrence(x, R, shift)
            assert got == want or (math.isnan(got) and math.isnan(want)), (R, n, shift, got, want)
            assert math.isfinite(want)
        rounded += float(RM.recurrence(x, R)) != float(x.astype(np.float64).sum())
        cases += 1
    print("recurrence R=%d: the fp16 roundings changed the result in %d of %d integer cases" % (R, rounded, cases))
    assert rounded >= 2        # the cases are not trivially exact


@pytest.mark.parametrize("R", [1, 4, 5])
def test_uniform_inputs_overflow_like_the_model(R, oracle_lib):
    x = W.generate("uniform01", 1 << 22, W.config_seed(2))
    assert math.isinf(float(RM.recurrence(x, R))) and gpu_recurrence(x, R) == math.inf
    assert gpu_recurrence(W.ones(1 << 20), R) == math.inf
    # the single-pass path keeps fp32 partials and does not overflow on the same input
    d = DeviceInput(x)
    o = Outputs(1)
    B.mfr_sum_f16(d.ptr, d.n, o.ptr(0), stream_handle())
    s, sa = oracle_lib.sum_f16(x)
    assert abs(float(o.get()[0]) - s) <= 1e-5 * sa
    m = 60000
    s, sa = oracle_lib.sum_f16(x[:m])
    got = gpu_recurrence(x[:m], R)
    assert math.isfinite(got) and abs(got - s) <= RM.error_bound(sa, m, R)


@pytest.mark.parametrize("kind", ["normal", "uniform_pm1"])
def test_random_inputs_within_fp16_rounding_bound_and_near_model(kind, oracle_lib):
    same = total = 0
    for R in (1, 2, 4, 5, 8):
        for n in (1000, 100003, (1 << 21) + 5, 1 << 24):
            x = W.generate(kind, n, 31 + n % 7)
            s, sa = oracle_lib.sum_f16(x)
            for shift in (0, 5):
                got = gpu_recurrence(x, R, shift)
                model = float(RM.recurrence(x, R, head=shift))
                bound = RM.error_bound(sa, n, R, shift)
                assert math.isfinite(got)
                assert abs(got - s) <= bound and abs(model - s) <= bound, (kind, R, n, got, model, s)
                assert abs(got - model) <= 2 * bound
                same += got == model
                total += 1
    print("recurrence (%s): GPU == CPU model bit-for-bit in %d of %d cases" % (kind, same, total))
    assert same >= total // 2          # ties that round differently are rare


def test_recurrence_argument_checks():
    d = DeviceInput(W.ones(64))
    o = Outputs(1)
    L = B.lib()
    assert L.mfr_sum_f16_recurrence(d.ptr, 64, o.ptr(0), 0, None) == B.MFR_ERR_INVALID_ARG
    assert L.mfr_sum_f16_recurrence(d.ptr, 64, o.ptr(0), 9, None) == B.MFR_ERR_INVALID_ARG
    assert L.mfr_sum_f16_recurrence(d.ptr + 1, 64, o.ptr(0), 4, None) == B.MFR_ERR_INVALID_ARG
    assert L.mfr_sum_f16_recurrence(None, 64, o.ptr(0), 4, None) == B.MFR_ERR_INVALID_ARG
    assert L.mfr_sum_f16_recurrence(d.ptr, 64, None, 4, None) == B.MFR_ERR_INVALID_ARG


def test_error_vs_n_table(oracle_lib):
    """Section 5.4's error experiment on this GPU: % error |gpu - cpu| / |cpu| against the fp64
    oracle over n, for normal(0,1) and uniform[0,1) inputs (printed; `bench.py --sweep variants`
    writes the same table)."""
    lines = ["# kind n cpu_fp64_sum single_pass_err% recurrence_R4_err% recurrence_R5_err% shuffle_err% single_pass_err/sum|x|"]
    for kind, cfg in (("normal", 3), ("uniform01", 2)):
        x = W.generate(kind, 1 << 26, W.config_seed(cfg))
        d = DeviceInput(x)
        for k in range(10, 27, 2):
            n = 1 << k
            s, sa = oracle_lib.sum_f16(x[:n])
            o = Outputs(4)
            B.mfr_sum_f16(d.ptr, n, o.ptr(0), stream_handle())
            B.mfr_sum_f16_recurrence(d.ptr, n, o.ptr(1), 4, stream_handle())
            B.mfr_sum_f16_recurrence(d.ptr, n, o.ptr(2), 5, stream_handle())
            B.mfr_sum_f16_tuned(d.ptr, n, o.ptr(3), 256, 4, 0, B.MFR_KERNEL_SHFL, stream_handle())
            r = o.get().astype(np.float64)
            pct = [100.0 * abs(v - s) / abs(s) if math.isfinite(v) else math.inf for v in r]
            lines.append("%s %d %.6f %.3g %.3g %.3g %.3g %.3g" % (kind, n, s, pct[0], pct[1], pct[2], pct[3], abs(r[0] - s) / sa))
            assert abs(r[0] - s) <= 1e-5 * sa and abs(r[3] - s) <= 1e-5 * sa
            for j, R in ((1, 4), (2, 5)):
                if kind == "normal":
                    assert abs(r[j] - s) <= RM.error_bound(sa, n, R)
                elif s > 65520:
                    assert r[j] == math.inf            # fp16 partials overflow (Section 5.4)
                else:
                    assert abs(r[j] - s) <= RM.error_bound(sa, n, R)
    print("\n".join(lines))

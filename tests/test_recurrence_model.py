"""Pins for the CPU model of the recurrence variant (Section 5.1, Algorithms 1-2):
exact where every stored value is binary16-exact, overflow where the paper says
it overflows, and within the binary16 rounding bound of the fp64 oracle elsewhere."""
import math

import numpy as np
import pytest

from oracle import recurrence_model as RM
from paper_2001_05585_amd import workloads as W


@pytest.mark.parametrize("R", [1, 2, 4, 5, 8])
def test_small_integer_inputs_are_exact(oracle_lib, R):
    # all partial sums are integers of magnitude <= 2048: every binary16 store is exact
    for n in (1, 2, 7, 511, 512, 513, 2047, 2048):
        x = W.ones(n)
        assert float(RM.recurrence(x, R)) == float(n)
    for n in (1, 100, 5000, 512 * R * 3 + 17):
        x = W.small_integers(n, seed=n + R, lo=-1, hi=1)
        if np.abs(x.astype(np.float64)).sum() <= 2048:
            assert float(RM.recurrence(x, R)) == oracle_lib.sum_f16(x)[0]
    x = W.alternating(100000, 3.0)
    assert float(RM.recurrence(x, R)) == 0.0
    for head in range(8):
        x = W.small_integers(1500, seed=head, lo=-1, hi=1)
        assert float(RM.recurrence(x, R, head)) == oracle_lib.sum_f16(x)[0]


def test_single_level_matches_the_two_step_definition():
    # one group, R = 1: column sums rounded to fp16, then added and rounded (eq. MMA1, MMA2 with fp16 A)
    rng = np.random.default_rng(1)
    x = rng.normal(0, 30, size=512).astype(np.float16)
    cols = np.zeros(16)
    for v, val in enumerate(x.astype(np.float64)):
        cols[(v // 8) % 16] += val
    want = np.float16(np.sum(cols.astype(np.float16).astype(np.float64)))
    assert RM.level(x, 1)[0] == want
    assert RM.level(x, 1).size == 1 and RM.level(np.concatenate([x, x[:1]]), 1).size == 2


@pytest.mark.parametrize("R", [1, 4, 5])
def test_uniform_inputs_overflow_as_the_paper_reports(oracle_lib, R):
    # positive inputs: once a stored value passes 65504 the result is +inf (Section 5.4)
    n = 1 << 20
    x = W.generate("uniform01", n, W.config_seed(2))
    s, _ = oracle_lib.sum_f16(x)
    assert s > 65520
    assert math.isinf(float(RM.recurrence(x, R)))
    # ... while a short prefix whose sum stays in range is still finite and close
    m = 60000
    s, sa = oracle_lib.sum_f16(x[:m])
    r = float(RM.recurrence(x[:m], R))
    assert math.isfinite(r) and abs(r - s) <= RM.error_bound(sa, m, R)
    assert float(RM.recurrence(W.ones(1 << 20), 4)) == math.inf     # 512 groups of 2048 -> 2^20 > 65504


@pytest.mark.parametrize("kind", ["normal", "uniform_pm1"])
@pytest.mark.parametrize("R", [1, 4, 8])
def test_random_inputs_within_the_fp16_rounding_bound(oracle_lib, kind, R):
    for n in (1000, 100003, 1 << 21):
        x = W.generate(kind, n, 77 + n % 11)
        s, sa = oracle_lib.sum_f16(x)
        r = float(RM.recurrence(x, R, head=n % 8))
        assert math.isfinite(r)
        assert abs(r - s) <= RM.error_bound(sa, n, R, n % 8), (kind, R, n, r, s)


def test_levels_needed():
    assert RM.levels_needed(1, 4) == 1 and RM.levels_needed(2048, 4) == 1 and RM.levels_needed(2049, 4) == 2
    assert RM.levels_needed(2048 * 2048, 4) == 2 and RM.levels_needed(2048 * 2048 + 1, 4) == 3
    assert RM.levels_needed(2041, 4, head=7) == 1 and RM.levels_needed(2042, 4, head=7) == 2

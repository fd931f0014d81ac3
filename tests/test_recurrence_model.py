"""Pins for the CPU model of the recurrence variant (Section 5.1, Algorithms 1-2, chains of Section 4.3).

The expected values below are worked out by hand from the algorithm's steps (the arithmetic is in the
comments), not taken from the model: each case is built so that one particular rounding decides the
result, and states what the result would be if that rounding were missing.  binary16 facts used:
spacing 1 in [1024, 2048), 2 in [2048, 4096), 4 in [4096, 8192); ties go to the even significand;
values above 65504 + 16 become infinity.
"""
import math

import numpy as np
import pytest

from oracle import recurrence_model as RM
from paper_2001_05585_amd import workloads as W


def tile_values(n, entries):
    x = np.zeros(n, dtype=np.float16)
    for index, value in entries:
        x[index] = value
        assert float(x[index]) == value          # every planted value is a binary16 number
    return x


# ----------------------------------------------------------------- one group, by hand ---

def test_copy_of_C_into_the_fp16_operand_rounds_each_column():
    # 32 x 16 tile, runs of eight values per column: values 8c .. 8c+7 lie in column c (c = 0..15).
    # Columns 0..14 hold 1024 and 1.5: column sum 1025.5, a tie between 1025 and 1026 -> 1026 (even).
    # Column 15 holds -8000 (= 4 * 2000, a binary16 number).
    # With the copy:    15 * 1026 - 8000 = 7390, a tie between 7388 = 4 * 1847 and 7392 = 4 * 1848 -> 7392.
    # Without the copy: 15 * 1025.5 - 8000 = 7382.5 -> 7384.       Exact sum: 7382.5.
    x = tile_values(512, [(8 * c, 1024.0) for c in range(15)] + [(8 * c + 1, 1.5) for c in range(15)] + [(120, -8000.0)])
    assert float(RM.recurrence(x, 1)) == 7392.0
    assert float(RM.kernel_mma(x, 1)[0]) == 7392.0
    # the same values in a 16 x 16 tile filled row by row: value v lies in column v mod 16, so column 0
    # gets the eight 1024s of even c (8192), column 1 their 1.5s (12), column 8 the seven 1024s of odd c
    # and -8000 (-832), column 9 seven 1.5s (10.5): all binary16 numbers, total 7382.5 -> 7384.
    assert float(RM.recurrence(x[:256], 1, shape=(16, 16), layout=RM.row_major)) == 7384.0


def test_store_into_the_fp16_array_rounds_the_group_total():
    # 2049 ones, R = 5: one group of 2560 values.  Every column sum is an integer below 2048 (exact in
    # binary16), the total 2049 is a tie between 2048 and 2050 -> 2048.  Without the final rounding: 2049.
    assert float(RM.recurrence(W.ones(2049), 5)) == 2048.0
    assert RM.kernel_mma(W.ones(2049), 5).size == 1
    # 2051 ones: tie between 2050 = 2 * 1025 and 2052 = 2 * 1026 -> 2052
    assert float(RM.recurrence(W.ones(2051), 5)) == 2052.0


def test_accumulator_is_binary32():
    # Column 0 holds 2048, 1 and 2^-20 (a binary16 subnormal).  The exact column sum 2049 + 2^-20 is not
    # a binary32 number (spacing 2^-12 there): C holds 2049, whose copy is a tie -> 2048.
    # An accumulator wider than binary32 would hand 2049.00000095 to the copy -> 2050.
    x = tile_values(512, [(0, 2048.0), (1, 1.0), (2, 2.0 ** -20)])
    assert float(RM.recurrence(x, 1)) == 2048.0
    # the same with the small value arriving in the second MMA of a chain (R = 2): C_1 = 2049 exactly,
    # C_2 = binary32(2049 + 2^-20) = 2049
    x = tile_values(1024, [(0, 2048.0), (1, 1.0), (512, 2.0 ** -20)])
    assert float(RM.recurrence(x, 2)) == 2048.0
    # the last MMA's result is binary32 too: 2048, 1 and 2^-20 in three different columns are copied
    # exactly, A x 1 = 2049 + 2^-20 is held as 2049, and the store rounds the tie to 2048 (a wider
    # result fragment would store 2050)
    x = tile_values(512, [(0, 2048.0), (8, 1.0), (16, 2.0 ** -20)])
    assert float(RM.recurrence(x, 1)) == 2048.0


def test_column_overflow_gives_infinity_although_the_sum_is_small():
    # column 0: 40000 + 40000 = 80000 > 65504 -> the copy is +inf; column 1: -60000.  Exact sum 20000.
    x = tile_values(512, [(0, 40000.0), (1, 40000.0), (8, -60000.0)])
    assert float(RM.recurrence(x, 1)) == math.inf
    # spread over two columns nothing overflows: 40000 + 40000 - 60000 = 20000 = 16 * 1250, exact
    x = tile_values(512, [(0, 40000.0), (16, 40000.0), (8, -60000.0)])
    assert float(RM.recurrence(x, 1)) == 20000.0


# ------------------------------------------------------------------- two levels, by hand ---

def test_two_levels_round_at_each_level():
    # R = 1, three groups of 512 values; each holds 2048 (column 0) and 1 (column 1): group total 2049,
    # stored as 2048.  Level 2 sees [2048, 2048, 2048] in column 0: 6144 = 4 * 1536, exact.
    # One rounding of the exact sum 6147 would give 6148.
    x = tile_values(3 * 512, [(512 * g, 2048.0) for g in range(3)] + [(512 * g + 8, 1.0) for g in range(3)])
    assert RM.levels_needed(x.size, 1) == 2
    assert [float(v) for v in RM.kernel_mma(x, 1)] == [2048.0, 2048.0, 2048.0]
    assert float(RM.recurrence(x, 1)) == 6144.0


def test_second_level_copy_rounding_decides():
    # R = 1, nine groups.  Groups 0..2 total 2050 each (exact), groups 3..7 are zero, group 8 totals -6000.
    # Level 2: values 0..7 share column 0 (sum 6150, a tie between 6148 = 4 * 1537 and 6152 = 4 * 1538
    # -> 6152), value 8 lies in column 1 (-6000).  6152 - 6000 = 152.  The exact sum is 150, and so is
    # the result if the level-2 copy did not round.
    x = tile_values(9 * 512, [(512 * g, 2050.0) for g in range(3)] + [(512 * 8, -6000.0)])
    assert [float(v) for v in RM.kernel_mma(x, 1)] == [2050.0] * 3 + [0.0] * 5 + [-6000.0]
    assert float(RM.recurrence(x, 1)) == 152.0


def test_head_padding_shifts_values_into_other_columns():
    # with 7 zeros before the first element, values 0 and 1 fall into runs 0 and 1, i.e. columns 0 and 1:
    # 1025.5 is no longer a column sum, nothing ties, the total 1025.5 is stored as 1026 by the final rounding
    x = tile_values(16, [(0, 1024.0), (1, 1.5)])
    assert float(RM.recurrence(x, 1, head=7)) == 1026.0
    assert float(RM.recurrence(x, 1, head=0)) == 1026.0      # same column: 1025.5 -> 1026 at the copy
    # a case where the padding changes the result: 2048, 1 and, eight places on, -2048 (exact sum 1).
    # head 0: values 0, 1 lie in column 0 (2049, a tie -> 2048) and value 8 in column 1 (-2048): total 0.
    # head 7: they sit at places 7, 8, 15: column 0 holds 2048, column 1 holds 1 - 2048 = -2047: total 1.
    x = tile_values(16, [(0, 2048.0), (1, 1.0), (8, -2048.0)])
    assert float(RM.recurrence(x, 1, head=0)) == 0.0
    assert float(RM.recurrence(x, 1, head=7)) == 1.0


# ------------------------------------------------------- exact cases, overflow, bounds ---

@pytest.mark.parametrize("R", [1, 2, 4, 5, 8])
def test_small_integer_inputs_are_exact(oracle_lib, R):
    # all partial sums are integers of magnitude <= 2048: every binary16 value is exact
    for n in (1, 2, 7, 511, 512, 513, 2047, 2048):
        assert float(RM.recurrence(W.ones(n), R)) == float(n)
    for n in (1, 100, 5000, 512 * R * 3 + 17):
        x = W.small_integers(n, seed=n + R, lo=-1, hi=1)
        if np.abs(x.astype(np.float64)).sum() <= 2048:
            assert float(RM.recurrence(x, R)) == oracle_lib.sum_f16(x)[0]
            assert float(RM.recurrence(x, R, shape=(16, 16), layout=RM.row_major)) == oracle_lib.sum_f16(x)[0]
    assert float(RM.recurrence(W.alternating(100000, 3.0), R)) == 0.0
    for head in range(8):
        x = W.small_integers(1500, seed=head, lo=-1, hi=1)
        assert float(RM.recurrence(x, R, head)) == oracle_lib.sum_f16(x)[0]


def test_layout_maps_are_bijections_with_the_stated_columns():
    for k, m in ((32, 16), (16, 16), (8, 4)):
        for layout in (RM.row_major, RM.runs_of_eight):
            assert sorted(layout(k, m).tolist()) == list(range(k * m))
    perm = RM.runs_of_eight(32, 16).reshape(32, 16)
    assert perm[:8, 0].tolist() == list(range(8))            # values 0..7: column 0, rows 0..7
    assert perm[:8, 15].tolist() == list(range(120, 128))    # values 120..127: column 15
    assert perm[8:16, 0].tolist() == list(range(128, 136))   # values 128..135: column 0 again, rows 8..15
    assert RM.row_major(16, 16).reshape(16, 16)[2, 5] == 37


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
    assert RM.levels_needed(256, 1, shape=(16, 16)) == 1 and RM.levels_needed(257, 1, shape=(16, 16)) == 2

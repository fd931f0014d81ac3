"""CPU model of the paper's Variant #1, "recurrence" (test infrastructure).

Algorithm 1 drives Algorithm 2 with the chained MMAs of Section 4.3; every
level stores one binary16 value per group of R * m^2 inputs.  The model takes
the algorithm's steps in the paper's order, for the matrix shape the GPU path
uses (B operand 32 x 16 per MMA: a group of R * 512 consecutive values, value
number v of the group lying in column (v // 8) mod 16):

    C_R      = sum_r 1 x M_r              the 16 column sums of the group
    A       <- C_R                        rounded to binary16 (the copy of C into
                                          an fp16 operand, Algorithm 2)
    C_{R+1}  = A x 1                      the sum of the 16 rounded column sums
    X'[g]    = binary16(C_{R+1}[0][0])    stored as binary16 (Algorithm 2, last line)

Sums inside a step are taken in binary64, where they are exact for binary16
inputs, so the only roundings are the two binary16 conversions above.  Nothing
here is shared with the HIP sources.
"""
from __future__ import annotations

import numpy as np


def level(values: np.ndarray, R: int, head: int = 0) -> np.ndarray:
    """One launch of KernelMMA: float16 array -> float16 array of group results.

    ``head`` zeros stand before the first value (groups are counted from a
    16-byte boundary at or before the first element)."""
    group = 512 * R
    v = np.asarray(values, dtype=np.float16)
    total = head + v.size
    groups = -(-total // group)
    padded = np.zeros(groups * group, dtype=np.float64)
    padded[head:head + v.size] = v.astype(np.float64)
    # (group, tile r, lane block of 16, column, 8 values per lane)
    cube = padded.reshape(groups, R, 4, 16, 8)
    with np.errstate(over="ignore", invalid="ignore"):
        C_R = cube.sum(axis=(1, 2, 4))                      # column sums, exact in binary64
        A = C_R.astype(np.float16)                          # copy of C into the fp16 operand
        C_last = A.astype(np.float64).sum(axis=1)           # A x 1
        return C_last.astype(np.float16)                    # stored as binary16


def recurrence(values: np.ndarray, R: int, head: int = 0) -> np.float32:
    """Algorithm 1: repeat until one value is left; returned as the fp32 the caller reads."""
    v = np.asarray(values, dtype=np.float16)
    if v.size == 0:
        return np.float32(0.0)
    v = level(v, R, head)
    while v.size > 1:
        v = level(v, R, 0)
    return np.float32(v[0])


def levels_needed(n: int, R: int, head: int = 0) -> int:
    group = 512 * R
    count = -(-(head + n) // group)
    k = 1
    while count > 1:
        count = -(-count // group)
        k += 1
    return k


def error_bound(sum_abs: float, n: int, R: int, head: int = 0) -> float:
    """First-order bound on |recurrence - exact sum| when nothing overflows: each level rounds
    the column sums and the group total to binary16 (relative 2^-11 each)."""
    return 2.0 * levels_needed(n, R, head) * 2.0 ** -11 * sum_abs * 1.01

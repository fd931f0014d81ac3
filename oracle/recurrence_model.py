"""CPU model of the paper's Variant #1, "recurrence" (test infrastructure).

Section 5.1 implements Algorithm 1 (the host loop) around Algorithm 2 (the
kernel) with the chained MMAs of Section 4.3.  For one group of R tiles
M_1 .. M_R the kernel takes these steps, which the model repeats in the same
order, with the precisions the paper names (Section 2.2: A and B hold
binary16, C and D hold binary32):

    C_0      = 0
    C_r      = 1 x M_r + C_{r-1},  r = 1..R     binary32 accumulator, rounded
                                                once per MMA
    A       <- C_R                               Algorithm 2's copy of C into
                                                the binary16 fragment A: rounds
    C_{R+1}  = A x 1 + 0                         binary32
    X'[g]    = C_{R+1}[0][0]                     written back into the binary16
                                                array: rounds again

and Algorithm 1 relaunches on X' until one value is left.

What the paper leaves open, and how it is read here:

* Shape of a tile.  The paper works with m x m fragments (m = 16).  The model
  takes any k x m tile (k rows, m columns, k*m consecutive values of X) and an
  explicit value -> (row, column) map, because with binary16 copies the result
  depends on which values share a column.  Two maps are provided:
  ``row_major(k, m)`` fills the tile row by row (value v at row v // m, column
  v mod m), the plain reading of "m^2 consecutive values are loaded into B";
  ``runs_of_eight(k, m)`` sends each run of eight consecutive values down one
  column (run q goes to column q mod m, rows 8 (q // m) .. 8 (q // m) + 7),
  which is the arrangement in which 64 lanes each load 16 contiguous bytes.
* Rounding inside one MMA.  The paper gives C as binary32 and nothing finer;
  the model forms 1 x M_r exactly and rounds once when it is added to C.
* Border.  Values past the end of X, and ``head`` values before its first
  element, are zeros (the text after Algorithm 2 leaves borders to the
  implementation).
* Algorithm 1's loop bound is read as "until one value is left".

Each step is written as the matrix product the paper prints; numpy's matmul is
the only library routine.  Nothing here is shared with the HIP sources.
"""
from __future__ import annotations

import numpy as np


def row_major(k: int, m: int) -> np.ndarray:
    """perm[row * m + col] = number (within the tile) of the value at (row, col)."""
    return np.arange(k * m, dtype=np.int64)


def runs_of_eight(k: int, m: int) -> np.ndarray:
    """Run q of eight consecutive values lies in column q mod m, rows 8 (q // m) + 0..7."""
    assert k % 8 == 0
    perm = np.empty(k * m, dtype=np.int64)
    for v in range(k * m):
        q, j = divmod(v, 8)
        row, col = 8 * (q // m) + j, q % m
        perm[row * m + col] = v
    return perm


# The tile the library's recurrence entry point is checked against: 32 x 16,
# runs of eight values per column (512 values per tile).
DEFAULT_SHAPE = (32, 16)


def kernel_mma(values: np.ndarray, R: int, head: int = 0, shape=DEFAULT_SHAPE, layout=runs_of_eight) -> np.ndarray:
    """One launch of Algorithm 2 with chains of R MMAs: binary16 array -> binary16 array, one value per group."""
    k, m = shape
    tile = k * m
    group = R * tile
    perm = layout(k, m)
    v = np.asarray(values, dtype=np.float16)
    total = head + v.size
    groups = -(-total // group)
    X = np.zeros(groups * group, dtype=np.float64)
    X[head:head + v.size] = v.astype(np.float64)
    M = X.reshape(groups, R, tile)[:, :, perm].reshape(groups, R, k, m)     # M[g, r] is the k x m tile M_{r+1} of group g
    ones_A = np.ones((m, k), dtype=np.float64)                                # the all-ones fragment A
    ones_B = np.ones((m, m), dtype=np.float64)                                # the all-ones fragment B of the last MMA
    with np.errstate(over="ignore", invalid="ignore"):
        C = np.zeros((groups, m, m), dtype=np.float32)                        # C_0 = 0
        for r in range(R):
            C = (ones_A @ M[:, r] + C.astype(np.float64)).astype(np.float32)  # C_r = 1 x M_r + C_{r-1}
        A = C.astype(np.float16)                                              # copyFromTo(C, A)
        C_last = (A.astype(np.float64) @ ones_B).astype(np.float32)           # C_{R+1} = A x 1 + 0
        return C_last[:, 0, 0].astype(np.float16)                             # X[offset / group] = C_{0,0}


def recurrence(values: np.ndarray, R: int, head: int = 0, shape=DEFAULT_SHAPE, layout=runs_of_eight) -> np.float32:
    """Algorithm 1: repeat the kernel until one value is left; returned as the binary32 the caller reads."""
    v = np.asarray(values, dtype=np.float16)
    if v.size == 0:
        return np.float32(0.0)
    v = kernel_mma(v, R, head, shape, layout)
    while v.size > 1:
        v = kernel_mma(v, R, 0, shape, layout)
    return np.float32(v[0])


def levels_needed(n: int, R: int, head: int = 0, shape=DEFAULT_SHAPE) -> int:
    group = R * shape[0] * shape[1]
    count = -(-(head + n) // group)
    levels = 1
    while count > 1:
        count = -(-count // group)
        levels += 1
    return levels


def error_bound(sum_abs: float, n: int, R: int, head: int = 0, shape=DEFAULT_SHAPE) -> float:
    """First-order bound on |recurrence - exact sum| when nothing overflows: each level rounds
    the column sums and the group total to binary16 (relative 2^-11 each)."""
    return 2.0 * levels_needed(n, R, head, shape) * 2.0 ** -11 * sum_abs * 1.01

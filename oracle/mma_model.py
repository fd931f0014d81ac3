"""fp64 model of the paper's ones-matrix MMA encoding (test infrastructure).

Written out in the paper's notation so that it can be checked against the text
by eye; numpy's matmul is the only library step.  Nothing here is blocked,
fused or reordered, and nothing is shared with the HIP sources.

* ``mma``            D = A x B + C                      (Section 4.1)
* ``two_step``       D = 1 x X + 0, then D' = D x 1 + 0 (eqs. MMA1, MMA2)
* ``chain``          C_r = 1 x M_r + C_{r-1}, r = 1..R, then C_{R+1} = C_R x 1
                     (Section 4.3)
* ``recurrence``     Algorithm 1 driving Algorithm 2 over a whole array, groups
                     of m^2 values, zero padding for the border (the text after
                     Algorithm 2 leaves border handling to the implementation)
* ``single_pass``    Variant #2 (Section 5.2): one chain of R MMAs per warp,
                     one value per block from its warps, all block values added
"""
from __future__ import annotations

import numpy as np


def ones(m: int) -> np.ndarray:
    return np.ones((m, m), dtype=np.float64)


def zeros(m: int) -> np.ndarray:
    return np.zeros((m, m), dtype=np.float64)


def mma(A: np.ndarray, B: np.ndarray, C: np.ndarray) -> np.ndarray:
    return A @ B + C


def load_matrix(x: np.ndarray, offset: int, m: int) -> np.ndarray:
    """m x m matrix B holding x[offset : offset + m^2], zero beyond the end."""
    g = np.zeros(m * m, dtype=np.float64)
    seg = np.asarray(x[offset:offset + m * m], dtype=np.float64)
    g[:seg.size] = seg
    return g.reshape(m, m)


def two_step(X: np.ndarray) -> np.ndarray:
    m = X.shape[0]
    D = mma(ones(m), X, zeros(m))        # eq. MMA1: partial sums, replicated
    Dp = mma(D, ones(m), zeros(m))       # eq. MMA2: the total, in every entry
    return Dp


def chain(tiles) -> np.ndarray:
    """tiles = [M_1 .. M_R]; returns C_{R+1} (the chain total in every entry)."""
    m = tiles[0].shape[0]
    C = zeros(m)                         # C_0
    for M_r in tiles:
        C = mma(ones(m), M_r, C)         # C_r = 1 x M_r + C_{r-1}
    return mma(C, ones(m), zeros(m))     # C_{R+1} = C_R x 1 + 0


def recurrence(x, m: int) -> float:
    """Algorithm 1: repeat KernelMMA until one group of m^2 values is left."""
    X = np.asarray(x, dtype=np.float64).copy()
    n = X.size
    if n == 0:
        return 0.0
    g = m * m
    while n > 1:                         # reading: loop until a single value remains
        groups = -(-n // g)
        Y = np.empty(groups, dtype=np.float64)
        for w in range(groups):          # one warp per group, offset = m^2 * w
            Y[w] = two_step(load_matrix(X[:n], g * w, m))[0, 0]
        X, n = Y, groups
    return float(X[0])


def single_pass(x, m: int, R: int, warps_per_block: int) -> float:
    """Variant #2: chains of R MMAs per warp, block combine, grid combine."""
    X = np.asarray(x, dtype=np.float64)
    n = X.size
    g = m * m
    per_warp = R * g
    warps = -(-n // per_warp) if n else 0
    blocks = -(-warps // warps_per_block) if warps else 0
    result = 0.0                         # the first global memory location
    for b in range(blocks):
        block_value = 0.0
        for w in range(b * warps_per_block, min((b + 1) * warps_per_block, warps)):
            tiles = [load_matrix(X, w * per_warp + r * g, m) for r in range(R)]
            block_value += chain(tiles)[0, 0]      # warp result, fp-wide partial
        result += block_value                      # one add per block
    return result

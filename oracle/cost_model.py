"""The paper's PRAM-like cost model (test infrastructure, documentation only).

Section 4.2: unit costs are 1 for a coalesced global read/write, 1 for an MMA,
1 for a transfer between global memory and fragments, and an order of magnitude
less for register / L1 operations.

* two-MMA reduction:      T_tc(n)   = 5 log_{m^2} n
* classic GPU reduction:  T(n)      = 4 log_2 n
* speedup:                S         = T / T_tc = (4/5) log_2 m^2
* chained (Section 4.3):  T_tc^R(n) = (2R + 3) log_{R m^2} n
"""
from __future__ import annotations

import math


def t_tensor_core(n: float, m: int) -> float:
    return 5.0 * math.log(n, m * m)


def t_classic(n: float) -> float:
    return 4.0 * math.log2(n)


def speedup(m: int) -> float:
    return 0.8 * math.log2(m * m)


def t_chained(n: float, m: int, R: int) -> float:
    return (2 * R + 3) * math.log(n, R * m * m)

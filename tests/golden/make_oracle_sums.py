#!/usr/bin/env python3
"""Writes tests/golden/oracle_sums.txt: the CPU oracle's (sum, sum |x|) for the
seeded workloads of the five configurations, at reduced and at full size.

Calls only ``oracle/`` (fp64 Kahan sum; definition R(X) = sum x_i, paper
Section 4) and the input generators.  Values are stored as C99 hex floats so
that they round-trip exactly.  Run from the repository root:

    python tests/golden/make_oracle_sums.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle                                              # noqa: E402
from paper_2001_05585_amd import workloads as W            # noqa: E402

CASES = [
    # (config, kind, n)
    (1, "uniform01", 1 << 20),
    (2, "uniform01", 1 << 22),
    (2, "uniform01", 1 << 26),
    (3, "normal", 1 << 22),
    (3, "normal", 1 << 28),
    (4, "uniform_pm1", 4_000_007),
    (4, "uniform_pm1", 400_000_000),
    (4, "uniform_pm1", 400_000_007),
    (5, "uniform01", (1 << 16) + 7),
    (5, "uniform01", 1 << 24),
    (5, "uniform01", (1 << 30) + 7),
]


def main():
    lines = ["# R(X) = sum_i x_i (paper Section 4, definition of the arithmetic reduction) and sum_i |x_i| of the seeded",
             "# fp16 workloads, as computed by the CPU oracle (fp64 Kahan); written by tests/golden/make_oracle_sums.py.",
             "# config kind n sum sum_abs   (C99 hex floats; seed = 20010558500 + config)"]
    for cfg, kind, n in CASES:
        x = W.generate(kind, n, W.config_seed(cfg))
        if n <= 1 << 26:
            s, sa = oracle.sum_f16(x)
        else:                       # same oracle over host threads (pinned to the exact sum in the CPU tests)
            s, sa, _ = oracle.sum_f16_blocked(x, os.cpu_count() or 1)
        lines.append("%d %s %d %s %s" % (cfg, kind, n, s.hex(), sa.hex()))
        print(lines[-1], flush=True)
        del x
    with open(os.path.join(ROOT, "tests", "golden", "oracle_sums.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()

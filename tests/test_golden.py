"""The stored oracle sums (tests/golden/oracle_sums.txt, written by
tests/golden/make_oracle_sums.py from ``oracle/`` alone) are reproduced by the
oracle and agree with the exact 128-bit integer sum: a regression pin for the
oracle and for the input generators.  Full-size rows are checked on the GPU machine
(tests/test_gpu_configs.py)."""
import math
import os

import pytest

from paper_2001_05585_amd import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))


def golden_rows():
    rows = []
    with open(os.path.join(HERE, "golden", "oracle_sums.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            cfg, kind, n, s, sa = line.split()
            rows.append((int(cfg), kind, int(n), float.fromhex(s), float.fromhex(sa)))
    return rows


def test_golden_file_covers_all_five_configs():
    assert sorted({r[0] for r in golden_rows()}) == [1, 2, 3, 4, 5]


@pytest.mark.parametrize("row", [r for r in golden_rows() if r[2] <= 1 << 23], ids=lambda r: "cfg%d-%d" % (r[0], r[2]))
def test_oracle_reproduces_golden(oracle_lib, row):
    cfg, kind, n, s, sa = row
    x = W.generate(kind, n, W.config_seed(cfg))
    got_s, got_sa = oracle_lib.sum_f16(x)
    assert got_s == s and got_sa == sa
    e, ea, bad = oracle_lib.exact_sum_f16(x)
    assert bad == 0
    assert abs(float(e) - s) <= 2 * math.ulp(s) and abs(float(ea) - sa) <= 2 * math.ulp(sa)

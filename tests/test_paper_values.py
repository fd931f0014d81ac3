"""The paper's printed figures for its cost model (tests/golden/paper_values.txt) against
oracle/cost_model.py."""
import math
import os

from oracle import cost_model as C

HERE = os.path.dirname(os.path.abspath(__file__))


def rows():
    out = []
    with open(os.path.join(HERE, "golden", "paper_values.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                q, arg, v = line.split()
                out.append((q, arg, float(v)))
    return out


def test_printed_values():
    seen = set()
    for q, arg, v in rows():
        seen.add(q)
        if q == "speedup":
            assert math.isclose(C.speedup(int(arg.split("=")[1])), v, rel_tol=1e-12)
        elif q == "t_tensor_core":
            for m in (2, 4, 16):
                assert math.isclose(C.t_tensor_core(m * m, m), v, rel_tol=1e-12)
        elif q == "t_chained_over_t_tensor_core":
            for m in (2, 4, 16):
                for n in (1e3, 1e6, 2.0 ** 28):
                    assert math.isclose(C.t_chained(n, m, 1) / C.t_tensor_core(n, m), v, rel_tol=1e-12)
    assert seen == {"speedup", "t_tensor_core", "t_chained_over_t_tensor_core"}


def test_speedup_is_the_ratio_of_the_two_running_times():
    for m in (2, 4, 16):
        for n in (1e4, 1e9):
            assert math.isclose(C.t_classic(n) / C.t_tensor_core(n, m), C.speedup(m), rel_tol=1e-12)
    # the recurrences themselves: T(n) = c + T(n / base)
    assert math.isclose(C.t_tensor_core(16.0 ** 5, 4), 5 + C.t_tensor_core(16.0 ** 4, 4))
    assert math.isclose(C.t_chained((3 * 16.0) ** 4, 4, 3), (2 * 3 + 3) + C.t_chained((3 * 16.0) ** 3, 4, 3))

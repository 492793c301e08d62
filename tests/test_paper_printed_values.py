"""The numbers the paper prints (tests/golden/paper_printed_values.txt, each with its passage) against the
oracle's headroom rule and the formulas of the cited passages."""
import math
import os

from oracle import gq_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def printed():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_printed_values.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        key, value, tol, where = [t.strip() for t in line.split("|", 3)]
        assert where.startswith(("Section", "Implementation section")), "every value carries its citation"
        out[key] = (float(value), float(tol))
    return out


def close(key, got, table):
    want, tol = table[key]
    assert abs(got - want) <= tol, (key, got, want)


def test_printed_values():
    t = printed()
    assert len(t) == 6
    # Section 4.2: each of the log2(n) reduce steps multiplies the second moment by at most 9/8
    close("variance_factor_n16", (9.0 / 8.0) ** math.log2(16), t)
    close("variance_factor_n1024", (9.0 / 8.0) ** math.log2(1024), t)
    # Theorem 1: theta_E = 1/(8n) + sqrt(d) / (sqrt(n) 2^(s-1)); Section 6 evaluates 1 + n^1.17 theta_E
    n, d, s = 16, 10 ** 6, 127
    theta_e = 1.0 / (8 * n) + math.sqrt(d) / (math.sqrt(n) * 2.0 ** (s - 1))
    close("iterations_factor_exp_example", 1.0 + n ** 1.17 * theta_e, t)
    # Section 4.2 / Implementation section headroom statements, from the oracle's rule n*s <= 2^(A-1) - 1
    close("linear_n16_A4_feasible_levels", sum(O.check_width(O.LINEAR, s_, 16, 4) for s_ in range(1, 64)), t)
    most = max(s_ for s_ in range(1, 16) if O.check_width(O.LINEAR, s_, 4, 4))
    close("linear_n4_A4_value_bits", math.log2(most + 1), t)
    # Section 4.2, the printed exponent-domain rule (it speaks about Algorithm 2's wire format, where exponents
    # up to s + log2(n) are stored next to a sign bit): largest s with 1 + log2(s + 1 + log2 n) <= A
    feasible = [s_ for s_ in range(1, 64) if 1 + math.log2(s_ + 1 + math.log2(16)) <= 4]
    close("exp_max_levels_n16_A4", max(feasible), t)

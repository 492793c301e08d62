"""Pins for the oracle's Algorithm 2 (arXiv 2305.18627, Section 4.3: reduce function for exponential
dithering).  Expected values come from exact rational arithmetic on the pairs (unbiased rounding of
x1 + x2 to one of its two neighbouring powers of two), from the law P(k > b) = 2^-b, from the 9/8
variance factor and the numbers the paper prints for it, and from the exact integer sum that the
reduce function must reproduce in expectation."""
from fractions import Fraction
import math

import numpy as np
import pytest

from oracle import gq_oracle as O


def val(sign, e):
    return Fraction(0) if e == 0 else Fraction(sign) / (1 << e)


def k_weights():
    """P(k = j) for the 32-bit draw: 2^-j for j = 1..32, and the all-zero word gives 33."""
    w = {j: Fraction(1, 1 << j) for j in range(1, 33)}
    w[33] = Fraction(1, 1 << 32)
    return w


def test_k_has_the_law_of_algorithm_2():
    # P(k > b) = 2^-b: exactly the words below 2^(32-b) give k > b
    for b in range(0, 33):
        lim = 1 << (32 - b)
        assert O.alg2_k(lim - 1) > b
        if lim < (1 << 32):
            assert O.alg2_k(lim) <= b
    rng = np.random.default_rng(0)
    r = np.sort(rng.integers(0, 1 << 32, 5000, dtype=np.uint64))
    ks = [O.alg2_k(int(v)) for v in r]
    assert all(a >= b for a, b in zip(ks[:-1], ks[1:]))             # monotone: fewer leading zeros, smaller k
    assert sum(k_weights().values()) == 1


def neighbours(x):
    """The powers of two 2^-a <= |x| <= 2^-(a-1) around a non-zero |x| < 1 (equal if |x| is one)."""
    ax = abs(x)
    a = 0
    while Fraction(1, 1 << a) > ax:
        a += 1
    low = Fraction(1, 1 << a)
    return (low, low) if low == ax else (low, 2 * low)


def test_reduce_pair_is_the_unbiased_rounding_of_the_sum_to_a_power_of_two():
    W = k_weights()
    worst = Fraction(0)
    for s1 in (1, -1):
        for s2 in (1, -1):
            for e1 in range(0, 13):
                for e2 in range(0, 13):
                    x = val(s1, e1) + val(s2, e2)
                    if abs(x) > Fraction(1, 2):
                        continue        # the 1/(2n) prescale keeps every partial sum within 1/2 (Section 4.3)
                    mean = Fraction(0); second = Fraction(0)
                    for k, w in W.items():
                        sr, er = O.exp_reduce_pair(s1, e1, s2, e2, k)
                        assert sr in (1, -1) and er >= 0
                        y = val(sr, er)
                        if x == 0:
                            assert er == 0
                        else:
                            low, up = neighbours(x)
                            assert abs(y) in (low, up) and (y > 0) == (x > 0)
                        mean += w * y; second += w * y * y
                    assert mean == x                             # E[C(x1 + x2)] = x1 + x2, exactly
                    if x != 0:
                        worst = max(worst, second / (x * x))
    # the rounding adds at most a factor 9/8 to the second moment (the paper's per-step factor; 9/8 itself
    # needs x = 4/3 * 2^a, which no sum of two powers of two hits: the worst such sum gives 28/25)
    assert Fraction(11, 10) < worst <= Fraction(9, 8)


def test_reduce_pair_case_by_case():
    # same sign, e1 <= e2: up to 2^-(e1-1) iff k > e2 - e1
    assert O.exp_reduce_pair(1, 3, 1, 5, 3) == (1, 2) and O.exp_reduce_pair(1, 3, 1, 5, 2) == (1, 3)
    assert O.exp_reduce_pair(-1, 5, -1, 3, 3) == (-1, 2) and O.exp_reduce_pair(-1, 5, -1, 3, 2) == (-1, 3)
    # equal exponents, same sign: exactly the next power of two, whatever k
    assert all(O.exp_reduce_pair(1, 4, 1, 4, k) == (1, 3) for k in range(1, 34))
    # opposite signs: equal exponents cancel; otherwise down to 2^-(e1+1) iff k > e2 - e1 - 1
    assert all(O.exp_reduce_pair(1, 4, -1, 4, k)[1] == 0 for k in range(1, 34))
    assert all(O.exp_reduce_pair(1, 3, -1, 4, k) == (1, 4) for k in range(1, 34))      # 1/8 - 1/16 = 1/16 exactly
    assert O.exp_reduce_pair(1, 3, -1, 5, 2) == (1, 4) and O.exp_reduce_pair(1, 3, -1, 5, 1) == (1, 3)
    assert O.exp_reduce_pair(-1, 6, 1, 3, 3) == (1, 4) and O.exp_reduce_pair(-1, 6, 1, 3, 2) == (1, 3)
    # zeros pass the other operand through
    assert O.exp_reduce_pair(1, 0, -1, 7, 1) == (-1, 7) and O.exp_reduce_pair(-1, 7, 1, 0, 1) == (-1, 7)
    assert O.exp_reduce_pair(-1, 0, 1, 0, 5)[1] == 0


def test_numbers_the_paper_prints_for_the_variance_growth():
    # Section 4.2: (9/8)^(log n) <= n^0.17; 1.6x for n = 16 and 3.25x for n = 1024
    assert (9 / 8) ** 4 == pytest.approx(1.6, abs=0.005)
    assert (9 / 8) ** 10 == pytest.approx(3.25, abs=0.005)
    for logn in range(1, 21):
        assert (9 / 8) ** logn <= (2 ** logn) ** 0.17


def test_tree_reduce_small_cases_by_hand():
    # s = 3, two workers both at the top level 1: each becomes 1/(2*2) = 2^-2; the sum 2^-1 is exact;
    # it stands for the mean 2^-1 * 4 / 2 = 1
    se = O.exp_tree_reduce([[3], [3]], 3, seed=1)
    assert se.tolist() == [1] and O.exp_reduce_dequantize(se, 1.0, 2).tolist() == [1.0]
    # one worker: only the change of representation, e = s - k + 1
    se = O.exp_tree_reduce([[0, 1, -2, 3]], 3, seed=1)
    assert se.tolist() == [0, 3, -2, 1]
    assert O.exp_reduce_dequantize(se, 8.0, 1).tolist() == [0.0, 2.0, -4.0, 8.0]       # 8 * 2^(k-3)
    # K = 2^L equal codes of one sign add up exactly: the result stands for the common level
    for K in (2, 4, 8, 16):
        for k in (1, 2, 5):
            se = O.exp_tree_reduce([[-k, k]] * K, 5, seed=3)
            assert np.array_equal(O.exp_reduce_dequantize(se, 1.0, K), [-(2.0 ** (k - 5)), 2.0 ** (k - 5)])
    # three workers are padded with a zero leaf: (a + b) + (c + 0); opposite equal levels cancel
    se = O.exp_tree_reduce([[2], [-2], [4]], 4, seed=9)          # L = 2: e(4) = 4 - 4 + 1 + 2 = 3
    assert se.tolist() == [3] and O.exp_reduce_dequantize(se, 3.0, 3).tolist() == [3.0 * 2.0 ** (1 + 2 - 3) / 3]
    # composition: a two-worker reduce is one call of the pair function with the word of node 1, stream 1
    for g in (0, 5, 4 * (2 ** 32) + 2):
        r = O.random_word_of(77, 1, 1, g)
        sr, er = O.exp_reduce_pair(1, 5 - 4 + 1 + 1, -1, 5 - 2 + 1 + 1, O.alg2_k(r))
        assert O.exp_tree_reduce([[4], [-2]], 5, seed=77, index_base=g).tolist() == [sr * er]
    assert O.random_word_of(77, 0, 0, 123) == int(O.random_words(77, 0, 123, 1)[0])


@pytest.mark.parametrize("K,s", [(2, 7), (4, 7), (8, 16), (16, 7), (5, 9)])
def test_tree_reduce_reproduces_the_exact_sum_in_expectation(K, s):
    rng = np.random.default_rng(K * 100 + s)
    d, T = 256, 3000
    qs = [rng.integers(-s, s + 1, d).astype(np.int32) for _ in range(K)]
    for q in qs:
        q[rng.random(d) < 0.3] = 0
    exact = O.dequantize(O.aggregate(qs, O.EXP), 1.0, O.EXP, s, K)     # the integer-sum path
    L = math.ceil(math.log2(K))
    acc = np.zeros(d); acc2 = np.zeros(d)
    for t in range(T):
        se = O.exp_tree_reduce(qs, s, seed=5000 + t)
        assert np.abs(se).max() <= s + L and np.all((se == 0) | (np.abs(se) >= 1))
        g = O.exp_reduce_dequantize(se, 1.0, K)
        acc += g; acc2 += g * g
    mean = acc / T
    sd = np.sqrt(np.maximum(acc2 / T - mean * mean, 0.0))
    assert np.all(np.abs(mean - exact) <= 5.0 * sd / np.sqrt(T) + 1e-12)
    # the reduction's own second moment stays within (9/8)^L of the squared leaf sum bound:
    # E[g^2] <= (9/8)^L * (sum_i |x_i| / K)^2 holds per coordinate for the worst case of equal signs
    bound = (9 / 8) ** L * (O.dequantize(O.aggregate([np.abs(q) for q in qs], O.EXP), 1.0, O.EXP, s, K)) ** 2
    assert np.all(acc2 / T <= bound * 1.05 + 1e-12)              # 5 % for the Monte Carlo noise at T = 3000
    # buckets: the reduce of a slice with its offset equals the slice of the whole
    whole = O.exp_tree_reduce(qs, s, seed=42)
    part = O.exp_tree_reduce([q[100:200] for q in qs], s, seed=42, index_base=100)
    assert np.array_equal(part, whole[100:200])

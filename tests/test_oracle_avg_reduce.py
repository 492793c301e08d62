"""Pins for the oracle's in-step averaging of low-bit linear codes (arXiv 2305.18627, Implementation section:
the average is taken inside every reduce step so that 4-bit codes do not overflow).  Expected values
are exact rational means, ranges, and the headroom statement the section opens with."""
from fractions import Fraction
import itertools
import math

import numpy as np
import pytest

from oracle import gq_oracle as O


def test_pair_is_the_unbiased_rounding_of_the_average():
    for a in range(-15, 16):
        for b in range(-15, 16):
            lo, hi = O.avg_pair(a, b, 0), O.avg_pair(a, b, 1)
            assert lo == math.floor((a + b) / 2) and hi == math.ceil((a + b) / 2)
            assert Fraction(lo + hi, 2) == Fraction(a + b, 2)            # a fair coin gives the exact average
            assert min(a, b) <= lo <= hi <= max(a, b)                    # never leaves the range of the inputs


def test_section7_headroom_statement_and_what_averaging_buys():
    # 4-bit linear, 4 workers: summing leaves a single value bit (s = 1) ...
    assert O.check_width(O.LINEAR, 1, 4, 4) and not O.check_width(O.LINEAR, 2, 4, 4)
    # ... while the averaged tree keeps s = 7 inside a signed nibble for any number of workers
    rng = np.random.default_rng(0)
    for K in (4, 16, 64):
        qs = [rng.integers(-7, 8, 500).astype(np.int32) for _ in range(K)]
        qs[0][:] = 7; qs[1][:] = 7
        out = O.avg_tree_reduce(qs, seed=1)
        assert np.abs(out).max() <= 7
        O.pack(out, O.PACK_I4)                                           # fits, or this raises


def test_tree_by_hand_and_exact_expectation_over_all_coins():
    # K = 1: identity; equal codes stay; two workers: one node
    assert O.avg_tree_reduce([[3, -2, 0]], seed=5).tolist() == [3, -2, 0]
    assert O.avg_tree_reduce([[5, -5]] * 8, seed=5).tolist() == [5, -5]
    assert O.avg_tree_reduce([[4], [2]], seed=5).tolist() == [3]
    assert O.avg_tree_reduce([[4], [3]], seed=5).tolist()[0] in (3, 4)
    # three workers are padded with a zero: ((a+b)/2 + (c+0)/2)/2
    assert O.avg_tree_reduce([[4], [4], [8]], seed=5).tolist() == [4]
    # norm 2, s = 8: the three workers hold 2*4/8 = 1, 1 and 2*8/8 = 2, whose mean is 4/3
    assert O.avg_reduce_dequantize([4], 2.0, 8, 3)[0] == pytest.approx(4.0 / 3.0, rel=1e-15)
    # the coin of node h at coordinate g is bit h of the stream-2 word: K = 2 uses node 1, i.e. bit 1
    for g in (0, 3, 17, 4 * (2 ** 32) + 1):
        r = O.random_word_of(99, 0, 2, g)
        assert O.avg_tree_reduce([[4], [3]], seed=99, index_base=g).tolist() == [O.avg_pair(4, 3, (r >> 1) & 1)]
    # exact expectation: enumerate the three coins of a 4-leaf tree by hand and average
    rng = np.random.default_rng(3)
    for _ in range(50):
        a, b, c, d4 = (int(v) for v in rng.integers(-7, 8, 4))
        tot = Fraction(0)
        for c2, c3, c1 in itertools.product((0, 1), repeat=3):           # nodes 2, 3 (children), 1 (root)
            tot += Fraction(O.avg_pair(O.avg_pair(a, b, c2), O.avg_pair(c, d4, c3), c1), 8)
        assert tot == Fraction(a + b + c + d4, 4)


@pytest.mark.parametrize("K,s", [(4, 7), (16, 7), (5, 15), (64, 7), (32, 127)])
def test_monte_carlo_mean_is_the_exact_mean(K, s):
    rng = np.random.default_rng(K + s)
    d, T = 256, 3000
    qs = [rng.integers(-s, s + 1, d).astype(np.int32) for _ in range(K)]
    exact = np.sum(np.stack(qs), axis=0) / K                            # mean code over the K workers
    npad = 1 << math.ceil(math.log2(K))
    acc = np.zeros(d); acc2 = np.zeros(d)
    for t in range(T):
        out = O.avg_tree_reduce(qs, seed=7000 + t)
        assert np.abs(out).max() <= s
        g = O.avg_reduce_dequantize(out, float(s), s, K)                 # norm = s: the mean in code units
        acc += g; acc2 += g * g
    mean = acc / T
    sd = np.sqrt(np.maximum(acc2 / T - mean * mean, 0.0))
    assert np.all(np.abs(mean - exact) <= 5.0 * sd / np.sqrt(T) + 1e-12)
    # each step adds at most 1/4 of variance in its own units: in all less than 1/3 code unit^2 at the root
    assert np.all(acc2 / T - mean * mean <= (1.0 / 3.0) * (npad / K) ** 2 * 1.1 + 1e-12)
    # buckets with their offsets reproduce the whole
    whole = O.avg_tree_reduce(qs, seed=42)
    assert np.array_equal(O.avg_tree_reduce([q[64:200] for q in qs], seed=42, index_base=64), whole[64:200])
    # the coins of different nodes are different bits: across coordinates the results are not all equal
    odd = [np.full(4096, 1, np.int32), np.zeros(4096, np.int32)]
    r = O.avg_tree_reduce(odd, seed=1)
    assert 0.45 < r.mean() < 0.55

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


def k_weights(s):
    """P(k = j) of Algorithm 2's first statement with m = s + 1: 2^-j for j = 1..s, and 2^-s for the cap k = m."""
    w = {j: Fraction(1, 1 << j) for j in range(1, s + 1)}
    w[s + 1] = Fraction(1, 1 << s)
    return w


def k_by_the_printed_formula(r, s):
    """k = -floor(log2(2^-m + [p - 2^-m]_+)), m = s + 1, p = r / 2^s, in exact rational arithmetic."""
    m = s + 1
    p = Fraction(r, 1 << s)
    q = Fraction(1, 1 << m) + max(Fraction(0), p - Fraction(1, 1 << m))
    fl = 0                                   # floor(log2 q) for 0 < q < 1: the largest fl with 2^fl <= q
    while Fraction(1, 1 << (-fl)) > q:
        fl -= 1
    return -fl


@pytest.mark.parametrize("s", [1, 2, 3, 7, 8, 9, 12, 16])
def test_k_has_the_law_of_algorithm_2(s):
    # over ALL 2^s values of the s-bit draw: P(k > b) = 2^-b for b < m, P(k = m) = 2^-(m-1), support 1..m,
    # and the value is the printed formula's
    m = s + 1
    ks = np.array([O.alg2_k(r, s) for r in range(1 << s)])
    assert ks.min() == 1 and ks.max() == m
    for b in range(0, m):
        assert int((ks > b).sum()) * (1 << b) == (1 << s)
    assert int((ks > m).sum()) == 0 and int((ks == m).sum()) == 1 and ks[0] == m        # 2^-s = 2^-(m-1)
    assert all(ks[r] == k_by_the_printed_formula(r, s) for r in (list(range(min(1 << s, 300))) + [(1 << s) - 1, 1 << (s - 1)]))
    assert np.all(np.diff(ks) <= 0)                                  # a larger p never gives a larger k
    assert sum(k_weights(s).values()) == 1


def test_k_with_wide_draws():
    # s up to 31 (32-bit fields): thresholds of the law instead of an enumeration
    for s in (17, 24, 31):
        m = s + 1
        assert O.alg2_k(0, s) == m and O.alg2_k((1 << s) - 1, s) == 1
        for b in range(0, s + 1):
            lim = 1 << (s - b)                                       # k > b  <=>  r < 2^(s-b)
            assert O.alg2_k(lim - 1, s) > b
            if lim < (1 << s):
                assert O.alg2_k(lim, s) <= b


def test_a_nodes_random_bits_are_the_top_of_its_field_of_the_philox_block():
    # W = 8 / 16 / 32 bits per (node, coordinate): counter (lo32(g/4), hi32(g/4), node / (32/W), 1), word g mod 4,
    # field node mod (32/W) from the low end; the draw is the field's top s bits
    seed = 0x1234567887654321
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for s in (1, 5, 7, 8, 9, 13, 16, 17, 31):
        W = O.alg2_field_bits(s)
        assert W == (8 if s <= 8 else 16 if s <= 16 else 32)
        per = 32 // W
        for node in (1, 2, 3, 4, 5, 31, 32, 63):
            for g in (0, 1, 2, 3, 4, 7, 4 * (1 << 32) + 2, (1 << 40) + 3):
                call = g // 4
                block = O.philox4x32([call & 0xFFFFFFFF, call >> 32, node // per, 1], key)
                field = (int(block[g % 4]) >> (W * (node % per))) & ((1 << W) - 1)
                assert O.alg2_draw(seed, node, g, s) == field >> (W - s)
    # the draws of the nodes that share a call are disjoint fields of the same word, so distinct nodes round
    # independently: with s = 8 the four draws of nodes 4..7 are the four bytes of one word
    g = 12345
    word = O.random_word_of(seed, 1, 1, g)
    assert [O.alg2_draw(seed, 4 + i, g, 8) for i in range(4)] == [(word >> (8 * i)) & 255 for i in range(4)]


def neighbours(x):
    """The powers of two 2^-a <= |x| <= 2^-(a-1) around a non-zero |x| < 1 (equal if |x| is one)."""
    ax = abs(x)
    a = 0
    while Fraction(1, 1 << a) > ax:
        a += 1
    low = Fraction(1, 1 << a)
    return (low, low) if low == ax else (low, 2 * low)


@pytest.mark.parametrize("s", [2, 3, 7, 11])
def test_reduce_pair_is_the_unbiased_rounding_of_the_sum_to_a_power_of_two(s):
    # Exact rational expectation over the law of k (m = s + 1).  Finding recorded here: the pair reduction is
    # EXACTLY unbiased as long as the gap between the exponents stays below m (same signs) resp. m + 1
    # (opposite signs) -- which covers every pair of leaves, whose gap is at most s - 1 -- and beyond that the
    # cap on k makes the result deterministic: the larger operand, the smaller one being dropped, an error of
    # at most 2^-(s+1) relative to the sum's larger operand.
    W = k_weights(s)
    m = s + 1
    worst = Fraction(0)
    emax = s + 6                                                   # exponents up to s + log2(64)
    dropped = 0
    for s1 in (1, -1):
        for s2 in (1, -1):
            for e1 in range(0, emax + 1):
                for e2 in range(0, emax + 1):
                    x = val(s1, e1) + val(s2, e2)
                    if abs(x) > Fraction(1, 2):
                        continue        # the 1/(2n) prescale keeps every partial sum within 1/2 (Section 4.3)
                    mean = Fraction(0); second = Fraction(0)
                    outcomes = set()
                    for k, w in W.items():
                        sr, er = O.exp_reduce_pair(s1, e1, s2, e2, k)
                        assert sr in (1, -1) and er >= 0
                        y = val(sr, er)
                        outcomes.add(y)
                        if x == 0:
                            assert er == 0
                        else:
                            low, up = neighbours(x)
                            assert abs(y) in (low, up) and (y > 0) == (x > 0)
                        mean += w * y; second += w * y * y
                    gap = abs(e1 - e2)
                    same = s1 == s2
                    exact = e1 == 0 or e2 == 0 or (gap < m if same else gap < m + 1)
                    if exact:
                        assert mean == x                         # E[C(x1 + x2)] = x1 + x2, exactly
                        if x != 0:
                            worst = max(worst, second / (x * x))
                    else:
                        big = val(s1, e1) if e1 < e2 else val(s2, e2)
                        small = x - big
                        assert outcomes == {big} and mean - x == -small
                        assert abs(small) <= abs(big) / (1 << m)
                        dropped += 1
    assert dropped > 0
    # the rounding adds at most a factor 9/8 to the second moment (the paper's per-step factor; 9/8 itself
    # needs x = 4/3 * 2^a, which no sum of two powers of two hits: the worst such sum gives 28/25)
    assert Fraction(11, 10) < worst <= Fraction(9, 8)


def test_small_trees_have_the_exact_expectation():
    # four leaves, s = 3 (m = 4): the expectation of the root over the law of k at the three nodes, in exact
    # rational arithmetic, composed from the pair function in heap order.  Every gap here stays below m, so
    # the tree is exactly unbiased for the sum of its leaves.
    s, L = 3, 2
    W = k_weights(s)
    rng = np.random.default_rng(4)
    for _ in range(40):
        codes = [int(c) for c in rng.integers(-s, s + 1, 4)]
        leaves = [((-1 if c < 0 else 1), (s - abs(c) + 1 + L) if c else 0) for c in codes]
        total = sum(val(sg, e) for sg, e in leaves)
        mean = Fraction(0)
        for k2, w2 in W.items():
            for k3, w3 in W.items():
                a = O.exp_reduce_pair(*leaves[0], *leaves[1], k2)
                b = O.exp_reduce_pair(*leaves[2], *leaves[3], k3)
                for k1, w1 in W.items():
                    mean += w1 * w2 * w3 * val(*O.exp_reduce_pair(*a, *b, k1))
        assert mean == total


def test_reduce_pair_case_by_case():
    # same sign, e1 <= e2: up to 2^-(e1-1) iff k > e2 - e1
    assert O.exp_reduce_pair(1, 3, 1, 5, 3) == (1, 2) and O.exp_reduce_pair(1, 3, 1, 5, 2) == (1, 3)
    assert O.exp_reduce_pair(-1, 5, -1, 3, 3) == (-1, 2) and O.exp_reduce_pair(-1, 5, -1, 3, 2) == (-1, 3)
    # equal exponents, same sign: exactly the next power of two, whatever k
    assert all(O.exp_reduce_pair(1, 4, 1, 4, k) == (1, 3) for k in range(1, 9))
    # opposite signs: equal exponents cancel; otherwise down to 2^-(e1+1) iff k > e2 - e1 - 1
    assert all(O.exp_reduce_pair(1, 4, -1, 4, k)[1] == 0 for k in range(1, 9))
    assert all(O.exp_reduce_pair(1, 3, -1, 4, k) == (1, 4) for k in range(1, 9))      # 1/8 - 1/16 = 1/16 exactly
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
    # composition: a two-worker reduce is one call of the pair function with the draw of node 1
    for g in (0, 5, 4 * (2 ** 32) + 2):
        sr, er = O.exp_reduce_pair(1, 5 - 4 + 1 + 1, -1, 5 - 2 + 1 + 1, O.alg2_k(O.alg2_draw(77, 1, g, 5), 5))
        assert O.exp_tree_reduce([[4], [-2]], 5, seed=77, index_base=g).tolist() == [sr * er]
    assert O.random_word_of(77, 0, 0, 123) == int(O.random_words(77, 0, 123, 1)[0])


@pytest.mark.parametrize("K,s", [(3, 4), (5, 7), (8, 12), (13, 20)])
def test_tree_reduce_is_the_pair_function_applied_in_heap_order(K, s):
    # the tree function against its own definition composed here: leaves n' + i (missing workers are zeros),
    # node h = pair(child 2h, child 2h + 1) with the draw of node h, root 1
    rng = np.random.default_rng(K + s)
    d, base, seed = 97, 4 * 1001, 31
    qs = [rng.integers(-s, s + 1, d).astype(np.int32) for _ in range(K)]
    L = math.ceil(math.log2(K)); npad = 1 << L
    got = O.exp_tree_reduce(qs, s, seed=seed, index_base=base)
    for j in range(d):
        node = {}
        for i in range(npad):
            c = int(qs[i][j]) if i < K else 0
            node[npad + i] = ((-1 if c < 0 else 1), (s - abs(c) + 1 + L) if c else 0)
        for h in range(npad - 1, 0, -1):
            k = O.alg2_k(O.alg2_draw(seed, h, base + j, s), s)
            node[h] = O.exp_reduce_pair(*node[2 * h], *node[2 * h + 1], k)
        sg, e = node[1]
        assert got[j] == (sg * e if e else 0)


def root_distribution(codes, s):
    """Exact law of the root of Algorithm 2's tree over the K codes of one coordinate: {(sign, e): probability},
    by propagating the laws of the nodes upwards with the pair function and the law of k."""
    K = len(codes)
    L = math.ceil(math.log2(K)) if K > 1 else 0
    npad = 1 << L
    W = k_weights(s)
    dist = {}
    for i in range(npad):
        c = int(codes[i]) if i < K else 0
        dist[npad + i] = {((-1 if c < 0 else 1), (s - abs(c) + 1 + L) if c else 0): Fraction(1)}
    for h in range(npad - 1, 0, -1):
        out = {}
        for a, pa in dist[2 * h].items():
            for b, pb in dist[2 * h + 1].items():
                t = abs(a[1] - b[1]) - (0 if a[0] == b[0] else 1)
                # the result depends on k only through k > t: two calls cover the whole law
                p_gt = sum(w for k, w in W.items() if k > t)
                for k, w in ((s + 1, p_gt), (min(max(t, 1), s + 1) if t >= 1 else None, 1 - p_gt)):
                    if w == 0 or k is None:
                        continue
                    assert (k > t) == (w is p_gt) or p_gt in (0, 1)
                    r = O.exp_reduce_pair(a[0], a[1], b[0], b[1], k)
                    r = (1, 0) if r[1] == 0 else r
                    out[r] = out.get(r, Fraction(0)) + pa * pb * w
        dist[h] = out
    return dist[1], L


@pytest.mark.parametrize("K,s", [(2, 7), (4, 3), (8, 16), (16, 7), (5, 9), (3, 2)])
def test_tree_reduce_has_the_exact_sum_as_its_exact_expectation(K, s):
    # the whole tree in exact rational arithmetic: E[root] equals the sum of the prescaled leaves whenever no
    # pair can reach the gap at which the cap on k drops the smaller operand (m same signs, m + 1 opposite);
    # where one can, the error is at most 2^-(s+1) of the leaves' absolute sum per tree level.  The second
    # moment stays within (9/8)^L of the squared absolute sum (the paper's factor per aggregation step).
    rng = np.random.default_rng(K * 10 + s)
    cases = [rng.integers(-s, s + 1, K) for _ in range(12)]
    cases.append(np.array(([s, -s, 1, s, 0, -2, 0, -3] * 8)[:K]))       # a large cancellation beside small values
    cases.append(np.array(([1, s] * 32)[:K]))
    exact_cases = 0
    for codes in cases:
        law, L = root_distribution(codes, s)
        assert sum(law.values()) == 1
        leaves = [Fraction((-1 if c < 0 else 1) * (1 << (abs(int(c)) - 1)), 1 << (s + L)) if c else Fraction(0) for c in codes]
        total, abs_total = sum(leaves), sum(abs(v) for v in leaves)
        mean = sum(p * val(sg, e) for (sg, e), p in law.items())
        second = sum(p * val(sg, e) ** 2 for (sg, e), p in law.items())
        # a gap of m or more needs exponents s + 1 apart: impossible when s + L - 1 < m, i.e. L < 2
        if L < 2:
            assert mean == total
            exact_cases += 1
        else:
            assert abs(mean - total) <= L * abs_total / (1 << (s + 1))
            exact_cases += mean == total
        assert second <= Fraction(9, 8) ** L * abs_total ** 2
        assert all(e == 0 or 1 <= e <= s + L for (_, e) in law)
    assert exact_cases >= len(cases) // 2                               # the cap only bites in rare configurations


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
    # E[g^2] <= (9/8)^L * (sum_i |x_i| / K)^2 per coordinate (the paper's factor per aggregation step), which also
    # bounds the standard deviation.  The sample deviation cannot be used for the test of the mean: a coordinate
    # with a large cancellation beside small values is rounded away from its usual value with a probability far
    # below 1/T and by a large amount, so its sample deviation is 0 while its true one is not.
    bound = (9 / 8) ** L * (O.dequantize(O.aggregate([np.abs(q) for q in qs], O.EXP), 1.0, O.EXP, s, K)) ** 2
    assert np.all(np.abs(mean - exact) <= 5.0 * np.sqrt(bound / T) + 1e-12)
    # (the exact expectation of the tree is pinned above in rational arithmetic; this is the end-to-end check
    #  of the same fact through the random stream)
    assert np.all(acc2 / T <= bound * 1.05 + 1e-12)              # 5 % for the Monte Carlo noise at T = 3000
    # buckets: the reduce of a slice with its offset equals the slice of the whole
    whole = O.exp_tree_reduce(qs, s, seed=42)
    part = O.exp_tree_reduce([q[100:200] for q in qs], s, seed=42, index_base=100)
    assert np.array_equal(part, whole[100:200])

"""Pins for the oracle's random rounding (arXiv 2305.18627, Definition 1, Eq. (1)-(2), the linear
and exponential grids of Section 4.2) and for the whole quantize -> sum -> dequantize chain.

Expected values come from exact rational arithmetic on the inputs (fractions.Fraction), from
counting over the random word, from the two-point-distribution closed form for the variance and
from the paper's Theorem 1 bound -- never from the oracle's own formulas.
"""
from fractions import Fraction
import itertools
import math

import numpy as np
import pytest

from oracle import gq_oracle as O

F32 = np.float32
TWO32 = 1 << 32


def count_up(scheme, x, norm, s, k_up):
    """Number of 32-bit random words for which the oracle returns magnitude k_up, found by bisection.
    Linear: 'up' holds for small words (monotone decreasing); exponential: for large words."""
    mag = lambda r: abs(O.code(scheme, x, norm, s, r))
    if scheme == O.LINEAR:
        if mag(0) != k_up:
            return 0
        if mag(TWO32 - 1) == k_up:
            return TWO32
        lo, hi = 0, TWO32 - 1                       # mag(lo) == k_up, mag(hi) != k_up
        while hi - lo > 1:
            mid = (lo + hi) // 2
            if mag(mid) == k_up: lo = mid
            else: hi = mid
        return hi
    if mag(TWO32 - 1) != k_up:
        return 0
    if mag(0) == k_up:
        return TWO32
    lo, hi = 0, TWO32 - 1                           # mag(lo) != k_up, mag(hi) == k_up
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if mag(mid) == k_up: hi = mid
        else: lo = mid
    return TWO32 - hi


def sample_words(n, seed):
    rng = np.random.default_rng(seed)
    r = rng.integers(0, TWO32, n, dtype=np.uint64).astype(np.uint32)
    r[:4] = [0, 1, TWO32 - 1, TWO32 - 2]
    return np.sort(r)


def exact_linear(x, norm, s):
    """(h, frac) of t = |x|/norm * s in exact arithmetic."""
    t = abs(Fraction(float(F32(x)))) / Fraction(float(F32(norm))) * s
    h = math.floor(t)
    return h, t - h


def exact_exp(x, norm, s):
    """(k_low, P(up)) on the grid {0} u {2^-j}: codes k stand for 2^(k-s)."""
    y = abs(Fraction(float(F32(x)))) / Fraction(float(F32(norm)))
    smallest = Fraction(1, 2 ** (s - 1))
    if y < smallest:
        return 0, y / smallest
    e = math.floor(math.log2(y))
    while Fraction(2) ** e > y: e -= 1
    while Fraction(2) ** (e + 1) <= y: e += 1
    low = Fraction(2) ** e
    return e + s, (y - low) / low                      # 2^e = 2^(k-s)  =>  k = e + s


LIN_CASES = [(-0.3, 1.0, 127), (0.3, 1.0, 127), (0.3, 1.0, 255), (1.234e-3, 0.5531, 127),
             (-7.7e-4, 2.0013, 127), (3.3e-9, 2.0013, 15), (-4.2e-7, 346.4, 15), (0.9991, 1.0, 7),
             (5e-4, 1e-3, 1), (0.61803, 0.70711, 3), (1e-30, 3e-29, 127), (123.4, 1000.0, 127)]


@pytest.mark.parametrize("x,norm,s", LIN_CASES)
def test_linear_rounding_law(x, norm, s):
    h, f = exact_linear(x, norm, s)
    sign = -1 if x < 0 else 1
    # only the two neighbouring levels occur, with the sign of x, and 'up' is monotone in the word
    r = sample_words(20000, 11)
    q = O.quantize_with_words(np.full(r.shape, x, F32), r, norm, O.LINEAR, s)
    assert set(np.unique(q).tolist()) <= {sign * h, sign * (h + 1)}
    up = (np.abs(q) == h + 1)
    assert np.all(up[:-1] >= up[1:])
    # P(upper level) = y*s - h  (Eq. (2) with l_u = (s-u)/s), to the resolution of binary32
    p = Fraction(count_up(O.LINEAR, x, norm, s, h + 1), TWO32)
    tol = Fraction(1, 2 ** 22) * max(1, h + 1) if h >= 1 else Fraction(1, 2 ** 22) * f + Fraction(1, 2 ** 31)
    assert abs(p - f) <= tol


EXP_CASES = [(-0.3, 1.0, 8), (0.3, 1.0, 16), (0.7, 1.0, 4), (1.234e-3, 0.5531, 16), (-7.7e-4, 2.0013, 16),
             (3.3e-3, 2.0013, 7), (-4.2e-5, 0.34, 7), (0.013, 1.0, 7), (0.0101, 1.0, 3), (0.4, 1.0, 1),
             (2.5e-6, 1.0, 16)]


@pytest.mark.parametrize("x,norm,s", EXP_CASES)
def test_exp_rounding_law(x, norm, s):
    k, pexact = exact_exp(x, norm, s)
    sign = -1 if x < 0 else 1
    r = sample_words(20000, 12)
    q = O.quantize_with_words(np.full(r.shape, x, F32), r, norm, O.EXP, s)
    assert set(np.unique(q).tolist()) <= {sign * k, sign * (k + 1)}
    up = (np.abs(q) == k + 1)
    assert np.all(up[:-1] <= up[1:])
    p = Fraction(count_up(O.EXP, x, norm, s, k + 1), TWO32)
    assert abs(p - pexact) <= Fraction(1, 2 ** 21)


def test_exp_counts_are_exact_when_the_scaling_is_exact():
    # norm a power of two => z = |x| * 2^(s-1) / norm carries no rounding, so over all 2^23 values
    # of the 23 dither bits the number of round-ups is exactly (z - 2^e)/2^e * 2^23 = the mantissa
    R = np.arange(1 << 23, dtype=np.uint32)
    low = np.random.default_rng(0).integers(0, 512, R.shape[0], dtype=np.uint32)
    words = (R << 9) | low                                   # the low 9 bits must not matter
    for x, norm, s in [(0.3, 1.0, 8), (-0.8125, 4.0, 5), (0.0123, 0.25, 16)]:
        k, pexact = exact_exp(x, norm, s)
        assert k >= 1
        q = O.quantize_with_words(np.full(R.shape, x, F32), words, norm, O.EXP, s)
        assert Fraction(int((np.abs(q) == k + 1).sum()), 1 << 23) == pexact
    # below the smallest level: round-ups = z * 2^23 rounded to nearest (exact when z has <= 23 bits)
    for x, norm, s in [(0.001953125 * 0.75, 1.0, 8), (3.0 / 1024.0, 2.0, 4), (2.0 ** -30, 1.0, 16)]:
        k, pexact = exact_exp(x, norm, s)
        assert k == 0
        q = O.quantize_with_words(np.full(R.shape, x, F32), words, norm, O.EXP, s)
        assert Fraction(int((q == 1).sum()), 1 << 23) == pexact
    # ... and to nearest otherwise
    x, norm, s = 1e-3 / 3.0, 1.0, 6
    k, pexact = exact_exp(x, norm, s)
    q = O.quantize_with_words(np.full(R.shape, x, F32), words, norm, O.EXP, s)
    assert abs(Fraction(int((q == 1).sum()), 1 << 23) - pexact) <= Fraction(1, 1 << 24)


def test_values_on_a_level_stay_there():
    r = sample_words(50000, 13)
    # linear: t = k exactly; v = fl32(k - U') can only fall to k-1 when U' is within half an ulp of
    # k of 1, so the level is kept with probability >= 1 - k * 2^-23, and with certainty for k <= 1
    # and for k = s (y = 1, recognised as |x| >= norm)
    for s, norm in [(4, 2.0), (8, 0.125), (128, 1.0), (16, 1024.0)]:
        for k in range(0, s + 1):
            for sign in (1, -1):
                x = sign * norm * k / s                          # exact: s and norm are powers of two
                q = O.quantize_with_words(np.full(r.shape, x, F32), r, norm, O.LINEAR, s)
                assert set(np.unique(q).tolist()) <= {sign * k, sign * max(k - 1, 0)}
                stay = Fraction(count_up(O.LINEAR, x, norm, s, k), TWO32)
                assert stay >= 1 - Fraction(k, 2 ** 23)
                if k <= 1 or k == s:
                    assert stay == 1
    # exponential: the decision is an integer carry, so a level is kept with certainty
    for s, norm in [(4, 2.0), (7, 0.125), (16, 1.0)]:
        for k in range(1, s + 1):
            for sign in (1, -1):
                x = sign * norm * 2.0 ** (k - s)
                q = O.quantize_with_words(np.full(r.shape, x, F32), r, norm, O.EXP, s)
                assert np.all(q == sign * k)
        q = O.quantize_with_words(np.zeros(r.shape, F32), r, norm, O.EXP, s)
        assert np.all(q == 0)


def test_zero_sign_symmetry_and_degenerate_norms():
    r = sample_words(5000, 14)
    rng = np.random.default_rng(15)
    x = rng.normal(0, 0.2, r.shape).astype(F32)
    for scheme, s in [(O.LINEAR, 127), (O.LINEAR, 15), (O.EXP, 16), (O.EXP, 7)]:
        q = O.quantize_with_words(x, r, 1.0, scheme, s)
        assert np.array_equal(O.quantize_with_words(-x, r, 1.0, scheme, s), -q)
        assert np.all(np.sign(q) * np.sign(x) >= 0) and np.abs(q).max() <= s
        for z in (0.0, -0.0):
            assert np.all(O.quantize_with_words(np.full(r.shape, z, F32), r, 1.0, scheme, s) == 0)
        for bad in (0.0, np.nan, np.inf, 1e-45):                # zero, non-finite, scale overflows
            assert np.all(O.quantize_with_words(x, r, bad, scheme, s) == 0)
    # denormal inputs with a denormal-sized norm are handled (no flush to zero): y = 1/2
    q = O.quantize_with_words(np.full(r.shape, 2e-39, F32), r, 4e-39, O.LINEAR, 1)
    assert 0.4 < q.mean() < 0.6


def test_top_of_range_is_clamped():
    rng = np.random.default_rng(16)
    norms = np.concatenate([rng.uniform(1e-6, 10.0, 4000), 10.0 ** rng.uniform(-30, 30, 4000)]).astype(F32)
    for s in (1, 7, 15, 127, 255):
        for r in (0, 1, 12345, TWO32 - 1):
            for sign in (1, -1):
                q = np.array([O.code(O.LINEAR, sign * n, n, s, r) for n in norms[:1500]])
                assert np.all(np.abs(q) <= s) and np.all(np.abs(q) >= s - 1) and np.all(np.sign(q) == sign)
    for s in (1, 7, 16):
        q = np.array([O.code(O.EXP, n, n, s, r) for n in norms[:1500] for r in (0, TWO32 - 1)])
        assert np.all(q >= s - 1) and np.all(q <= s)


# ------------------------------------------------------------------------------------------------
# exhaustive tiny vectors: exact expectation and exact variance of the whole chain
# ------------------------------------------------------------------------------------------------
def level_value(scheme, s, k):
    """The real number a code magnitude stands for (the grid of Section 4.2)."""
    if scheme == O.LINEAR:
        return Fraction(k, s)
    return Fraction(0) if k == 0 else Fraction(2) ** (k - s)


def two_point(scheme, x, norm, s):
    """(k_low, P(k_low + 1)) as the oracle realises them, by counting random words."""
    if scheme == O.LINEAR:
        k, _ = exact_linear(x, norm, s)
    else:
        k, _ = exact_exp(x, norm, s)
    k = min(k, s)
    if k == s:
        return s - 1, Fraction(count_up(scheme, x, norm, s, s), TWO32)
    return k, Fraction(count_up(scheme, x, norm, s, k + 1), TWO32)


@pytest.mark.parametrize("scheme", [O.LINEAR, O.EXP])
@pytest.mark.parametrize("s", [1, 2, 3, 7])
@pytest.mark.parametrize("K,d", [(1, 3), (2, 2), (2, 3)])
def test_tiny_vectors_exact_mean_and_variance(scheme, s, K, d):
    rng = np.random.default_rng(100 * s + 10 * K + d + scheme)
    xs = [rng.normal(0, 1.0, d).astype(F32) for _ in range(K)]
    xs[0][0] = 0.0                                              # one exact zero
    for kind in (O.NORM_LINF, O.NORM_L2):
        _, norm, _ = O.global_norm(xs, kind)
        nrm = Fraction(float(norm))
        xbar = [sum(Fraction(float(xs[i][j])) for i in range(K)) / K for j in range(d)]
        tp = [[two_point(scheme, xs[i][j], norm, s) for j in range(d)] for i in range(K)]
        mean = [Fraction(0)] * d
        var = Fraction(0)
        # every tuple of (lower | upper) choices, with its probability, through aggregate+dequantize
        for choice in itertools.product((0, 1), repeat=K * d):
            prob = Fraction(1)
            qs = [np.zeros(d, np.int32) for _ in range(K)]
            for i in range(K):
                for j in range(d):
                    k, p = tp[i][j]
                    c = choice[i * d + j]
                    prob *= p if c else (1 - p)
                    qs[i][j] = (k + c) * (-1 if xs[i][j] < 0 else 1)
            if prob == 0:
                continue
            A = O.aggregate(qs, scheme)
            g = O.dequantize(A, float(norm), scheme, s, K)
            # dequantize against the definition, Eq. (1): norm/n * sum sign * level
            for j in range(d):
                want = nrm / K * sum((-1 if xs[i][j] < 0 else 1) * level_value(scheme, s, abs(int(qs[i][j])))
                                     for i in range(K))
                assert abs(Fraction(float(g[j])) - want) <= abs(want) * Fraction(1, 10 ** 14)
                mean[j] += prob * want
                var += prob * (want - xbar[j]) ** 2
        # unbiasedness (Definition 3 / Lemma 2): E[G(x)] = mean of the workers
        scale = max(abs(v) for v in xbar) + Fraction(1, 10 ** 30)
        for j in range(d):
            assert abs(mean[j] - xbar[j]) <= scale * Fraction(1, 10 ** 6)
        # variance of independent two-point roundings: (norm/n)^2 sum (l_up - y)(y - l_low)
        closed = Fraction(0)
        for i in range(K):
            for j in range(d):
                y = abs(Fraction(float(xs[i][j]))) / nrm
                k, _ = tp[i][j]
                lo, hi = level_value(scheme, s, k), level_value(scheme, s, k + 1)
                closed += (hi - y) * (y - lo)
        closed *= (nrm / K) ** 2
        assert abs(var - closed) <= closed * Fraction(1, 10 ** 5) + Fraction(1, 10 ** 30)


# ------------------------------------------------------------------------------------------------
# Monte Carlo with the real Philox stream, and the variance bound of Theorem 1
# ------------------------------------------------------------------------------------------------
def closed_form_variance(xs, norm, scheme, s):
    """Per-coordinate variance of G(x): (norm/n)^2 * sum_i (l_up - y_ij)(y_ij - l_low), in float64."""
    K = len(xs)
    tot = np.zeros(xs[0].shape[0])
    for x in xs:
        y = np.abs(x.astype(np.float64)) / float(norm)
        if scheme == O.LINEAR:
            lo = np.floor(y * s) / s
            hi = lo + 1.0 / s
        else:
            small = 2.0 ** -(s - 1)
            e = np.floor(np.log2(np.maximum(y, 1e-300)))
            lo = np.where(y < small, 0.0, 2.0 ** e)
            hi = np.where(y < small, small, 2.0 ** (e + 1))
        tot += np.clip(hi - y, 0, None) * np.clip(y - lo, 0, None)
    return tot * (float(norm) / K) ** 2


def theta_linear(n, d, s):
    return math.sqrt(d) / (math.sqrt(n) * s)


def theta_exp(n, d, s):
    return 1.0 / (8 * n) + math.sqrt(d) / (math.sqrt(n) * 2.0 ** (s - 1))


def test_theta_formula_reproduces_the_papers_worked_number():
    # Section 6: n = 16, d = 1e6, 7 bits for levels (s = 127), exponential dithering:
    # 1 + n^1.17 * theta_E is a 20 % increase in iterations
    assert 1.0 + 16 ** 1.17 * theta_exp(16, 10 ** 6, 127) == pytest.approx(1.20, abs=0.005)


@pytest.mark.parametrize("scheme,s,kind", [(O.LINEAR, 127, O.NORM_LINF), (O.LINEAR, 15, O.NORM_L2),
                                           (O.LINEAR, 1, O.NORM_L2), (O.EXP, 16, O.NORM_L2),
                                           (O.EXP, 7, O.NORM_LINF), (O.EXP, 3, O.NORM_L2)])
def test_monte_carlo_unbiased_with_closed_form_variance_and_theorem1_bound(scheme, s, kind):
    K, d, T = 4, 384, 3000
    rng = np.random.default_rng(1000 + 10 * s + scheme)
    xs = [(rng.standard_t(3, d) * 1e-3).astype(F32) for _ in range(K)]
    xs[1][5] = 0.0
    _, norm, _ = O.global_norm(xs, kind)
    xbar = np.mean(np.stack(xs).astype(np.float64), axis=0)
    var = closed_form_variance(xs, norm, scheme, s)
    acc = np.zeros(d); sq = 0.0
    for t in range(T):
        A = O.quantize_aggregate(xs, norm, scheme, s, seed=0xABC000 + t)
        g = O.dequantize(A, float(norm), scheme, s, K)
        acc += g
        sq += ((g - xbar) ** 2).sum()
    mean = acc / T
    # E[G(x)] = mean of the workers: every coordinate within 5 standard errors
    assert np.all(np.abs(mean - xbar) <= 5.0 * np.sqrt(var / T) + 1e-12 * np.abs(xbar))
    # E||G(x) - xbar||^2 equals the closed form (3 % at this T) ...
    assert sq / T == pytest.approx(var.sum(), rel=0.03)
    # ... and obeys Theorem 1: <= theta/n * ||x||_{2,2}^2
    # (the theorem states its theta for s <= sqrt(nd), resp. s <= 1 + log2 sqrt(nd))
    in_range = s <= math.sqrt(K * d) if scheme == O.LINEAR else s <= 1 + math.log2(math.sqrt(K * d))
    if in_range:
        theta = theta_linear(K, d, s) if scheme == O.LINEAR else theta_exp(K, d, s)
        norm22sq = sum((x.astype(np.float64) ** 2).sum() for x in xs)
        assert var.sum() <= theta / K * norm22sq
        assert sq / T <= theta / K * norm22sq


def test_workers_round_independently():
    # the same gradient on two workers: the roundings must differ and be uncorrelated (Lemma 2 needs it)
    d = 1 << 16
    x = np.full(d, 0.5 / 127.0, F32)                               # P(up) = 1/2 at every coordinate
    q0 = O.quantize(x, 1.0, O.LINEAR, 127, seed=7, worker=0)
    q1 = O.quantize(x, 1.0, O.LINEAR, 127, seed=7, worker=1)
    assert set(np.unique(q0).tolist()) == {0, 1}
    assert abs(q0.mean() - 0.5) < 5 * 0.5 / math.sqrt(d)
    corr = ((q0 - 0.5) * (q1 - 0.5)).mean() / 0.25
    assert abs(corr) < 5 / math.sqrt(d)
    # neighbouring coordinates of one worker as well
    corr = ((q0[:-1] - 0.5) * (q0[1:] - 0.5)).mean() / 0.25
    assert abs(corr) < 5 / math.sqrt(d)


def test_quantize_is_a_function_of_the_global_index():
    rng = np.random.default_rng(21)
    x = rng.normal(0, 1e-3, 5000).astype(F32)
    for scheme, s in [(O.LINEAR, 127), (O.EXP, 16)]:
        whole = O.quantize(x, 4e-3, scheme, s, seed=99, worker=2)
        for lo, hi in [(0, 1234), (1234, 1237), (1237, 5000)]:
            part = O.quantize(x[lo:hi], 4e-3, scheme, s, seed=99, worker=2, index_base=lo)
            assert np.array_equal(part, whole[lo:hi])
        big = O.quantize(x[:64], 4e-3, scheme, s, seed=99, worker=2, index_base=2 ** 35)
        assert not np.array_equal(big, whole[:64])


def test_worst_case_sum_reaches_n_times_s_and_never_more():
    # Section 4.2: the largest aggregated value is n*s (linear); |x| = norm everywhere reaches it
    K, d = 16, 257
    xs = [np.full(d, 0.25 * (-1) ** (i // 8), F32) for i in range(K)]   # 8 workers +, 8 workers -
    A = O.quantize_aggregate([np.abs(x) for x in xs], 0.25, O.LINEAR, 127, seed=1)
    assert np.all(A == 16 * 127)                              # y = 1 is the top level with certainty
    assert O.fits_width(A, 16) and not O.fits_width(A, 8)
    assert np.abs(O.quantize_aggregate(xs, 0.25, O.LINEAR, 127, seed=1)).max() <= 2
    one = O.quantize_aggregate([np.abs(x) for x in xs], 0.25, O.LINEAR, 1, seed=1)
    assert np.all(one == 16)                                  # s = 1: the top level is kept with certainty
    A = O.quantize_aggregate([-np.abs(x) for x in xs], 0.25, O.EXP, 7, seed=1)
    assert np.all(A == -16 * 64)
    # arbitrary norms: |x| = norm is y = 1 whatever fl32(s / norm) is, on both grids; one ulp below the norm the
    # sum stays within n*s whatever the rounding at the top does
    rng = np.random.default_rng(4)
    for norm in rng.uniform(1e-3, 3.0, 50).astype(F32):
        A = O.quantize_aggregate([np.full(33, norm, F32)] * K, norm, O.LINEAR, 127, seed=2)
        assert np.all(A == K * 127)
        A = O.quantize_aggregate([np.full(33, -norm, F32)] * K, norm, O.EXP, 9, seed=2)
        assert np.all(A == -K * 256)
        below = np.nextafter(norm, F32(0))
        A = O.quantize_aggregate([np.full(33, below, F32)] * K, norm, O.LINEAR, 127, seed=2)
        assert np.abs(A).max() <= K * 127 and np.abs(A).min() >= K * 126


def test_composition_equals_its_parts():
    rng = np.random.default_rng(8)
    K, d = 5, 777
    xs = [rng.normal(0, 1e-2, d).astype(F32) for _ in range(K)]
    for scheme, s in [(O.LINEAR, 127), (O.EXP, 7)]:
        qs = [O.quantize(xs[i], 0.05, scheme, s, seed=3, worker=i, index_base=40) for i in range(K)]
        assert np.array_equal(O.aggregate(qs, scheme), O.quantize_aggregate(xs, 0.05, scheme, s, 3, 40))

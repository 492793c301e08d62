"""Pins for the oracle's sparse branch (arXiv 2305.18627, Algorithm 1's sparse branch; Theorem 1's sparsity
statement for p = q = 2).  Expected values: numpy's nonzero, the dense aggregate, and the expected
number of non-zero codes that Eq. (2) implies."""
import math

import numpy as np
import pytest

from oracle import gq_oracle as O


def test_compact_is_nonzero_in_index_order():
    rng = np.random.default_rng(0)
    for d in (0, 1, 5, 1000, 4097):
        q = rng.integers(-3, 4, d).astype(np.int32)
        q[rng.random(d) < 0.6] = 0
        n, idx, val = O.compact(q)
        nz = np.nonzero(q)[0]
        assert n == nz.shape[0] and np.array_equal(idx, nz.astype(np.uint32)) and np.array_equal(val, q[nz])
        if n > 2:                                              # a short buffer: true count, first entries only
            n2, idx2, val2 = O.compact(q, capacity=2)
            assert n2 == n and np.array_equal(idx2, idx[:2]) and np.array_equal(val2, val[:2])
    assert O.compact(np.zeros(10, np.int32))[0] == 0


@pytest.mark.parametrize("scheme,s", [(O.LINEAR, 15), (O.EXP, 7)])
def test_sparse_aggregate_equals_dense_aggregate(scheme, s):
    rng = np.random.default_rng(s)
    K, d = 6, 3001
    qs = []
    for _ in range(K):
        q = rng.integers(-s, s + 1, d).astype(np.int32)
        q[rng.random(d) < 0.8] = 0
        qs.append(q)
    lists = [O.compact(q) for q in qs]
    A = O.sparse_aggregate([l[1] for l in lists], [l[2] for l in lists], d, scheme)
    assert np.array_equal(A, O.aggregate(qs, scheme))
    # the order of the workers' lists does not matter
    assert np.array_equal(O.sparse_aggregate([l[1] for l in lists[::-1]], [l[2] for l in lists[::-1]], d, scheme), A)


def test_expected_number_of_nonzeros_under_the_l2_norm():
    # Eq. (2): below the first level (y*s < 1) a coordinate is non-zero with probability y*s, above it always.
    # Hence E[nnz] = sum min(1, y*s).  At most s^2 coordinates can have y >= 1/s (since sum y^2 <= 1) and
    # sum y <= sqrt(nd), so E[nnz] <= s^2 + s*sqrt(nd): the form of Theorem 1's sparsity bound that follows
    # from Eq. (2).  (As printed, s^2 + sqrt(nd) without the factor s, the bound fails for Gaussian inputs
    # already at s = 4, which the last assertion documents.)
    K, d, s, T = 4, 1024, 4, 400
    rng = np.random.default_rng(2)
    xs = [rng.normal(0, 1e-3, d).astype(np.float32) for _ in range(K)]
    _, norm, _ = O.global_norm(xs, O.NORM_L2)
    y = np.abs(np.stack(xs).astype(np.float64)) / float(norm)
    expected = np.minimum(1.0, y * s).sum()
    counts = []
    for t in range(T):
        counts.append(sum(O.compact(O.quantize(xs[i], norm, O.LINEAR, s, 900 + t, i))[0] for i in range(K)))
    mean = np.mean(counts)
    assert abs(mean - expected) <= 5.0 * np.std(counts) / math.sqrt(T) + 1e-9
    assert expected <= s * s + s * math.sqrt(K * d)
    assert expected > s * s + math.sqrt(K * d)


def expected_nonzeros(xs, norm, top):
    """Exact expectation of the number of non-zero codes that Eq. (2) gives: a coordinate with y * top >= 1 is non-zero
    always, below that with probability y * top (top = s, or 2^(s-1) on the exponential grid)."""
    y = np.abs(np.stack(xs).astype(np.float64)) / float(norm)
    return float(np.minimum(1.0, y * top).sum())


@pytest.mark.parametrize("scheme,s", [(O.LINEAR, 1), (O.LINEAR, 4), (O.LINEAR, 15), (O.LINEAR, 127), (O.EXP, 1), (O.EXP, 4), (O.EXP, 7)])
def test_sparsity_bound_holds_for_the_exact_expectation_and_both_terms_are_attained(scheme, s):
    top = float(s) if scheme == O.LINEAR else float(2 ** (s - 1))
    K, d = 3, 5000
    rng = np.random.default_rng(10 * s + scheme)
    bound = O.sparse_nnz_bound(scheme, s, K, d)
    # (a) the bound covers the exact expectation for light tails, heavy tails and a few spikes
    for kind in range(3):
        if kind == 0:
            xs = [rng.normal(0, 1e-3, d).astype(np.float32) for _ in range(K)]
        elif kind == 1:
            xs = [(1e-4 * rng.standard_t(3, d)).astype(np.float32) for _ in range(K)]
        else:
            xs = [np.where(rng.random(d) < 0.002, 1.0, 1e-6).astype(np.float32) * rng.choice([-1.0, 1.0], d).astype(np.float32) for _ in range(K)]
        _, norm, _ = O.global_norm(xs, O.NORM_L2)
        assert expected_nonzeros(xs, norm, top) <= bound
    # (b) the first term alone is attained: top^2 coordinates exactly on the smallest non-zero level, zeros elsewhere
    #     (sum y^2 = 1): all of them are non-zero with certainty and nothing else is
    m = int(top * top)
    if m <= K * d:
        flat = np.zeros(K * d, np.float64); flat[:m] = 1.0 / top
        assert abs(np.sum(flat ** 2) - 1.0) < 1e-12
        assert abs(np.minimum(1.0, flat * top).sum() - m) < 1e-9 * m
        assert bound == K * d or abs((bound - top * math.sqrt(K * d)) - m) < 1e-9 * bound
    # (c) the second term alone is attained: all K d coordinates equal, y = 1/sqrt(K d) each (if that is below 1/top):
    #     E[nnz] = top * sqrt(K d) exactly
    y = 1.0 / math.sqrt(K * d)
    if y * top <= 1.0:
        e = K * d * y * top
        assert abs(e - top * math.sqrt(K * d)) < 1e-9 * e
        assert bound == K * d or abs((bound - top * top) - e) < 1e-9 * e
    # (d) never more than there are coordinates; invalid arguments
    assert O.sparse_nnz_bound(scheme, s, 1, 3) <= 3.0
    assert O.sparse_nnz_bound(scheme, s, 2, 0) == 0.0
    assert O.sparse_nnz_bound(scheme, 0, K, d) == -1.0 and O.sparse_nnz_bound(scheme, s, 0, d) == -1.0
    assert O.sparse_nnz_bound(2, s, K, d) == -1.0 and O.sparse_nnz_bound(O.EXP, 32, K, d) == -1.0


def test_sparsity_bound_values_by_hand():
    # linear s = 4, K d = 4096: 16 + 4 * 64 = 272; exponential s = 4 (top = 8): 64 + 8 * 64 = 576; the printed form
    # 16 + 64 = 80 is what a Gaussian gradient exceeds (test above)
    assert O.sparse_nnz_bound(O.LINEAR, 4, 4, 1024) == 272.0
    assert O.sparse_nnz_bound(O.EXP, 4, 4, 1024) == 576.0
    assert O.sparse_nnz_bound(O.LINEAR, 127, 16, 110_000_000) == 127.0 ** 2 + 127.0 * math.sqrt(16 * 110_000_000)
    assert O.sparse_nnz_bound(O.LINEAR, 127, 1, 100) == 100.0                      # capped at K d

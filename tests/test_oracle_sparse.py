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

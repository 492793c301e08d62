"""Pins for the oracle's short draws (16 random bits per coordinate, one Philox call per eight
coordinates).  Eq. (2) of arXiv 2305.18627 fixes probabilities only, so the number of random bits is a
free choice; what must hold is that the 16 bits of the eight coordinates of a call are exactly the 128
bits of the Philox block (pinned by the publication's known answers elsewhere), each used once, and
that over all 2^16 values of a coordinate's bits the upper level is taken with the probability of
Eq. (2) to 2^-16.  Expected counts come from exact rational arithmetic on the inputs.
"""
from fractions import Fraction
import math

import numpy as np
import pytest

from oracle import gq_oracle as O
from test_oracle_rounding import exact_linear, exact_exp, LIN_CASES, EXP_CASES

F32 = np.float32
ALL16 = (np.arange(1 << 16, dtype=np.uint32) << 16)          # every short draw, as the oracle presents it


def test_the_eight_draws_of_a_call_are_the_bytes_of_the_philox_block():
    seed = 0x0123456789ABCDEF
    for call in [0, 1, 5, 2**32 + 7, 2**36 + 1]:
        for worker in [0, 3, 63]:
            blk = O.philox4x32([call & 0xFFFFFFFF, call >> 32, worker, 0], [seed & 0xFFFFFFFF, seed >> 32])
            raw = np.asarray(blk, dtype="<u4").tobytes()               # 16 bytes, little endian words
            r = O.random_words(seed, worker, 8 * call, 8, rng_bits=16)
            assert np.all((r & 0xFFFF) == 0)                             # only the top half is populated
            got = (r >> 16).astype("<u2").tobytes()
            assert got == raw
    # a run of draws is the per-index draw whatever the base, also for a base inside a call
    a = O.random_words(seed, 3, 0, 1000, rng_bits=16)
    b = O.random_words(seed, 3, 123, 877, rng_bits=16)
    assert np.array_equal(a[123:], b)
    # and the two modes do not share their stream layout (g/8 against g/4)
    assert not np.array_equal(a[:64] >> 16, O.random_words(seed, 3, 0, 64) >> 16)


def test_short_draws_look_uniform_and_workers_differ():
    n = 1 << 20
    r0 = O.random_words(0xC0FFEE, 0, 0, n, rng_bits=16) >> 16
    r1 = O.random_words(0xC0FFEE, 1, 0, n, rng_bits=16) >> 16
    assert (r0 != r1).mean() > 0.999
    for shift in (0, 8):
        h = np.bincount((r0 >> shift) & 0xFF, minlength=256).astype(np.float64)
        chi2 = ((h - n / 256.0) ** 2 / (n / 256.0)).sum()
        assert chi2 < 400.0                                              # 255 d.o.f., sd 22.6
    u = r0 / 65536.0 - 0.5
    assert abs(u.mean()) < 5.0 / np.sqrt(12.0 * n)
    assert abs((u[:-1] * u[1:]).mean()) < 5.0 / (12.0 * np.sqrt(n))


@pytest.mark.parametrize("x,norm,s", LIN_CASES)
def test_linear_law_over_all_short_draws(x, norm, s):
    h, f = exact_linear(x, norm, s)
    sign = -1 if x < 0 else 1
    q = O.quantize_with_words(np.full(ALL16.shape, x, F32), ALL16, norm, O.LINEAR, s)
    assert set(np.unique(q).tolist()) <= {sign * h, sign * (h + 1)}
    up = np.abs(q) == h + 1
    assert np.all(up[:-1] >= up[1:])                                     # 'up' for small draws
    # 'up' iff r16/2^16 < frac, i.e. for ceil(frac * 2^16) of the 2^16 draws; binary32 rounding of
    # t = |x| s / norm (relative 2^-23 each for the scale and the product) can move the threshold by
    # one draw when t*2^-22 reaches 2^-16, never by more for these cases
    want = math.ceil(f * (1 << 16))
    slack = 1 if (h + 1) * 2.0 ** -22 * 65536 < 1 else 2
    assert abs(int(up.sum()) - want) <= slack
    assert abs(Fraction(int(up.sum()), 1 << 16) - f) <= Fraction(slack + 1, 1 << 16)


@pytest.mark.parametrize("x,norm,s", EXP_CASES)
def test_exp_law_over_all_short_draws(x, norm, s):
    k, pexact = exact_exp(x, norm, s)
    sign = -1 if x < 0 else 1
    q = O.quantize_with_words(np.full(ALL16.shape, x, F32), ALL16, norm, O.EXP, s)
    assert set(np.unique(q).tolist()) <= {sign * k, sign * (k + 1)}
    up = np.abs(q) == k + 1
    assert np.all(up[:-1] <= up[1:])                                     # 'up' for large draws
    assert abs(Fraction(int(up.sum()), 1 << 16) - pexact) <= Fraction(2, 1 << 16)


def test_exp_short_draw_counts_are_exact_when_the_scaling_is_exact():
    # norm a power of two: z carries no rounding; 'up' iff mantissa + r16 * 2^7 >= 2^23, which holds for
    # floor(mantissa / 2^7) of the draws: the probability of Eq. (2) rounded DOWN to a multiple of 2^-16
    for x, norm, s in [(0.3, 1.0, 8), (-0.8125, 4.0, 5), (0.0123, 0.25, 16), (0.001953125 * 0.75, 1.0, 8)]:
        k, pexact = exact_exp(x, norm, s)
        q = O.quantize_with_words(np.full(ALL16.shape, x, F32), ALL16, norm, O.EXP, s)
        assert int((np.abs(q) == k + 1).sum()) == math.floor(pexact * (1 << 16))


def test_quantize_with_short_draws_is_the_rule_applied_to_those_draws():
    rng = np.random.default_rng(5)
    d = 4001
    x = (rng.standard_normal(d) * 1e-3).astype(F32)
    norm = F32(np.abs(x).max())
    for scheme, s in [(O.LINEAR, 127), (O.LINEAR, 7), (O.EXP, 7), (O.EXP, 16)]:
        for worker, base in [(0, 0), (5, 8 * 12345), (2, 2**35 + 24)]:
            q = O.quantize(x, norm, scheme, s, 99, worker, base, rng_bits=16)
            r = O.random_words(99, worker, base, d, rng_bits=16)
            assert np.array_equal(q, O.quantize_with_words(x, r, norm, scheme, s))
            assert not np.array_equal(q, O.quantize(x, norm, scheme, s, 99, worker, base))   # differs from 32-bit draws
    # the fused composition takes the same flag
    xs = [(rng.standard_normal(d) * 1e-3).astype(F32) for _ in range(3)]
    A = O.quantize_aggregate(xs, norm * 4, O.LINEAR, 127, 7, 64, rng_bits=16)
    want = sum(O.quantize(xs[i], norm * 4, O.LINEAR, 127, 7, i, 64, rng_bits=16).astype(np.int64) for i in range(3))
    assert np.array_equal(A, want)


def test_short_draws_are_unbiased_to_two_to_minus_16():
    # mean over all 2^16 draws of the dequantised value against x: Definition 1 asks E = x
    for scheme, s in [(O.LINEAR, 127), (O.LINEAR, 3), (O.EXP, 7)]:
        for x, norm in [(0.3, 1.0), (-0.0123, 0.7), (5e-4, 1.0)]:
            q = O.quantize_with_words(np.full(ALL16.shape, x, F32), ALL16, norm, scheme, s).astype(np.int64)
            vals = np.array([O.code_value(scheme, int(v)) for v in np.unique(q)])
            lut = dict(zip(np.unique(q).tolist(), vals.tolist()))
            unit = s if scheme == O.LINEAR else 2 ** (s - 1)
            mean = sum(lut[int(v)] * int(c) for v, c in zip(*np.unique(q, return_counts=True))) / 65536.0
            got = mean * float(F32(norm)) / unit
            step = float(F32(norm)) / unit                          # spacing of the two neighbouring levels (at most)
            top = step if scheme == O.LINEAR else max(abs(x), step)  # exponential: spacing <= |x| above the smallest level
            assert abs(got - float(F32(x))) <= 3 * top * 2.0 ** -16

"""Pins for the oracle's random stream, norm, storage formats, width rule and dequantisation.

Each expected value here comes from outside the oracle: the Philox publication's known-answer
vectors, numpy brute force, closed forms, bytes and numbers worked out by hand, or statements the
paper prints (arXiv 2305.18627, Section 4.2 and the Implementation section on integer headroom).
"""
import os

import numpy as np
import pytest

from oracle import gq_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- Philox (Salmon et al., SC'11)
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for row in rows:
        v = [int(t, 16) for t in row]
        out = O.philox4x32(v[0:4], v[4:6], rounds=10)
        assert [int(o) for o in out] == v[6:10]


def test_random_word_counter_layout():
    # counter = (lo32(g/4), hi32(g/4), worker, 0), key = (lo32(seed), hi32(seed)), word g mod 4;
    # the index is taken past 2^34 so that the high counter word is exercised
    seed = 0x0123456789ABCDEF
    for g in [0, 1, 2, 3, 4, 7, 4 * (2**32) + 5, 2**40 + 3]:
        for worker in [0, 1, 31]:
            blk = O.philox4x32([(g // 4) & 0xFFFFFFFF, (g // 4) >> 32, worker, 0],
                               [seed & 0xFFFFFFFF, seed >> 32])
            assert int(O.random_words(seed, worker, g, 1)[0]) == int(blk[g % 4])
    # a run of words is the per-index word, whatever the base: bucketed == unbucketed
    a = O.random_words(seed, 3, 0, 1000)
    b = O.random_words(seed, 3, 123, 877)
    assert np.array_equal(a[123:], b)


def test_random_words_look_uniform_and_workers_differ():
    n = 1 << 20
    r0 = O.random_words(0xC0FFEE, 0, 0, n)
    r1 = O.random_words(0xC0FFEE, 1, 0, n)
    r2 = O.random_words(0xC0FFEF, 0, 0, n)
    assert (r0 != r1).mean() > 0.999 and (r0 != r2).mean() > 0.999
    # chi-square of every byte lane against the uniform law: 255 degrees of freedom,
    # mean 255, sd 22.6; 400 is beyond 6 sd
    for shift in (0, 8, 16, 24):
        h = np.bincount((r0 >> shift) & 0xFF, minlength=256).astype(np.float64)
        chi2 = ((h - n / 256.0) ** 2 / (n / 256.0)).sum()
        assert chi2 < 400.0
    # mean of r/2^32 is 1/2 with sd 1/sqrt(12 n)
    assert abs((r0 / 2.0**32).mean() - 0.5) < 5.0 / np.sqrt(12.0 * n)
    # adjacent-word correlation is that of independent draws
    u = r0 / 2.0**32 - 0.5
    assert abs((u[:-1] * u[1:]).mean()) < 5.0 / (12.0 * np.sqrt(n))


# ---------------------------------------------------------------- norm (Algorithm 1's norm step)
def test_norm_against_numpy_bruteforce():
    rng = np.random.default_rng(1)
    xs = [rng.normal(0, 1e-3, 5001).astype(np.float32) for _ in range(5)]
    cat = np.concatenate(xs).astype(np.float64)
    ne, nf, fl = O.global_norm(xs, O.NORM_LINF)
    assert ne == np.abs(cat).max() and nf == np.float32(np.abs(cat).max()) and fl == 0
    ne, nf, fl = O.global_norm(xs, O.NORM_L2)
    assert abs(ne - np.sqrt((cat * cat).sum())) <= 1e-12 * ne and fl == 0
    ne, nf, fl = O.global_norm(xs, O.NORM_L2_MAX)
    per = [np.sqrt((x.astype(np.float64) ** 2).sum()) for x in xs]
    assert abs(ne - max(per)) <= 1e-12 * ne


def test_norm_closed_forms_and_ordering():
    K, d, c = 3, 4096, np.float32(0.125)
    xs = [np.full(d, c, np.float32) * (-1) ** i for i in range(K)]
    assert O.global_norm(xs, O.NORM_LINF)[0] == 0.125
    assert O.global_norm(xs, O.NORM_L2)[0] == pytest.approx(0.125 * np.sqrt(K * d), rel=1e-14)
    assert O.global_norm(xs, O.NORM_L2_MAX)[0] == pytest.approx(0.125 * np.sqrt(d), rel=1e-14)
    # the norms the paper's variance theorem relies on: (inf,inf) <= (2,inf) <= (2,2)
    rng = np.random.default_rng(2)
    ys = [rng.standard_normal(333).astype(np.float32) for _ in range(4)]
    a, b, c2 = (O.global_norm(ys, k)[0] for k in (O.NORM_LINF, O.NORM_L2_MAX, O.NORM_L2))
    assert a <= b <= c2
    # a single non-zero coordinate: all three norms are its magnitude
    z = [np.zeros(10, np.float32) for _ in range(2)]
    z[1][7] = -3.5
    for k in (O.NORM_LINF, O.NORM_L2, O.NORM_L2_MAX):
        assert O.global_norm(z, k)[0] == 3.5


def test_norm_flags():
    z = [np.zeros(8, np.float32)]
    assert O.global_norm(z, O.NORM_LINF)[2] == 2 and O.global_norm(z, O.NORM_L2)[2] == 2
    z[0][3] = -0.0
    assert O.global_norm(z, O.NORM_LINF)[2] == 2
    for bad in (np.nan, np.inf, -np.inf):
        for pos in (0, 7):
            y = [np.ones(8, np.float32), np.ones(8, np.float32)]
            y[1][pos] = bad
            for k in (O.NORM_LINF, O.NORM_L2, O.NORM_L2_MAX):
                assert O.global_norm(y, k)[2] & 1
    # squares that overflow binary32 but whose norm does not: still finite (accumulated in binary64)
    y = [np.full(4, 1e30, np.float32)]
    ne, nf, fl = O.global_norm(y, O.NORM_L2)
    assert fl == 0 and nf == np.float32(2e30)


# ---------------------------------------------------------------- storage formats
def test_pack_bytes_by_hand():
    # I8: two's complement bytes
    lv, sp = O.pack([0, 1, -1, 127, -127], O.PACK_I8)
    assert lv.tolist() == [0x00, 0x01, 0xFF, 0x7F, 0x81] and sp is None
    # I4: even index in the low nibble, two's complement nibbles, odd d pads the last high nibble with 0
    lv, sp = O.pack([-1, 7, 3, -7, -2], O.PACK_I4)
    assert lv.tolist() == [0x7F, 0x93, 0x0E] and sp is None
    # U8 + sign plane: magnitudes, and bit t of word w set iff coordinate 32w+t is negative
    q = np.zeros(40, np.int32); q[0] = -255; q[5] = 200; q[31] = -1; q[33] = -9
    lv, sp = O.pack(q, O.PACK_U8_SIGNPLANE)
    assert lv[0] == 255 and lv[5] == 200 and lv[31] == 1 and lv[33] == 9
    assert sp.tolist() == [(1 << 0) | (1 << 31), 1 << 1]
    # U4 + sign plane
    lv, sp = O.pack([-15, 15, 0, -1], O.PACK_U4_SIGNPLANE)
    assert lv.tolist() == [0xFF, 0x10] and sp.tolist() == [0b1001]


@pytest.mark.parametrize("fmt,lim", [(O.PACK_I8, 127), (O.PACK_I4, 7), (O.PACK_U8_SIGNPLANE, 255),
                                     (O.PACK_U4_SIGNPLANE, 15)])
def test_pack_roundtrip_full_range_and_limits(fmt, lim):
    full = np.arange(-lim, lim + 1, dtype=np.int32)
    rng = np.random.default_rng(fmt)
    for d in (2 * lim + 1, 1, 2, 31, 32, 33, 64, 65, 1001):
        q = full if d == 2 * lim + 1 else rng.integers(-lim, lim + 1, d).astype(np.int32)
        lv, sp = O.pack(q, fmt)
        assert np.array_equal(O.unpack(lv, sp, d, fmt), q)
        assert lv.shape[0] == (d if fmt in (O.PACK_I8, O.PACK_U8_SIGNPLANE) else (d + 1) // 2)
        if sp is not None:
            assert sp.shape[0] == (d + 31) // 32
            if d % 32:
                assert int(sp[-1]) >> (d % 32) == 0          # pad bits are zero
    with pytest.raises(OverflowError):
        O.pack([lim + 1], fmt)
    with pytest.raises(OverflowError):
        O.pack([-(lim + 1)], fmt)


# ---------------------------------------------------------------- integer sum and its headroom
def test_code_values():
    assert [O.code_value(O.LINEAR, q) for q in (-127, -1, 0, 1, 5)] == [-127, -1, 0, 1, 5]
    # exponential: code k >= 1 stands for 2^(k-s), i.e. 2^(k-1) units of the smallest level
    assert [O.code_value(O.EXP, q) for q in (0, 1, 2, 3, 7, -1, -4, 16)] == [0, 1, 2, 4, 64, -1, -8, 32768]


def test_aggregate_is_the_plain_sum_and_order_free():
    rng = np.random.default_rng(5)
    qs = [rng.integers(-7, 8, 1000).astype(np.int32) for _ in range(6)]
    A = O.aggregate(qs, O.LINEAR)
    assert np.array_equal(A, np.sum(np.stack(qs).astype(np.int64), axis=0))
    assert np.array_equal(O.aggregate(qs[::-1], O.LINEAR), A)
    vals = np.sign(np.stack(qs)) * np.where(np.stack(qs) == 0, 0, 2 ** (np.abs(np.stack(qs)) - 1).clip(0))
    assert np.array_equal(O.aggregate(qs, O.EXP), vals.astype(np.int64).sum(axis=0))


def test_width_rule_statements_of_the_paper():
    # Section 4.2: with linear dithering the largest sum is n*s and one more bit holds the sign;
    # n = 16 workers and A = 4 bits cannot be satisfied for any s
    assert not any(O.check_width(O.LINEAR, s, 16, 4) for s in range(1, 16))
    # Implementation section: 4-bit linear with 4 workers leaves a single bit for the value
    assert O.check_width(O.LINEAR, 1, 4, 4) and not O.check_width(O.LINEAR, 2, 4, 4)
    # the same rule written as the paper does, 1 + log2(s+1) + log2(n) <= A, for powers of two
    for A in (4, 8, 16, 32):
        for logn in range(0, 6):
            for logs1 in range(1, 9):                      # s + 1 = 2^logs1
                s, n = 2 ** logs1 - 1, 2 ** logn
                # n*s <= 2^(A-1) - 1  <=>  n*(s+1) <= 2^(A-1) when both are powers of two
                assert O.check_width(O.LINEAR, s, n, A) == (1 + logs1 + logn <= A)
    # the workloads: 16*127 in int32, 8*2^15 in int32, 32*2^6 in int16 hold; 32*2^14 in int16 does not
    assert O.check_width(O.LINEAR, 127, 16, 32) and O.check_width(O.EXP, 16, 8, 32)
    assert O.check_width(O.EXP, 7, 32, 16) and not O.check_width(O.EXP, 15, 32, 16)
    assert O.max_aggregate(O.LINEAR, 127, 16) == 2032 and O.max_aggregate(O.EXP, 7, 32) == 2048


def test_fits_width():
    assert O.fits_width([32767, -32768, 0], 16) and not O.fits_width([32768], 16)
    assert not O.fits_width([-32769], 16) and O.fits_width([2**31 - 1, -2**31], 32)


# ---------------------------------------------------------------- dequantisation (Eq. (1))
def test_dequantize_by_hand():
    # linear: norm * A / (n s):  2 * [4,-8,0,1] / (2*4)
    out = O.dequantize([4, -8, 0, 1], 2.0, O.LINEAR, 4, 2)
    assert out.tolist() == [1.0, -2.0, 0.0, 0.25]
    # exponential: unit 2^-(s-1):  8 * [4,-1,0] * 2^-2 / 2
    out = O.dequantize([4, -1, 0], 8.0, O.EXP, 3, 2)
    assert out.tolist() == [4.0, -1.0, 0.0]
    # linear in A, and exact zeros stay zero
    rng = np.random.default_rng(3)
    A = rng.integers(-2032, 2033, 500)
    B = rng.integers(-2032, 2033, 500)
    f = lambda a: O.dequantize(a, 0.37, O.LINEAR, 127, 16)
    assert np.allclose(f(A) + f(B), f(A + B), rtol=1e-13, atol=1e-15)
    assert np.all(f(np.zeros(5, np.int64)) == 0.0)

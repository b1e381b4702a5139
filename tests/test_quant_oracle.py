"""Pins of the quantization-variant oracle (paper Section 4.2: simQ, Q, rounding strategies)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle as O
from oracle import quant as OQ

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_philox_known_answers():
    for line in open(os.path.join(ROOT, "tests", "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        got = OQ.philox4x32_10(np.array([w[0:4]], dtype=np.uint32), (w[4], w[5]))[0]
        assert [int(v) for v in got] == w[6:10]


def test_random_words_take_word_e_mod_4_of_block_e_div_4():
    idx = np.arange(0, 23)
    words = OQ.random_words(idx, seed=(7 << 32) | 5)
    for e in idx:
        blk = OQ.philox4x32_10(np.array([[e // 4, 0, 0, 0]], dtype=np.uint32), (5, 7))[0]
        assert int(words[e]) == int(blk[e % 4])
    # 64-bit element indices reach the second counter word
    big = np.array([(1 << 34) + 6], dtype=np.uint64)
    blk = OQ.philox4x32_10(np.array([[((1 << 34) + 6) // 4 & 0xffffffff, ((1 << 34) + 6) // 4 >> 32, 0, 0]], dtype=np.uint32), (5, 7))[0]
    assert int(OQ.random_words(big, (7 << 32) | 5)[0]) == int(blk[2])


@pytest.mark.parametrize("s", [0, 1, 2, 5, 11, 16])
def test_integer_rounding_modes_against_exact_rationals(s):
    acc = np.arange(-(1 << 12), (1 << 12) + 1, dtype=np.int64)
    if s > 10:
        acc = acc * 37 + 11
    import math
    want = {OQ.FLOOR: [math.floor(Fraction(int(a), 1 << s)) for a in acc],
            OQ.CEIL: [math.ceil(Fraction(int(a), 1 << s)) for a in acc],
            OQ.NEAREST: [math.floor(Fraction(int(a), 1 << s) + Fraction(1, 2)) for a in acc]}
    for mode, w in want.items():
        assert OQ.rshift_mode(acc, s, mode).tolist() == w
    # the nearest mode is the library-wide requantization rule
    assert np.array_equal(OQ.rshift_mode(acc, s, OQ.NEAREST), O.rshift_round(acc, s))
    # stochastic: always one of the two neighbours, exact multiples unchanged, reproducible, seed-dependent
    idx = np.arange(acc.size)
    st = OQ.rshift_mode(acc, s, OQ.STOCHASTIC, seed=99, index=idx)
    assert np.all((st == want[OQ.FLOOR]) | (st == want[OQ.CEIL]))
    exact = (acc % (1 << s)) == 0
    assert np.array_equal(st[exact], np.array(want[OQ.FLOOR])[exact])
    assert np.array_equal(st, OQ.rshift_mode(acc, s, OQ.STOCHASTIC, seed=99, index=idx))
    if s >= 2:
        assert not np.array_equal(st, OQ.rshift_mode(acc, s, OQ.STOCHASTIC, seed=100, index=idx))


@pytest.mark.parametrize("s", [29, 30, 31])
def test_integer_rounding_modes_near_the_int32_limits(s):
    """Accumulators close to +-2^31 with shifts close to 31: acc + addend leaves int32 there, the
    quotient does not, and the oracle (int64) must still equal the exact rationals."""
    import math
    edge = [-(1 << 31) + 1, -(1 << 31) + 2, -(1 << 30) - 1, -(1 << 30), -(1 << 30) + 1, -3, -1, 0, 1, 2, 3,
            (1 << 30) - 1, 1 << 30, (1 << 30) + 1, (1 << 31) - 2, (1 << 31) - 1]
    g = np.random.default_rng(31 + s)
    acc = np.array(edge + g.integers(-(1 << 31) + 1, 1 << 31, 500).tolist(), dtype=np.int64)
    fl = [math.floor(Fraction(int(a), 1 << s)) for a in acc]
    ce = [math.ceil(Fraction(int(a), 1 << s)) for a in acc]
    assert OQ.rshift_mode(acc, s, OQ.FLOOR).tolist() == fl
    assert OQ.rshift_mode(acc, s, OQ.CEIL).tolist() == ce
    assert OQ.rshift_mode(acc, s, OQ.NEAREST).tolist() == [math.floor(Fraction(int(a), 1 << s) + Fraction(1, 2)) for a in acc]
    st = OQ.rshift_mode(acc, s, OQ.STOCHASTIC, seed=3, index=np.arange(acc.size))
    assert np.all((st == fl) | (st == ce))
    assert OQ.rshift_mode(np.array([1]), 31, OQ.CEIL).tolist() == [1]      # (a 32-bit add would wrap to -1)


def test_stochastic_rounding_is_unbiased():
    # acc / 2^s = 2.25: rounds to 3 with probability 1/4 (over element indices, one seed)
    s, acc = 4, 36
    n = 200_000
    got = OQ.rshift_mode(np.full(n, acc, dtype=np.int64), s, OQ.STOCHASTIC, seed=3, index=np.arange(n))
    assert set(np.unique(got)) == {2, 3}
    assert abs(got.mean() - 2.25) < 4 * np.sqrt(0.25 * 0.75 / n)
    x = np.full(n, 2.25 / 64, dtype=np.float32)          # float path: x / rho * 2^(beta-sigma) = 2.25 for rho = 2
    codes = OQ.quantize_codes(x, 2.0, 8, 1, OQ.STOCHASTIC, seed=3)
    assert set(np.unique(codes)) == {2.0, 3.0}
    assert abs(codes.mean() - 2.25) < 4 * np.sqrt(0.25 * 0.75 / n)


@pytest.mark.parametrize("mode", [OQ.NEAREST, OQ.FLOOR, OQ.CEIL])
def test_Q_with_power_of_two_range_is_the_integer_shift(mode):
    """For integer-valued x and rho = 2^e the float formula collapses to x * 2^(beta-sigma-e): a shift
    by s = e - (beta - sigma), which is exactly what the realized conv's requantization computes."""
    rng = np.random.default_rng(5)
    x = rng.integers(-60000, 60000, 5000).astype(np.float32)
    for e in (7, 9, 12, 16):
        s = e - 7
        want = np.clip(OQ.rshift_mode(x.astype(np.int64), s, mode), -127, 127).astype(np.int8)
        assert np.array_equal(OQ.Q(x, 2.0 ** e, 8, 1, mode), want)


def test_simQ_properties():
    rng = np.random.default_rng(6)
    x = (rng.standard_normal(4000) * 3).astype(np.float32)
    for rho, beta in ((4.0, 8), (1.0, 8), (6.5, 8), (8.0, 4)):
        y = OQ.simQ(x, beta, 1, rho)
        step = np.float32(rho) / np.float32(2 ** (beta - 1))
        lim = np.float32(rho) * np.float32(2 ** (beta - 1) - 1) / np.float32(2 ** (beta - 1))
        assert np.all(np.abs(y) <= lim * (1 + 1e-6))                     # clipped to the symmetric range
        inside = np.abs(x) < lim
        assert np.all(np.abs(y[inside] - x[inside]) <= step * 0.5 * (1 + 1e-5))   # nearest: within half a step
        assert np.array_equal(OQ.simQ(y, beta, 1, rho), y)               # idempotent: y is representable
        assert np.all(np.diff(OQ.simQ(np.sort(x), beta, 1, rho)) >= 0)   # monotone
        codes = OQ.quantize_codes(x, rho, beta, 1)
        assert np.array_equal(codes, np.round(codes)) and codes.max() <= 2 ** (beta - 1) - 1
        # floor <= nearest <= ceil, ceil - floor in {0, 1}
        f, c = OQ.quantize_codes(x, rho, beta, 1, OQ.FLOOR), OQ.quantize_codes(x, rho, beta, 1, OQ.CEIL)
        assert np.all(f <= codes) and np.all(codes <= c) and np.all(c - f <= 1)
    # ties go toward +infinity, as in the integer path: 2.5 -> 3, -2.5 -> -2
    assert OQ.quantize_codes(np.array([2.5, -2.5, 0.5, -0.5], dtype=np.float32) / 64, 2.0, 8, 1).tolist() == [3, -2, 1, 0]


def test_qconv_modes_reduce_to_the_plain_requant_and_bracket_it():
    rng = np.random.default_rng(8)
    x = rng.integers(-127, 128, (2, 16, 6, 7)).astype(np.int8)
    w = rng.integers(-127, 128, (8, 16, 3, 3)).astype(np.int8)
    res = rng.integers(-127, 128, (2, 8, 6, 7)).astype(np.int8)
    kw = dict(stride=(1, 1), pad=(1, 1), residual=res, residual_lshift=9, out_rshift=11)
    base = O.qconv2d_requant(x, w, **kw)
    assert np.array_equal(OQ.qconv2d_requant_mode(x, w, mode=OQ.NEAREST, **kw), base)
    fl = OQ.qconv2d_requant_mode(x, w, mode=OQ.FLOOR, **kw).astype(int)
    ce = OQ.qconv2d_requant_mode(x, w, mode=OQ.CEIL, **kw).astype(int)
    st = OQ.qconv2d_requant_mode(x, w, mode=OQ.STOCHASTIC, seed=77, **kw).astype(int)
    assert np.all(fl <= base) and np.all(base <= ce) and np.all(ce - fl <= 1)
    assert np.all((st == fl) | (st == ce)) and np.any(st != fl) and np.any(st != ce)
    # the stochastic draw is indexed by the NHWC position of the output element
    acc = O.conv2d_int(x, w, (1, 1), (1, 1)) + (res.astype(np.int64) << 9)
    n, k, p, q = 1, 5, 3, 2
    e = ((n * 6 + p) * 7 + q) * 8 + k
    u = int(OQ.random_words(np.array([e]), 77)[0]) & ((1 << 11) - 1)
    assert st[n, k, p, q] == max(-127, min(127, (int(acc[n, k, p, q]) + u) >> 11))


def test_unsigned_target_type():
    """sigma = 0: an unsigned type.  For x >= 0 an unsigned beta-bit code is the signed (beta+1)-bit
    code (same scale 2^beta, same upper clip 2^beta - 1); negative values clip to 0; the top code
    is 2^beta - 1; simQ returns values on the grid rho / 2^beta."""
    rng = np.random.default_rng(71)
    for rho, beta in ((4.0, 8), (1.0, 7), (6.5, 4)):
        x = rng.uniform(-0.5 * rho, 1.5 * rho, size=4000).astype(np.float32)
        for mode in (OQ.NEAREST, OQ.FLOOR, OQ.CEIL, OQ.STOCHASTIC):
            u = OQ.quantize_codes(x, rho, beta, 0, mode, seed=9)
            s = OQ.quantize_codes(x, rho, beta + 1, 1, mode, seed=9)
            assert np.array_equal(u[x >= 0], s[x >= 0])
            assert (u[x < -rho / 2 ** beta] == 0).all() and u.min() == 0 and u.max() == 2 ** beta - 1
        q = OQ.Q(x, rho, beta, 0)
        assert q.dtype == np.uint8 and int(q.max()) == 2 ** beta - 1
        y = OQ.simQ(x, beta, 0, rho)
        assert y.min() == 0 and np.array_equal(OQ.simQ(y, beta, 0, rho), y)
        assert np.allclose(y / (np.float32(rho) / np.float32(2 ** beta)), np.round(y / (np.float32(rho) / np.float32(2 ** beta))))
    # hand values: rho = 2, beta = 3 -> scale 4, codes 0..7
    assert OQ.Q(np.array([-1.0, 0.0, 0.12, 0.13, 0.9, 1.7, 1.8, 5.0], np.float32), 2.0, 3, 0).tolist() == [0, 0, 0, 1, 4, 7, 7, 7]

"""Pins of the oracle for the further quantization schemes (paper Section 4.2 and the 8/16, 16/32
rows of the accuracy table of Section 5.4): exact rationals, reductions to the power-of-two form,
brute force on tiny shapes, hand-worked saturation, and the zero-point identity of unsigned inputs."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle as O
from oracle import schemes as S


@pytest.mark.parametrize("M,s", [(1 << 30, 0), (1 << 30, 7), ((1 << 31) - 1, 0), (1518500250, 3), (1 << 30 | 12345, 31), (1, 0), (3, 1)])
def test_scaled_requant_against_exact_rationals(M, s):
    acc = np.concatenate([np.arange(-3000, 3001), np.array([-(2 ** 31) + 1, -(2 ** 30), 2 ** 30, 2 ** 31 - 1]),
                          np.random.default_rng(M % 1000 + s).integers(-(2 ** 31) + 1, 2 ** 31, 400)]).astype(np.int64)
    want = [math.floor(Fraction(int(a) * M, 1 << (31 + s)) + Fraction(1, 2)) for a in acc]
    assert S.requant_scaled(acc.reshape(1, 1, -1, 1), M, s).ravel().tolist() == want


@pytest.mark.parametrize("s", [0, 1, 5, 12, 30])
def test_scaled_requant_with_half_scale_is_the_shift_form(s):
    """M = 2^30 is the scale 1/2: round(acc / 2^(s+1)), the library's power-of-two requantization."""
    acc = np.random.default_rng(s).integers(-(2 ** 31) + 1, 2 ** 31, 2000).astype(np.int64)
    assert np.array_equal(S.requant_scaled(acc.reshape(1, 1, -1, 1), 1 << 30, s).ravel(), O.rshift_round(acc, s + 1))


def test_scaled_requant_per_channel():
    acc = np.random.default_rng(3).integers(-10 ** 6, 10 ** 6, (2, 3, 4, 5)).astype(np.int64)
    M, s = [1 << 30, 1518500250, (1 << 31) - 1], [3, 0, 9]
    got = S.requant_scaled(acc, M, s)
    for k in range(3):
        assert np.array_equal(got[:, k], S.requant_scaled(acc[:, k:k + 1], M[k], s[k])[:, 0])


@pytest.mark.parametrize("scale", [0.5, 0.75, 1e-3, 0.3333333, 2.0 ** -20, 0.99999999999, 2.0 ** -31 * 1.5])
def test_quantize_multiplier_decomposition(scale):
    M, s = S.quantize_multiplier(scale)
    assert (1 << 30) <= M < (1 << 31) and 0 <= s <= 31
    assert abs(Fraction(M, 1 << (31 + s)) - Fraction(scale)) <= Fraction(scale) * Fraction(1, 1 << 30)
    if scale == 0.5:
        assert (M, s) == (1 << 30, 0)


def test_scaled_conv_is_the_shift_conv_for_power_of_two_scales():
    g = np.random.default_rng(5)
    x = g.integers(-127, 128, (2, 6, 7, 5)).astype(np.int8)
    w = g.integers(-127, 128, (4, 6, 3, 3)).astype(np.int8)
    b = g.integers(-3000, 3000, 4).astype(np.int32)
    r = g.integers(-127, 128, (2, 4, 7, 5)).astype(np.int8)
    for s in (1, 6, 11):
        a = S.qconv2d_requant_scaled(x, w, stride=(1, 1), pad=(1, 1), bias=b, residual=r, residual_lshift=4, mult=1 << 30, rshift=s - 1, relu_flag=True)
        c = O.qconv2d_requant(x, w, stride=(1, 1), pad=(1, 1), bias=b, residual=r, residual_lshift=4, out_rshift=s, relu_flag=True)
        assert np.array_equal(a, c)


def test_acc16_saturates_by_hand_and_equals_8_32_when_it_fits():
    # 1x1 conv with one weight: acc = x * w.  100*127 = 12700 fits; two channels of 127*127 = 32258 > 32767: saturates
    x = np.array([100, -100], dtype=np.int8).reshape(1, 1, 1, 2)
    w = np.array([127], dtype=np.int8).reshape(1, 1, 1, 1)
    assert S.qconv2d_requant_acc16(x, w, out_rshift=7).ravel().tolist() == [99, -99]          # 12700/128 = 99.2
    x2 = np.full((1, 2, 1, 1), 127, dtype=np.int8)
    w2 = np.full((1, 2, 1, 1), 127, dtype=np.int8)                                              # exact sum 32258
    assert S.qconv2d_requant_acc16(x2, w2, out_rshift=8).ravel().tolist() == [126]              # 32258/256 = 126.0
    x3 = np.full((1, 3, 1, 1), 127, dtype=np.int8)
    w3 = np.full((1, 3, 1, 1), 127, dtype=np.int8)                                              # exact sum 48387 -> 32767
    assert S.qconv2d_requant_acc16(x3, w3, out_rshift=8).ravel().tolist() == [127]              # 32767/256 = 127.99 -> 128 -> clip 127
    assert S.qconv2d_requant_acc16(x3, -w3, out_rshift=9).ravel().tolist() == [-64]             # -32768/512 = -64
    assert not S.fits_int16(x3, w3) and S.fits_int16(x2, w2)
    g = np.random.default_rng(6)
    xs = g.integers(-7, 8, (2, 16, 6, 6)).astype(np.int8)
    ws = g.integers(-7, 8, (5, 16, 3, 3)).astype(np.int8)
    assert S.fits_int16(xs, ws, pad=(1, 1))
    assert np.array_equal(S.qconv2d_requant_acc16(xs, ws, pad=(1, 1), out_rshift=4, relu_flag=True),
                          O.qconv2d_requant(xs, ws, pad=(1, 1), out_rshift=4, relu_flag=True))


def _brute(x, w, stride, pad):
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    ho, wo = O.out_hw(h, r, stride, pad), O.out_hw(wd, s, stride, pad)
    y = np.zeros((n, k, ho, wo), dtype=object)
    for nn in range(n):
        for kk in range(k):
            for p in range(ho):
                for q in range(wo):
                    t = 0
                    for cc in range(c):
                        for rr in range(r):
                            for ss in range(s):
                                ih, iw = p * stride - pad + rr, q * stride - pad + ss
                                if 0 <= ih < h and 0 <= iw < wd:
                                    t += int(x[nn, cc, ih, iw]) * int(w[kk, cc, rr, ss])
                    y[nn, kk, p, q] = t
    return y


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
def test_i16_and_u8_convs_against_brute_force(stride, pad):
    g = np.random.default_rng(7 + stride)
    x16 = g.integers(-3000, 3000, (1, 3, 5, 6)).astype(np.int16)
    w16 = g.integers(-3000, 3000, (2, 3, 3, 3)).astype(np.int16)
    b = g.integers(-10 ** 6, 10 ** 6, 2).astype(np.int64)
    acc = _brute(x16, w16, stride, pad)
    want = np.array([[max(-32767, min(32767, (int(v) + int(b[k]) + (1 << 9)) >> 10)) for v in acc[0, k].ravel()] for k in range(2)])
    got = S.qconv2d_requant_i16(x16, w16, stride=(stride, stride), pad=(pad, pad), bias=b, out_rshift=10)
    assert got.dtype == np.int16 and np.array_equal(got.reshape(2, -1), want)
    xu = g.integers(0, 256, (1, 3, 5, 6)).astype(np.uint8)
    w8 = g.integers(-127, 128, (2, 3, 3, 3)).astype(np.int8)
    accu = _brute(xu, w8, stride, pad)
    wantu = np.array([[max(0, min(255, (int(v) + (1 << 6)) >> 7)) for v in accu[0, k].ravel()] for k in range(2)])
    gotu = S.qconv2d_requant_u8(xu, w8, stride=(stride, stride), pad=(pad, pad), out_rshift=7, out_unsigned=True)
    assert gotu.dtype == np.uint8 and np.array_equal(gotu.reshape(2, -1), wantu)


def test_unsigned_input_is_a_signed_conv_plus_a_zero_point_term():
    """x_u = x_s + 128 with the border of the padded tensor at x_s = -128 (the code of the unsigned zero):
    conv_u(x_u, w) = conv_s(padded x_s, w, no padding) + 128 * sum(w[k]) -- the identity a signed
    matrix unit uses to take unsigned activations."""
    g = np.random.default_rng(9)
    xu = g.integers(0, 256, (2, 5, 6, 7)).astype(np.uint8)
    w8 = g.integers(-127, 128, (3, 5, 3, 3)).astype(np.int8)
    xs = np.full((2, 5, 8, 9), -128, dtype=np.int8)
    xs[:, :, 1:-1, 1:-1] = (xu.astype(np.int16) - 128).astype(np.int8)
    zp = 128 * w8.astype(np.int64).sum(axis=(1, 2, 3))
    for s, relu in ((9, True), (0, False)):
        a = S.qconv2d_requant_u8(xu, w8, stride=(1, 1), pad=(1, 1), out_rshift=s, relu_flag=relu)
        c = O.qconv2d_requant(xs, w8, stride=(1, 1), pad=(0, 0), bias=zp, out_rshift=s, relu_flag=relu)
        assert np.array_equal(a, c)

"""CPU oracle -- TEST INFRASTRUCTURE ONLY: the quantization schemes of the paper's generic flow beyond
8-bit signed with power-of-two scales (Section 4.2: a scheme chooses its integer types, signed or
unsigned, and how the realized operator scales, "multiplication and rounding"; the accuracy table
of Section 5.4 lists 8/16 and 16/32 beside 8/32, "m/n" = m-bit multiplies accumulated in n bits).

Everything here is exact integer arithmetic on int64 (asserted not to overflow) over the exact
sums of the plain loop nests.  Readings fixed here, the paper leaves them open:
  * a general scale is a positive 32-bit multiplier M and a shift s: q = round(acc * M / 2^(31+s)),
    ties toward +infinity like every rounding of this library; per output channel;
  * n = 16: the accumulator of the scheme is an int16, and the value handed to the requantization is
    the exact sum saturated to [-32768, 32767] (equal to a true 16-bit accumulation whenever that
    does not overflow, which is the scheme's precondition; defined beyond it);
  * 16/32: int16 activations and filters, exact sums that must fit int32, codes clipped to +-32767;
  * unsigned activations: codes 0..255, zero padding is the code 0; an unsigned result is clipped to
    [0, 255] (which contains the relu).
"""
from __future__ import annotations

import math

import numpy as np

from . import conv2d, out_hw


def _exact_conv(x, w, stride, pad) -> np.ndarray:
    """Exact integer sums of a conv over integer arrays of any width (fp64 is exact below 2^53)."""
    x = np.asarray(x)
    w = np.asarray(w)
    bound = float(np.abs(x.astype(np.int64)).max(initial=0)) * float(np.abs(w.astype(np.int64)).max(initial=0)) * w[0].size
    assert bound < 2.0 ** 52
    return np.rint(conv2d(x.astype(np.float64), w.astype(np.float64), stride, pad)).astype(np.int64)


def quantize_multiplier(scale: float):
    """(M, s) with scale = M / 2^31 * 2^-s, 2^30 <= M < 2^31 (M rounded to nearest), 0 <= s <= 31; 2^-32 < scale < 1."""
    assert scale > 0
    m, e = math.frexp(scale)              # scale = m * 2^e, 0.5 <= m < 1
    M = int(math.floor(m * 2.0 ** 31 + 0.5))
    if M == 1 << 31:                      # m rounded up to 1.0
        M, e = 1 << 30, e + 1
    s = -e
    if s == -1 and scale < 1.0:           # so close to 1 that M rounded up to 2^31: the largest representable scale
        M, s = (1 << 31) - 1, 0
    assert 0 <= s <= 31, "scale outside (2^-32, 1)"
    return M, s


def requant_scaled(acc, mult, rshift) -> np.ndarray:
    """round(acc * M / 2^(31+s)), ties toward +infinity; mult, rshift scalars or arrays broadcast on axis 1."""
    a = np.asarray(acc, dtype=np.int64)
    M = np.asarray(mult, dtype=np.int64)
    s = np.asarray(rshift, dtype=np.int64)
    if M.ndim == 1:
        shape = [1] * a.ndim
        shape[1] = -1
        M, s = M.reshape(shape), s.reshape(shape)
    assert np.all(M > 0) and np.all(M < 2 ** 31) and np.all(s >= 0) and np.all(s <= 31)
    assert np.all(np.abs(a) < 2 ** 31)
    sh = np.int64(31) + s
    return np.floor_divide(a * M + (np.int64(1) << (sh - np.int64(1))), np.int64(1) << sh)


def _tail(acc, bias, residual, residual_lshift):
    if bias is not None:
        acc = acc + np.asarray(bias, dtype=np.int64).reshape(1, -1, 1, 1)
    if residual is not None:
        acc = acc + np.asarray(residual, dtype=np.int64) * (1 << int(residual_lshift))
    return acc


def _finish(q, relu_flag, lo, hi, dtype):
    q = np.clip(q, lo, hi)
    if relu_flag:
        q = np.maximum(q, 0)
    return q.astype(dtype)


def qconv2d_requant_scaled(x, w, *, stride=(1, 1), pad=(0, 0), bias=None, residual=None, residual_lshift=0,
                           mult=1 << 30, rshift=0, relu_flag=False) -> np.ndarray:
    """int8 conv, exact sum -> [bias] -> [+res*2^l] -> round(acc*M[k]/2^(31+s[k])) -> clip +-127 -> [relu]."""
    acc = _tail(_exact_conv(np.asarray(x, dtype=np.int8), np.asarray(w, dtype=np.int8), stride, pad), bias, residual, residual_lshift)
    assert np.all(np.abs(acc) < 2 ** 31)
    return _finish(requant_scaled(acc, mult, rshift), relu_flag, -127, 127, np.int8)


def fits_int16(x, w, *, stride=(1, 1), pad=(0, 0), bias=None, residual=None, residual_lshift=0) -> bool:
    acc = _tail(_exact_conv(x, w, stride, pad), bias, residual, residual_lshift)
    return bool(np.all((acc >= -32768) & (acc <= 32767)))


def qconv2d_requant_acc16(x, w, *, stride=(1, 1), pad=(0, 0), bias=None, residual=None, residual_lshift=0, out_rshift=0,
                          relu_flag=False) -> np.ndarray:
    """The 8/16 scheme: the exact sum saturated to int16, then round-shift, clip +-127, [relu]."""
    acc = _tail(_exact_conv(np.asarray(x, dtype=np.int8), np.asarray(w, dtype=np.int8), stride, pad), bias, residual, residual_lshift)
    acc = np.clip(acc, -32768, 32767)
    q = acc if out_rshift == 0 else np.floor_divide(acc + (1 << (out_rshift - 1)), 1 << out_rshift)
    return _finish(q, relu_flag, -127, 127, np.int8)


def qconv2d_requant_i16(x, w, *, stride=(1, 1), pad=(0, 0), bias=None, out_rshift=0, relu_flag=False) -> np.ndarray:
    """The 16/32 scheme: int16 x int16, exact sums that fit int32 -> [bias] -> round-shift -> clip +-32767 -> [relu]."""
    x = np.asarray(x)
    w = np.asarray(w)
    assert x.dtype == np.int16 and w.dtype == np.int16
    acc = _tail(_exact_conv(x, w, stride, pad), bias, None, 0)
    assert np.all(np.abs(acc) < 2 ** 31), "precondition of the 16/32 scheme: sums fit int32"
    q = acc if out_rshift == 0 else np.floor_divide(acc + (1 << (out_rshift - 1)), 1 << out_rshift)
    return _finish(q, relu_flag, -32767, 32767, np.int16)


def qconv2d_requant_u8(x, w, *, stride=(1, 1), pad=(0, 0), bias=None, out_rshift=0, relu_flag=False,
                       out_unsigned=False) -> np.ndarray:
    """Unsigned 8-bit activations (codes 0..255, zero padding = code 0) with signed 8-bit filters."""
    x = np.asarray(x)
    assert x.dtype == np.uint8
    acc = _tail(_exact_conv(x, np.asarray(w, dtype=np.int8), stride, pad), bias, None, 0)
    assert np.all(np.abs(acc) < 2 ** 31)
    q = acc if out_rshift == 0 else np.floor_divide(acc + (1 << (out_rshift - 1)), 1 << out_rshift)
    if out_unsigned:
        return _finish(q, False, 0, 255, np.uint8)
    return _finish(q, relu_flag, -127, 127, np.int8)

"""CPU oracle -- TEST INFRASTRUCTURE ONLY (tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product path never does).

Python face of ``oracle.c``: the unfused operators as plain loops in double / int64, and
the fused primitive functions written as nothing more than those operators called one
after another (paper, Section 4.1: a fused group is the original expression factored
into a function, so its value is that of the unfused sequence; Section 4.2: the realized
quantize operator Q = cast(clip(round(x * 2^(-s)))) expands into ordinary elementwise
operators behind the convolution).

All tensors are numpy, NCHW / OIHW.  Floating-point inputs of any width are widened to
double exactly; results come back as double (or int64) and are narrowed only by the
explicit ``cast_*`` step, which uses numpy's round-to-nearest-even conversion.

Readings of the paper fixed here (the paper leaves them open):
  * conv2d is cross-correlation (no kernel flip), dilation 1, zero padding;
  * epilogue order: conv -> bias -> scale*x+shift -> +residual -> relu -> cast;
  * ``round`` is to nearest with ties toward +infinity (add half, floor-divide);
  * ``clip`` is to [-127, 127]; the residual enters the accumulator as res * 2^l before
    the single rounding.
The tie rule and the residual alignment are conventions of this library, not recoverable
from the paper: on those two points parity is pinned by this file's definition only.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SRC = os.path.join(_HERE, "oracle.c")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (host only)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", _SO, _SRC]
        subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
        _lib.oracle_cast_i8.restype = C.c_size_t
        _lib.oracle_count_outside_i32.restype = C.c_size_t
    return _lib


def num_threads() -> int:
    """Host threads the conv / dense loop nests use (OpenMP over independent outputs)."""
    return int(lib().oracle_num_threads())


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def out_hw(h: int, r: int, stride: int, pad: int) -> int:
    """Ho = floor((H + 2*pad - R)/stride) + 1."""
    return (h + 2 * pad - r) // stride + 1


# ----------------------------------------------------------------------------- unfused ops
def conv2d(x, w, stride: Tuple[int, int] = (1, 1), pad: Tuple[int, int] = (0, 0)) -> np.ndarray:
    x, w = _f64(x), _f64(w)
    n, c, h, wd = x.shape
    k, c2, r, s = w.shape
    assert c == c2
    ho, wo = out_hw(h, r, stride[0], pad[0]), out_hw(wd, s, stride[1], pad[1])
    y = np.empty((n, k, ho, wo), dtype=np.float64)
    lib().oracle_conv2d_f64(_p(x), _p(w), _p(y), n, c, h, wd, k, r, s,
                            stride[0], stride[1], pad[0], pad[1], ho, wo)
    return y


def conv2d_int(x, w, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """int8 x int8 -> exact int64 sums."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    w = np.ascontiguousarray(w, dtype=np.int8)
    n, c, h, wd = x.shape
    k, c2, r, s = w.shape
    assert c == c2
    ho, wo = out_hw(h, r, stride[0], pad[0]), out_hw(wd, s, stride[1], pad[1])
    y = np.empty((n, k, ho, wo), dtype=np.int64)
    lib().oracle_conv2d_i8(_p(x), _p(w), _p(y), n, c, h, wd, k, r, s,
                           stride[0], stride[1], pad[0], pad[1], ho, wo)
    return y


def dwconv2d(x, w, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    x, w = _f64(x), _f64(w)
    n, c, h, wd = x.shape
    c2, r, s = w.shape
    assert c == c2
    ho, wo = out_hw(h, r, stride[0], pad[0]), out_hw(wd, s, stride[1], pad[1])
    y = np.empty((n, c, ho, wo), dtype=np.float64)
    lib().oracle_dwconv2d_f64(_p(x), _p(w), _p(y), n, c, h, wd, r, s,
                              stride[0], stride[1], pad[0], pad[1], ho, wo)
    return y


def dense(x, w) -> np.ndarray:
    x, w = _f64(x), _f64(w)
    m, kin = x.shape
    nout, kin2 = w.shape
    assert kin == kin2
    y = np.empty((m, nout), dtype=np.float64)
    lib().oracle_dense_f64(_p(x), _p(w), _p(y), m, nout, kin)
    return y


def _nkhw(y: np.ndarray) -> Tuple[int, int, int]:
    n, k = y.shape[0], y.shape[1]
    hw = int(np.prod(y.shape[2:])) if y.ndim > 2 else 1
    return n, k, hw


def bias_add(y: np.ndarray, b) -> np.ndarray:
    y = _f64(y).copy()
    b = _f64(b)
    n, k, hw = _nkhw(y)
    assert b.shape == (k,)
    lib().oracle_bias_add_f64(_p(y), _p(b), n, k, hw)
    return y


def scale_shift(y: np.ndarray, scale, shift) -> np.ndarray:
    y = _f64(y).copy()
    scale, shift = _f64(scale), _f64(shift)
    n, k, hw = _nkhw(y)
    assert scale.shape == (k,) and shift.shape == (k,)
    lib().oracle_scale_shift_f64(_p(y), _p(scale), _p(shift), n, k, hw)
    return y


def fold_bn(gamma, beta, mean, var, eps: float):
    """Unfolded batch norm (inference) -> (scale, shift): scale = g/sqrt(var+eps), shift = b - mean*scale."""
    gamma, beta, mean, var = _f64(gamma), _f64(beta), _f64(mean), _f64(var)
    scale = gamma / np.sqrt(var + eps)
    return scale, beta - mean * scale


def add(y: np.ndarray, other) -> np.ndarray:
    y = _f64(y).copy()
    other = _f64(other)
    assert other.shape == y.shape
    lib().oracle_add_f64(_p(y), _p(other), C.c_size_t(y.size))
    return y


def relu(y: np.ndarray) -> np.ndarray:
    y = _f64(y).copy()
    lib().oracle_relu_f64(_p(y), C.c_size_t(y.size))
    return y


def cast_f16(y: np.ndarray) -> np.ndarray:
    """double -> fp16, round to nearest even (numpy converts directly, one rounding)."""
    return np.asarray(y, dtype=np.float64).astype(np.float16)


def cast_f32(y: np.ndarray) -> np.ndarray:
    return np.asarray(y, dtype=np.float64).astype(np.float32)


def maxpool2d(x, r: int, stride: int, pad: int) -> np.ndarray:
    x = _f64(x)
    n, c, h, w = x.shape
    ho, wo = out_hw(h, r, stride, pad), out_hw(w, r, stride, pad)
    y = np.empty((n, c, ho, wo), dtype=np.float64)
    lib().oracle_maxpool2d_f64(_p(x), _p(y), n, c, h, w, r, stride, pad, ho, wo)
    return y


def global_avgpool(x) -> np.ndarray:
    x = _f64(x)
    n, c, h, w = x.shape
    y = np.empty((n, c), dtype=np.float64)
    lib().oracle_global_avgpool_f64(_p(x), _p(y), n, c, h * w)
    return y


# ----------------------------------------------------------------------- integer operators
def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int64)


def bias_add_int(y, b) -> np.ndarray:
    y = _i64(y).copy()
    b = _i64(b)
    n, k, hw = _nkhw(y)
    assert b.shape == (k,)
    lib().oracle_bias_add_i64(_p(y), _p(b), n, k, hw)
    return y


def add_lshift_int(y, res_i8, lshift: int) -> np.ndarray:
    assert lshift >= 0
    y = _i64(y).copy()
    res = np.ascontiguousarray(res_i8, dtype=np.int8)
    assert res.shape == y.shape
    lib().oracle_add_lshift_i64(_p(y), _p(res), int(lshift), C.c_size_t(y.size))
    return y


def rshift_round(y, s: int) -> np.ndarray:
    """round(y / 2^s), ties toward +infinity; s = 0 returns y."""
    assert 0 <= s <= 31
    y = _i64(y).copy()
    lib().oracle_rshift_round_i64(_p(y), int(s), C.c_size_t(y.size))
    return y


def clip_int(y, lo: int = -127, hi: int = 127) -> np.ndarray:
    y = _i64(y).copy()
    lib().oracle_clip_i64(_p(y), C.c_int64(lo), C.c_int64(hi), C.c_size_t(y.size))
    return y


def relu_int(y) -> np.ndarray:
    y = _i64(y).copy()
    lib().oracle_relu_i64(_p(y), C.c_size_t(y.size))
    return y


def cast_i8(y) -> np.ndarray:
    y = _i64(y)
    out = np.empty(y.shape, dtype=np.int8)
    bad = lib().oracle_cast_i8(_p(y), _p(out), C.c_size_t(y.size))
    if bad:
        raise OverflowError(f"{bad} values do not fit int8")
    return out


def assert_fits_i32(y) -> None:
    y = _i64(y)
    bad = lib().oracle_count_outside_i32(_p(y), C.c_size_t(y.size))
    if bad:
        raise OverflowError(f"{bad} accumulators do not fit int32 (precondition of the quantized path)")


# ------------------------------------------------------------- fused primitive functions
def fused_conv2d(x, w, *, stride=(1, 1), pad=(0, 0), bias=None, scale=None, shift=None,
                 residual=None, relu_flag=False, out_dtype="f16") -> np.ndarray:
    """conv -> [bias] -> [scale, shift] -> [+residual] -> [relu] -> cast.  Unfused calls only."""
    y = conv2d(x, w, stride, pad)
    if bias is not None:
        y = bias_add(y, bias)
    if scale is not None:
        y = scale_shift(y, scale, shift)
    if residual is not None:
        y = add(y, residual)
    if relu_flag:
        y = relu(y)
    return _narrow(y, out_dtype)


def fused_dwconv2d(x, w, *, stride=(1, 1), pad=(0, 0), bias=None, scale=None, shift=None,
                   relu_flag=False, out_dtype="f16") -> np.ndarray:
    y = dwconv2d(x, w, stride, pad)
    if bias is not None:
        y = bias_add(y, bias)
    if scale is not None:
        y = scale_shift(y, scale, shift)
    if relu_flag:
        y = relu(y)
    return _narrow(y, out_dtype)


def fused_dense(x, w, *, bias=None, relu_flag=False, out_dtype="f16") -> np.ndarray:
    y = dense(x, w)
    if bias is not None:
        y = bias_add(y, bias)
    if relu_flag:
        y = relu(y)
    return _narrow(y, out_dtype)


def qconv2d_requant(x, w, *, stride=(1, 1), pad=(0, 0), bias=None, residual=None,
                    residual_lshift: int = 0, out_rshift: int = 0, relu_flag=False) -> np.ndarray:
    """int8 conv, exact sum -> [bias] -> [+res*2^l] -> round-shift -> clip[-127,127] -> [relu] -> int8."""
    acc = conv2d_int(x, w, stride, pad)
    if bias is not None:
        acc = bias_add_int(acc, bias)
    if residual is not None:
        acc = add_lshift_int(acc, residual, residual_lshift)
    assert_fits_i32(acc)
    q = rshift_round(acc, out_rshift)
    q = clip_int(q, -127, 127)
    if relu_flag:
        q = relu_int(q)
    return cast_i8(q)


def _narrow(y: np.ndarray, out_dtype: str) -> np.ndarray:
    if out_dtype == "f16":
        return cast_f16(y)
    if out_dtype == "f32":
        return cast_f32(y)
    if out_dtype == "f64":
        return y
    raise ValueError(out_dtype)


# -------------------------------------------------- single output elements (large shapes)
def conv2d_points(x, w, points: Sequence[Tuple[int, int, int, int]], stride=(1, 1), pad=(0, 0),
                  integer: bool = False) -> np.ndarray:
    """conv2d outputs at chosen (n, k, p, q), each straight from the definition.

    Used where the whole tensor is too large for the loop nest to finish in seconds.
    """
    x = np.asarray(x)
    w = np.asarray(w)
    n_, c_, h_, w_ = x.shape
    r_, s_ = w.shape[2], w.shape[3]
    out = []
    for (n, k, p, q) in points:
        acc = 0 if integer else 0.0
        for r in range(r_):
            ih = p * stride[0] - pad[0] + r
            if ih < 0 or ih >= h_:
                continue
            for s in range(s_):
                iw = q * stride[1] - pad[1] + s
                if iw < 0 or iw >= w_:
                    continue
                if integer:
                    acc += int(np.dot(x[n, :, ih, iw].astype(np.int64), w[k, :, r, s].astype(np.int64)))
                else:
                    acc += float(np.dot(x[n, :, ih, iw].astype(np.float64), w[k, :, r, s].astype(np.float64)))
        out.append(acc)
    return np.array(out, dtype=np.int64 if integer else np.float64)


def dwconv2d_points(x, w, points, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    x = np.asarray(x)
    w = np.asarray(w)
    h_, w_ = x.shape[2], x.shape[3]
    out = []
    for (n, c, p, q) in points:
        acc = 0.0
        for r in range(w.shape[1]):
            for s in range(w.shape[2]):
                ih, iw = p * stride[0] - pad[0] + r, q * stride[1] - pad[1] + s
                if 0 <= ih < h_ and 0 <= iw < w_:
                    acc += float(x[n, c, ih, iw]) * float(w[c, r, s])
        out.append(acc)
    return np.array(out, dtype=np.float64)


def float_epilogue_points(acc, ks, *, bias=None, scale=None, shift=None, residual=None, relu_flag=False):
    """The float epilogue on a vector of raw sums; ks = output channel of each sum."""
    t = np.asarray(acc, dtype=np.float64).copy()
    ks = np.asarray(ks)
    if bias is not None:
        t = t + _f64(bias)[ks]
    if scale is not None:
        t = t * _f64(scale)[ks]
        t = t + _f64(shift)[ks]
    if residual is not None:
        t = t + _f64(residual)
    if relu_flag:
        t = np.maximum(t, 0.0)
    return t


def requant_points(acc, *, bias=None, ks=None, residual=None, residual_lshift=0, out_rshift=0, relu_flag=False):
    """The quantized epilogue on a vector of exact integer sums (Python big ints)."""
    out = []
    for i, a in enumerate(acc):
        t = int(a)
        if bias is not None:
            t += int(bias[ks[i]])
        if residual is not None:
            t += int(residual[i]) * (1 << residual_lshift)
        if out_rshift > 0:
            t = (t + (1 << (out_rshift - 1))) // (1 << out_rshift)   # Python // floors
        t = max(-127, min(127, t))
        if relu_flag:
            t = max(t, 0)
        out.append(t)
    return np.array(out, dtype=np.int8)


# --------------------------------------------------------------------------- error metric
def max_rel_err(got, ref) -> float:
    """max_i |g_i - r_i| / max(|r_i|, RMS(r)): relative error with the tensor's RMS as floor,
    so that exact zeros behind a relu do not divide by zero."""
    g = np.asarray(got, dtype=np.float64).ravel()
    r = np.asarray(ref, dtype=np.float64).ravel()
    if r.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(r * r)))
    den = np.maximum(np.abs(r), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(g - r) / den))

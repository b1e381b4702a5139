"""Pins of the calibrate / fold / realize oracle (paper Sections 4.2 and 4.4)."""
import numpy as np
import pytest

import oracle as O
from oracle import quant as OQ
from oracle import realize as R
from oracle.stack import run_float, run_quantized
from workloads import inputs, nets


def test_pow2_range():
    assert R.pow2_range(1.0) == 1.0 and R.pow2_range(1.0001) == 2.0 and R.pow2_range(0.75) == 1.0
    assert R.pow2_range(0.5) == 0.5 and R.pow2_range(5.9) == 8.0 and R.pow2_range(0.0) == 2.0 ** -20
    for v in (3e-4, 0.02, 7.0, 129.0):
        r = R.pow2_range(v)
        assert r >= v > r / 2


def test_axis_scale_folding_moves_the_multiply_into_the_filters():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 5, 9, 8))
    w = rng.standard_normal((7, 5, 3, 3))
    sc = rng.standard_normal(7)
    a = O.scale_shift(O.conv2d(x, w, (2, 2), (1, 1)), sc, np.zeros(7))
    b = O.conv2d(x, R.fold_scale(w, sc), (2, 2), (1, 1))
    assert np.max(np.abs(a - b)) <= 1e-12 * np.max(np.abs(a))
    assert R.fold_scale(w, None) is not None and np.array_equal(R.fold_scale(w, None), w)


@pytest.mark.parametrize("with_bias", [False, True])
@pytest.mark.parametrize("with_res", [False, True])
def test_realized_conv_is_exact_on_representable_values(with_res, with_bias):
    """When inputs, folded filters, shift and residual already lie on their 8-bit grids, the integer
    conv with the realized bias and shifts reproduces Q(float result) bit for bit: pins the
    formulas for bias_q, s and l (a wrong power of two or a dropped term changes every output)."""
    rng = np.random.default_rng(2 + with_res)
    rho = {"x": 4.0, "y": 64.0, "r": 16.0}
    xq = rng.integers(-127, 128, (1, 8, 6, 6)).astype(np.int8)
    wq = rng.integers(-127, 128, (4, 8, 3, 3)).astype(np.int8)
    rq = rng.integers(-127, 128, (1, 4, 6, 6)).astype(np.int8)
    rho_w = 0.5
    x = R.dequantize(xq, rho["x"])
    scale = np.array([1.0, 0.5, 0.25, 1.0])                      # powers of two keep w * scale on a grid
    w = R.dequantize(wq, rho_w) / scale.reshape(-1, 1, 1, 1)
    w[0, 0, 0, 0] = 127 * rho_w / 128 / scale[0]                 # the maximum code is present: rho_w is recovered
    unit = rho["x"] * rho_w / 2 ** 14
    shift = rng.integers(-40000, 40000, 4) * unit
    res = R.dequantize(rq, rho["r"])

    class Op:
        kind, name, src, dst, res = "conv", "c", "x", "y", ("r" if with_res else None)
    p = {"w": w, "scale": scale, "shift": shift}
    bias = None
    if with_bias:          # a conv bias in front of the scale: it reaches the accumulator as bias * scale
        bias = rng.integers(-30000, 30000, 4) * unit / scale
        p["bias"] = bias
    qp, sh = R.realize([Op], [p], rho)
    assert np.array_equal(qp[0]["w"][1:], wq[1:]) and qp[0]["w"][0, 0, 0, 0] == 127
    assert sh[0]["s"] == int(np.log2(2 ** 7 * 64.0 / (4.0 * 0.5)))
    # the float operator sequence itself, unfolded: conv -> [bias] -> scale, shift
    y_float = O.conv2d(x, w, (1, 1), (1, 1))
    if with_bias:
        y_float = O.bias_add(y_float, bias)
    y_float = O.scale_shift(y_float, scale, shift)
    if with_res:
        y_float = y_float + res
        assert sh[0]["l"] == int(np.log2(2 ** 7 * 16.0 / (4.0 * 0.5)))
    want = OQ.Q(y_float, rho["y"], 8, 1)
    got = O.qconv2d_requant(xq, qp[0]["w"], stride=(1, 1), pad=(1, 1), bias=qp[0]["bias"],
                            residual=rq if with_res else None, residual_lshift=sh[0]["l"], out_rshift=sh[0]["s"])
    assert np.array_equal(got, want)


def test_realized_block_tracks_the_float_block():
    ops = nets.basic_block(64)
    params = inputs.net_params(ops, 2, "f16")
    x = inputs.image(2, 1, 64, 28, 28, "f16")
    t = run_float(ops, params, x, "f16")
    for global_scale in (False, True):
        rho = R.calibrate(ops, t, global_scale)
        assert all(r >= float(np.max(np.abs(t[n].astype(np.float64)))) for n, r in rho.items())     # no overflow
        if not global_scale:
            assert all(r / 2 < float(np.max(np.abs(t[n].astype(np.float64)))) for n, r in rho.items())
        qp, sh = R.realize(ops, params, rho)
        tq = run_quantized(ops, qp, sh, OQ.Q(x, rho["x"], 8, 1))
        for op in ops:
            ref = t[op.dst].astype(np.float64)
            deq = R.dequantize(tq[op.dst], rho[op.dst])
            sqnr = 10 * np.log10((ref ** 2).sum() / ((deq - ref) ** 2).sum())
            assert sqnr > (25 if not global_scale else 15), (op.name, sqnr)
            assert np.abs(tq[op.dst].astype(int)).max() <= 127

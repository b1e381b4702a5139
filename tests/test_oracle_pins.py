"""Pins of the CPU oracle against things other than itself: hand-worked fixtures, closed
forms, reductions to library routines, brute force and invariants.  No GPU."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(20190408)


def _read_fixture(name):
    rows = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            rows[k] = [float(t) for t in v]
    return rows


# ------------------------------------------------------------------ hand-worked fixtures
def test_handworked_conv_fixture():
    fx = _read_fixture("handworked_conv.txt")
    x = np.array(fx["x"]).reshape(1, 1, 3, 3)
    w = np.array(fx["w"]).reshape(1, 1, 2, 2)
    assert O.conv2d(x, w).ravel().tolist() == fx["y"]
    assert O.conv2d(x, w, (2, 2), (1, 1)).ravel().tolist() == fx["y_pad1_stride2"]
    # the same numbers through the depthwise and point-wise entry points
    assert O.dwconv2d(x, w[0]).ravel().tolist() == fx["y"]
    pts = [(0, 0, p, q) for p in range(2) for q in range(2)]
    assert O.conv2d_points(x, w, pts).tolist() == fx["y"]
    assert O.conv2d_points(x, w, pts, (2, 2), (1, 1)).tolist() == fx["y_pad1_stride2"]
    assert O.conv2d_int(x.astype(np.int8), w.astype(np.int8)).ravel().tolist() == fx["y"]


def test_handworked_requant_fixture():
    with open(os.path.join(GOLD, "handworked_requant.txt")) as f:
        rows = [tuple(int(t) for t in l.split()) for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) >= 12
    for acc, s, rl, want in rows:
        q = O.clip_int(O.rshift_round(np.array([acc]), s))
        if rl:
            q = O.relu_int(q)
        assert int(O.cast_i8(q)[0]) == want, (acc, s, rl)
        assert int(O.requant_points([acc], out_rshift=s, relu_flag=bool(rl))[0]) == want


def test_handworked_float_epilogue_fixture():
    """float_epilogue_points (the expected values of the full-size sampled GPU checks) on values
    worked by hand: order bias -> scale, shift -> residual -> relu, constants indexed by channel."""
    bias, scale, shift = [0.5, -1.0, 2.0], [2.0, 0.5, -1.5], [0.25, -0.75, 1.0]
    with open(os.path.join(GOLD, "handworked_float_epilogue.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) >= 6
    for acc, k, res, rl, want in rows:
        got = O.float_epilogue_points([float(acc)], [int(k)], bias=bias, scale=scale, shift=shift,
                                      residual=[float(res)], relu_flag=bool(int(rl)))
        assert got.tolist() == [float(want)], (acc, k, res, rl)
    # without the optional operands the raw sum passes through
    assert O.float_epilogue_points([1.25, -2.0], [0, 1]).tolist() == [1.25, -2.0]
    assert O.float_epilogue_points([1.25, -2.0], [0, 1], relu_flag=True).tolist() == [1.25, 0.0]


@pytest.mark.parametrize("flags", list(itertools.product([False, True], repeat=4)))
def test_float_epilogue_points_equals_the_loop_nest_operators(flags):
    """On every output element of a small random layer the point-wise path (conv2d_points +
    float_epilogue_points + cast) gives the bits of the whole-tensor fused operator, which is
    nothing but the unfused C loop nests called one after another."""
    has_bias, has_bn, has_res, rl = flags
    g = np.random.default_rng(77 + sum(b << i for i, b in enumerate(flags)))
    x = g.standard_normal((2, 5, 7, 6)).astype(np.float16)
    w = (g.standard_normal((4, 5, 3, 3)) * 0.2).astype(np.float16)
    bias = g.standard_normal(4).astype(np.float32) if has_bias else None
    scale = (1 + 0.1 * g.standard_normal(4)).astype(np.float32) if has_bn else None
    shift = (0.1 * g.standard_normal(4)).astype(np.float32) if has_bn else None
    for stride, pad in (((1, 1), (1, 1)), ((2, 2), (1, 1))):
        ho, wo = O.out_hw(7, 3, stride[0], pad[0]), O.out_hw(6, 3, stride[1], pad[1])
        res = g.standard_normal((2, 4, ho, wo)).astype(np.float16) if has_res else None
        want = O.fused_conv2d(x, w, stride=stride, pad=pad, bias=bias, scale=scale, shift=shift, residual=res,
                              relu_flag=rl, out_dtype="f16")
        pts = [(n, k, p, q) for n in range(2) for k in range(4) for p in range(ho) for q in range(wo)]
        acc = O.conv2d_points(x, w, pts, stride, pad)
        rs = None if res is None else np.array([res[t] for t in pts], dtype=np.float64)
        got = O.cast_f16(O.float_epilogue_points(acc, [t[1] for t in pts], bias=bias, scale=scale, shift=shift,
                                                 residual=rs, relu_flag=rl))
        # the two paths add the taps in different orders: equal up to the last bit of the fp64 sum,
        # which the fp16 rounding hides except at a rounding boundary
        d = np.abs(got.astype(np.float64) - want.reshape(-1).astype(np.float64))
        assert np.all(d <= np.spacing(np.abs(want.reshape(-1)).astype(np.float16)).astype(np.float64))
        assert (d == 0).mean() > 0.99


# -------------------------------------------------------------------------- closed forms
@pytest.mark.parametrize("cin", [1, 3])
def test_all_ones_counts_valid_taps(cin):
    x = np.ones((1, cin, 6, 7))
    w = np.ones((2, cin, 3, 3))
    y = O.conv2d(x, w, (1, 1), (1, 1))
    assert y.shape == (1, 2, 6, 7)
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * cin)
    assert np.all(y[:, :, 0, 1:-1] == 6 * cin) and np.all(y[:, :, 1:-1, 0] == 6 * cin)
    for p, q in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(y[:, :, p, q] == 4 * cin)
    # pad 3 / 7x7 / stride 2 (the ResNet stem geometry): corner sees a 4x4 window
    y7 = O.conv2d(np.ones((1, 1, 10, 10)), np.ones((1, 1, 7, 7)), (2, 2), (3, 3))
    assert y7.shape == (1, 1, 5, 5) and y7[0, 0, 0, 0] == 16 and y7[0, 0, 2, 2] == 49


def test_zero_sum_kernel_kills_constants():
    x = np.full((1, 2, 8, 8), 3.5)
    w = rng.standard_normal((3, 2, 3, 3))
    w -= w.mean(axis=(2, 3), keepdims=True)
    y = O.conv2d(x, w, (1, 1), (1, 1))
    assert np.max(np.abs(y[:, :, 1:-1, 1:-1])) < 1e-12


@pytest.mark.parametrize("r0,s0", [(1, 1), (0, 2), (2, 0), (0, 0)])
def test_delta_kernel_shifts_without_flip(r0, s0):
    c = 3
    x = rng.standard_normal((2, c, 5, 6))
    w = np.zeros((c, c, 3, 3))
    for k in range(c):
        w[k, k, r0, s0] = 1.0
    y = O.conv2d(x, w, (1, 1), (1, 1))
    # y[p,q] = x[p - 1 + r0, q - 1 + s0] with zero fill
    want = np.zeros_like(x)
    dp, dq = r0 - 1, s0 - 1
    for p in range(5):
        for q in range(6):
            if 0 <= p + dp < 5 and 0 <= q + dq < 6:
                want[:, :, p, q] = x[:, :, p + dp, q + dq]
    assert np.array_equal(y, want)
    if (r0, s0) == (1, 1):
        assert np.array_equal(y, x)


# ---------------------------------------------------------- reductions to library routines
def test_1x1_conv_is_a_gemm():
    x = rng.standard_normal((2, 5, 4, 3))
    w = rng.standard_normal((7, 5, 1, 1))
    y = O.conv2d(x, w)
    a = x.transpose(0, 2, 3, 1).reshape(-1, 5)          # [N*H*W, C]
    g = (a @ w.reshape(7, 5).T).reshape(2, 4, 3, 7).transpose(0, 3, 1, 2)
    assert np.allclose(y, g, rtol=0, atol=1e-13)


def test_dense_is_1x1_conv_on_1x1_image_and_matmul():
    x = rng.standard_normal((3, 11))
    w = rng.standard_normal((6, 11))
    y = O.dense(x, w)
    assert np.allclose(y, x @ w.T, atol=1e-13)
    yc = O.conv2d(x.reshape(3, 11, 1, 1), w.reshape(6, 11, 1, 1)).reshape(3, 6)
    assert np.array_equal(y, yc)
    # a transposed weight would not even have this shape; check orientation on a one-hot
    w1 = np.zeros((2, 3)); w1[1, 2] = 1.0
    assert O.dense(np.array([[10., 20., 30.]]), w1).tolist() == [[0.0, 30.0]]


def test_depthwise_is_block_diagonal_dense_conv():
    c = 4
    x = rng.standard_normal((2, c, 7, 6))
    wd = rng.standard_normal((c, 3, 3))
    wf = np.zeros((c, c, 3, 3))
    for i in range(c):
        wf[i, i] = wd[i]
    for st, pd in [(1, 1), (2, 1), (2, 0)]:
        assert np.allclose(O.dwconv2d(x, wd, (st, st), (pd, pd)), O.conv2d(x, wf, (st, st), (pd, pd)), atol=1e-13)


def test_stride2_is_subsampled_stride1():
    x = rng.standard_normal((1, 3, 9, 8))
    w = rng.standard_normal((2, 3, 3, 3))
    y1 = O.conv2d(x, w, (1, 1), (1, 1))
    y2 = O.conv2d(x, w, (2, 2), (1, 1))
    assert np.array_equal(y2, y1[:, :, ::2, ::2])
    y12 = O.conv2d(x, w, (1, 2), (1, 1))                 # mixed strides pin the h/w roles
    assert np.array_equal(y12, y1[:, :, :, ::2])


def _im2col_matmul(x, w, st, pd):
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    ho, wo = (h + 2 * pd - r) // st + 1, (wd + 2 * pd - s) // st + 1
    xp = np.zeros((n, c, h + 2 * pd, wd + 2 * pd))
    xp[:, :, pd:pd + h, pd:pd + wd] = x
    cols = np.empty((n, ho, wo, c * r * s))
    for p in range(ho):
        for q in range(wo):
            cols[:, p, q, :] = xp[:, :, p * st:p * st + r, q * st:q * st + s].reshape(n, -1)
    return (cols.reshape(-1, c * r * s) @ w.reshape(k, -1).T).reshape(n, ho, wo, k).transpose(0, 3, 1, 2)


@pytest.mark.parametrize("st,pd,r", [(1, 1, 3), (2, 1, 3), (2, 3, 7), (1, 0, 1), (2, 0, 1)])
def test_conv_matches_im2col_matmul_and_torch(st, pd, r):
    x = rng.standard_normal((2, 3, 12, 11))
    w = rng.standard_normal((4, 3, r, r))
    y = O.conv2d(x, w, (st, st), (pd, pd))
    assert np.allclose(y, _im2col_matmul(x, w, st, pd), atol=1e-12)
    t = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=st, padding=pd).numpy()
    assert y.shape == t.shape and np.allclose(y, t, atol=1e-12)
    # the one-by-one evaluator agrees with the loop nest
    pts = [(int(a), int(b), int(c), int(d)) for a, b, c, d in
           zip(rng.integers(0, 2, 9), rng.integers(0, 4, 9), rng.integers(0, y.shape[2], 9), rng.integers(0, y.shape[3], 9))]
    assert np.allclose(O.conv2d_points(x, w, pts, (st, st), (pd, pd)), [y[p] for p in pts], atol=1e-12)


def test_dwconv_and_pools_match_torch():
    x = rng.standard_normal((2, 6, 9, 10))
    w = rng.standard_normal((6, 3, 3))
    for st in (1, 2):
        t = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w[:, None]), stride=st, padding=1, groups=6)
        y = O.dwconv2d(x, w, (st, st), (1, 1))
        assert np.allclose(y, t.numpy(), atol=1e-12)
        pts = [(1, 5, 0, 0), (0, 2, y.shape[2] - 1, y.shape[3] - 1), (1, 3, 2, 1)]
        assert np.allclose(O.dwconv2d_points(x, w, pts, (st, st), (1, 1)), [y[p] for p in pts], atol=1e-12)
    mp = torch.nn.functional.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    assert np.array_equal(O.maxpool2d(x, 3, 2, 1), mp)
    assert np.allclose(O.global_avgpool(x), x.mean(axis=(2, 3)), atol=1e-14)
    # all-negative input: padding must not contribute a zero to the max
    assert np.all(O.maxpool2d(-np.ones((1, 1, 4, 4)), 3, 2, 1) == -1)


# ------------------------------------------------------------------- brute force, tiny shapes
def _brute(x, w, st, pd):
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    ho, wo = (h + 2 * pd - r) // st + 1, (wd + 2 * pd - s) // st + 1
    y = [[[[0] * wo for _ in range(ho)] for _ in range(k)] for _ in range(n)]
    for a, b, p, q, cc, rr, ss in itertools.product(range(n), range(k), range(ho), range(wo), range(c), range(r), range(s)):
        ih, iw = p * st - pd + rr, q * st - pd + ss
        if 0 <= ih < h and 0 <= iw < wd:
            y[a][b][p][q] += int(x[a, cc, ih, iw]) * int(w[b, cc, rr, ss])
    return np.array(y, dtype=np.int64).reshape(n, k, ho, wo)


@pytest.mark.parametrize("st", [1, 2])
@pytest.mark.parametrize("pd", [0, 1, 3])
def test_bruteforce_tiny_integer(st, pd):
    x = rng.integers(-128, 128, (2, 3, 5, 5)).astype(np.int8)
    w = rng.integers(-128, 128, (4, 3, 3, 3)).astype(np.int8)
    want = _brute(x, w, st, pd)
    assert np.array_equal(O.conv2d_int(x, w, (st, st), (pd, pd)), want)
    assert np.array_equal(O.conv2d(x, w, (st, st), (pd, pd)), want.astype(np.float64))


# ------------------------------------------------------------------------------ invariants
def test_int_conv_is_linear_exactly():
    x = rng.integers(-127, 128, (1, 4, 6, 6)).astype(np.int8)
    w1 = rng.integers(-60, 60, (3, 4, 3, 3)).astype(np.int8)
    w2 = rng.integers(-60, 60, (3, 4, 3, 3)).astype(np.int8)
    a = O.conv2d_int(x, (w1 + w2).astype(np.int8), (1, 1), (1, 1))
    assert np.array_equal(a, O.conv2d_int(x, w1, (1, 1), (1, 1)) + O.conv2d_int(x, w2, (1, 1), (1, 1)))


def test_translation_equivariance_interior():
    x = rng.standard_normal((1, 2, 10, 10))
    w = rng.standard_normal((2, 2, 3, 3))
    xs = np.roll(x, (1, 2), axis=(2, 3))
    y, ys = O.conv2d(x, w, (1, 1), (1, 1)), O.conv2d(xs, w, (1, 1), (1, 1))
    assert np.allclose(ys[:, :, 3:-2, 4:-2], y[:, :, 2:-3, 2:-4], atol=1e-13)


def test_elementwise_ops_and_bn_folding():
    y = rng.standard_normal((2, 3, 4, 5))
    b = rng.standard_normal(3)
    assert np.array_equal(O.bias_add(y, b), y + b[None, :, None, None])
    sc, sh = rng.standard_normal(3), rng.standard_normal(3)
    assert np.array_equal(O.scale_shift(y, sc, sh), y * sc[None, :, None, None] + sh[None, :, None, None])
    # folded (scale, shift) against the unfolded inference batch norm of a library
    g, be, mu, var = rng.standard_normal(3), rng.standard_normal(3), rng.standard_normal(3), rng.uniform(0.5, 2, 3)
    sc, sh = O.fold_bn(g, be, mu, var, 1e-5)
    t = torch.nn.functional.batch_norm(torch.from_numpy(y), torch.from_numpy(mu), torch.from_numpy(var),
                                       torch.from_numpy(g), torch.from_numpy(be), False, 0.0, 1e-5).numpy()
    assert np.allclose(O.scale_shift(y, sc, sh), t, atol=1e-12)
    r = O.relu(y)
    assert r.min() >= 0 and np.array_equal(O.relu(r), r) and np.array_equal(r, np.where(y > 0, y, 0))
    assert np.array_equal(O.add(y, 2 * y), 3 * y)


def test_fused_equals_unfused_sequence_and_order():
    x = rng.standard_normal((2, 3, 6, 6)).astype(np.float16)
    w = rng.standard_normal((4, 3, 3, 3)).astype(np.float16)
    b, sc, sh = rng.standard_normal(4), rng.standard_normal(4), rng.standard_normal(4)
    res = rng.standard_normal((2, 4, 6, 6)).astype(np.float16)
    f = O.fused_conv2d(x, w, stride=(1, 1), pad=(1, 1), bias=b, scale=sc, shift=sh, residual=res,
                       relu_flag=True, out_dtype="f64")
    c = x.astype(np.float64)
    y = torch.nn.functional.conv2d(torch.from_numpy(c), torch.from_numpy(w.astype(np.float64)), padding=1).numpy()
    y = np.maximum((y + b[None, :, None, None]) * sc[None, :, None, None] + sh[None, :, None, None] + res, 0)
    assert np.allclose(f, y, atol=1e-12)
    assert f.min() >= 0
    # order matters and is pinned: scaling before the bias would differ
    wrong = np.maximum(y * 0 + (torch.nn.functional.conv2d(torch.from_numpy(c), torch.from_numpy(w.astype(np.float64)), padding=1).numpy()
                                * sc[None, :, None, None] + b[None, :, None, None]) + sh[None, :, None, None] + res, 0)
    assert not np.allclose(f, wrong, atol=1e-6)
    # narrowing: one rounding to fp16
    f16 = O.fused_conv2d(x, w, stride=(1, 1), pad=(1, 1), bias=b, scale=sc, shift=sh, residual=res, relu_flag=True)
    assert f16.dtype == np.float16 and np.array_equal(f16, f.astype(np.float16))


def test_cast_f16_is_round_to_nearest_even():
    # 2049 lies halfway between 2048 and 2050 in fp16 -> even mantissa 2048; 2051 -> 2052
    assert O.cast_f16(np.array([2049.0, 2051.0, 1.0 + 2 ** -11, 1.0 + 3 * 2 ** -11])).tolist() == [2048.0, 2052.0, 1.0, 1.0 + 2 ** -9]
    # a double just above the tie must round up (no double rounding through fp32)
    assert float(O.cast_f16(np.array([2049.0 + 1e-9]))[0]) == 2050.0


# ----------------------------------------------------------------------- requant, exhaustive
def test_requant_exhaustive_against_rationals():
    acc = np.arange(-(1 << 12), (1 << 12) + 1, dtype=np.int64)
    for s in range(0, 17):
        q = O.rshift_round(acc, s)
        want = [int((Fraction(int(a), 1 << s) + Fraction(1, 2)).__floor__()) for a in acc]
        assert q.tolist() == want, s
        assert np.all(np.diff(q) >= 0)
        assert q[acc == 0][0] == 0
    # a wider sweep against numpy's floor on exact binary fractions
    acc = np.arange(-(1 << 17), (1 << 17) + 1, dtype=np.int64)
    for s in range(0, 17):
        want = np.floor(acc.astype(np.float64) / float(1 << s) + 0.5).astype(np.int64)
        assert np.array_equal(O.rshift_round(acc, s), want)
        assert np.array_equal(O.requant_points(acc[::97], out_rshift=s),
                              np.clip(want[::97], -127, 127).astype(np.int8))


def test_requant_ties_clip_and_relu_commute():
    for s in range(1, 20):
        for j in (-5, -2, -1, 0, 1, 4):
            acc = (2 * j + 1) * (1 << (s - 1))            # exactly j + 1/2
            assert int(O.rshift_round(np.array([acc]), s)[0]) == j + 1
        assert int(O.rshift_round(np.array([-3 * (1 << (s - 1))]), s)[0]) == -1
    acc = rng.integers(-(1 << 20), 1 << 20, 5000)
    for s in (0, 3, 9, 12):
        a = O.relu_int(O.clip_int(O.rshift_round(acc, s)))
        b = O.clip_int(O.rshift_round(O.relu_int(acc), s))
        assert np.array_equal(a, b)
        assert a.max() <= 127 and O.clip_int(O.rshift_round(acc, s)).min() >= -127
    with pytest.raises(OverflowError):
        O.cast_i8(np.array([200]))
    with pytest.raises(OverflowError):
        O.assert_fits_i32(np.array([1 << 31]))


def test_qconv_fused_equals_separate_ops_and_bigints():
    x = rng.integers(-127, 128, (2, 5, 6, 7)).astype(np.int8)
    w = rng.integers(-127, 128, (3, 5, 3, 3)).astype(np.int8)
    bias = rng.integers(-5000, 5000, 3)
    res = rng.integers(-127, 128, (2, 3, 6, 7)).astype(np.int8)
    y = O.qconv2d_requant(x, w, stride=(1, 1), pad=(1, 1), bias=bias, residual=res, residual_lshift=6,
                          out_rshift=9, relu_flag=False)
    acc = _brute(x, w, 1, 1)
    want = np.empty(acc.shape, dtype=np.int64)
    for idx in np.ndindex(acc.shape):
        t = int(acc[idx]) + int(bias[idx[1]]) + int(res[idx]) * 64
        want[idx] = max(-127, min(127, (Fraction(t, 512) + Fraction(1, 2)).__floor__()))
    assert y.dtype == np.int8 and np.array_equal(y, want)
    pts = [(1, 2, 5, 6), (0, 0, 0, 0), (1, 1, 3, 2)]
    a = O.conv2d_points(x, w, pts, (1, 1), (1, 1), integer=True)
    rp = O.requant_points(a, bias=bias, ks=[p[1] for p in pts], residual=[res[p] for p in pts],
                          residual_lshift=6, out_rshift=9)
    assert rp.tolist() == [int(y[p]) for p in pts]


def test_stack_runner_narrows_between_layers():
    from oracle.stack import run_float
    from workloads import nets, inputs
    ops = nets.basic_block(8)
    params = inputs.net_params(ops, 2, "f16")
    x = inputs.image(2, 1, 8, 6, 6, "f16")
    t = run_float(ops, params, x, "f16")
    assert t["blk.t"].dtype == np.float16 and t["blk.out"].shape == (1, 8, 6, 6)
    mid = O.fused_conv2d(x, params[0]["w"], stride=(1, 1), pad=(1, 1), scale=params[0]["scale"],
                         shift=params[0]["shift"], relu_flag=True)
    out = O.fused_conv2d(mid, params[1]["w"], stride=(1, 1), pad=(1, 1), scale=params[1]["scale"],
                         shift=params[1]["shift"], residual=x, relu_flag=True)
    assert np.array_equal(t["blk.out"], out)

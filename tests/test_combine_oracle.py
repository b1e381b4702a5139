"""Pins of the oracle's axis scale folding and parallel convolution combination (paper Section 4.4)
against what the definitions fix: the algebraic identities, hand-worked values, and the plain
operator-by-operator evaluation.  CPU only."""
import numpy as np
import pytest

import oracle as O
from oracle import combine as OC
from oracle import stack as OS
from workloads import inputs, nets


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ------------------------------------------------------------------------------ scale folding
def test_fold_handworked_values():
    w = np.arange(1, 9, dtype=np.float64).reshape(2, 2, 1, 2)       # [k][c][r][s]
    out = OC.fold_scale_axis(w, [2.0, -0.5], "out", "f32")
    assert out.dtype == np.float32
    assert out.reshape(2, 4).tolist() == [[2, 4, 6, 8], [-2.5, -3, -3.5, -4]]
    inn = OC.fold_scale_axis(w, [10.0, 0.25], "in", "f32")
    assert inn.reshape(2, 4).tolist() == [[10, 20, 0.75, 1.0], [50, 60, 1.75, 2.0]]


@pytest.mark.parametrize("stride,pad,r", [(1, 1, 3), (2, 1, 3), (1, 0, 1), (2, 3, 7), (1, 2, 5)])
def test_scale_after_conv_moves_into_the_filters(stride, pad, r):
    x, w, s = _rand(1, 2, 5, 9, 8), _rand(2, 6, 5, r, r), _rand(3, 6)
    lhs = O.conv2d(x, w, (stride, stride), (pad, pad)) * s[None, :, None, None]
    # folding without the narrowing step: the identity itself, to rounding of the fp64 sums
    rhs = O.conv2d(x, w * s[:, None, None, None], (stride, stride), (pad, pad))
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    # and through the oracle's function in fp32 filters: off by the narrowing only
    rhs32 = O.conv2d(x, OC.fold_scale_axis(w, s, "out", "f32"), (stride, stride), (pad, pad))
    np.testing.assert_allclose(lhs, rhs32, rtol=0, atol=1e-5)


@pytest.mark.parametrize("stride,pad,r", [(1, 1, 3), (2, 1, 3), (1, 2, 5)])
def test_scale_before_conv_moves_into_the_filters(stride, pad, r):
    x, w, s = _rand(4, 2, 5, 9, 8), _rand(5, 6, 5, r, r), _rand(6, 5)
    lhs = O.conv2d(x * s[None, :, None, None], w, (stride, stride), (pad, pad))     # borders included
    rhs = O.conv2d(x, OC.fold_scale_axis(w, s, "in", "f32").astype(np.float64), (stride, stride), (pad, pad))
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-5)
    # the two axes are different things: folding along the wrong one is caught
    if w.shape[0] != w.shape[1]:
        with pytest.raises(AssertionError):
            OC.fold_scale_axis(w, s, "out", "f32")


def test_fold_narrows_once_to_the_working_type():
    w = np.array([[[[1.0 + 2.0 ** -10]]]], dtype=np.float16)          # 1 + one fp16 ulp
    s = np.array([1.0 + 2.0 ** -10])
    out = OC.fold_scale_axis(w, s, "out", "f16")
    # exact product 1 + 2^-9 + 2^-20 rounds to 1 + 2^-9 in fp16
    assert out.dtype == np.float16 and float(out[0, 0, 0, 0]) == 1.0 + 2.0 ** -9


def test_folded_batch_norm_is_shift_only_and_equal():
    op = nets.conv("c", "x", "y", 16, 24, 3, 1, 1, bias=True)
    p = inputs.layer_params(op, 7, 0, "f32")
    x = inputs.activation(7, 0, (2, 16, 10, 11), "f32")
    q = OC.fold_bn_into_conv(p, "f32")
    assert set(q) == {"w", "bias"}
    want = O.fused_conv2d(x, p["w"], stride=(1, 1), pad=(1, 1), bias=p["bias"], scale=p["scale"], shift=p["shift"],
                          relu_flag=True, out_dtype="f32")
    got = O.fused_conv2d(x, q["w"], stride=(1, 1), pad=(1, 1), bias=q["bias"], relu_flag=True, out_dtype="f32")
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-5)
    # a conv without scale/shift is left as it is
    p2 = {"w": p["w"], "bias": p["bias"]}
    assert OC.fold_bn_into_conv(p2, "f32").keys() == p2.keys()


# ------------------------------------------------------------------------ parallel combination
def test_groups_of_the_inception_block_and_of_networks_without_parallel_convs():
    ops = nets.inception_block()
    assert OC.combine_groups(ops) == [[0, 1, 3]]                     # the three 1x1 convs reading x
    assert [ops[i].name for i in (0, 1, 3)] == ["b1", "b3r", "b5r"]
    # ResNet: the 3x3/s2 conv and the 1x1/s2 shortcut share an input but not a window
    assert OC.combine_groups(nets.resnet18()) == []
    assert OC.combine_groups(nets.mobilenet_v1()) == []


def test_group_rules():
    c = nets.conv
    ops = [c("a", "x", "a", 32, 8, 3, 1, 1), c("b", "x", "b", 32, 16, 3, 1, 1),
           c("c", "x", "c", 32, 16, 3, 2, 1),                        # other stride
           c("d", "x", "d", 32, 16, 3, 1, 1, relu=False),            # other tail
           c("e", "a", "e", 8, 8, 1, 1, 0), c("f", "a", "f", 8, 24, 1, 1, 0),
           c("g", "a", "g", 8, 8, 1, 1, 0, res="e"),                 # residual operand: left alone
           c("h", "x", "h", 32, 40, 3, 1, 1)]
    assert OC.combine_groups(ops) == [[0, 1, 7], [4, 5]]


@pytest.mark.parametrize("seed", range(4))
def test_combined_conv_equals_its_members_exactly(seed):
    rng = np.random.default_rng(40 + seed)
    cin, r = int(rng.integers(3, 9)), int(rng.choice([1, 3]))
    ks = [int(k) for k in rng.integers(1, 7, size=int(rng.integers(2, 5)))]
    x = rng.standard_normal((2, cin, 7, 6)).astype(np.float16)
    members = []
    for j, k in enumerate(ks):
        op = nets.conv(f"m{j}", "x", f"m{j}", cin, k, r, 1, r // 2, bias=bool(seed & 1))
        members.append(inputs.layer_params(op, 8, 10 * seed + j, "f16"))
    outs = OC.combined_conv2d(x, members, stride=(1, 1), pad=(r // 2, r // 2), relu_flag=True)
    assert [o.shape[1] for o in outs] == ks
    for m, got in zip(members, outs):
        want = O.fused_conv2d(x, m["w"], stride=(1, 1), pad=(r // 2, r // 2), bias=m.get("bias"), scale=m["scale"],
                              shift=m["shift"], relu_flag=True, out_dtype="f16")
        assert np.array_equal(got, want)                              # output channels do not interact


def test_concat_in_the_network_oracle():
    ops = nets.inception_block((8, 4, 4, 6, 2, 3, 5))
    params = inputs.net_params(ops, 9, "f16")
    x = inputs.activation(9, 0, (1, 8, 6, 6), "f16")
    t = OS.run_float(ops, params, x)
    assert t["cat"].shape == (1, 4 + 6 + 3 + 5, 6, 6)
    assert np.array_equal(t["cat"][:, :4], t["b1.out"]) and np.array_equal(t["cat"][:, 4:10], t["b3.out"])
    assert np.array_equal(t["cat"][:, 10:13], t["b5.out"]) and np.array_equal(t["cat"][:, 13:], t["bp.out"])
    # the pool branch really is a 3x3 / stride 1 max over the input
    assert float(t["pool.out"][0, 0, 0, 0]) == float(x[0, 0, :2, :2].max())
    assert nets.trace_shapes(ops, 6, 6, 8)["cat"] == (18, 6, 6)


# ------------------------------------------------------- members with different windows (1x1 inside r x r)
@pytest.mark.parametrize("r,stride,hw", [(3, 2, (8, 8)), (3, 2, (9, 7)), (3, 1, (5, 6)), (5, 2, (11, 8)), (7, 3, (13, 9))])
def test_a_1x1_conv_is_the_centre_tap_of_a_padded_odd_window(r, stride, hw):
    """The identity the merged launch rests on, in fp64, exact: same output shape and same values."""
    rng = np.random.default_rng(50 + r + stride)
    x = rng.standard_normal((2, 5) + hw)
    w = rng.standard_normal((4, 5, 1, 1))
    a = O.conv2d(x, w, (stride, stride), (0, 0))
    b = O.conv2d(x, OC.embed_centre(w, r), (stride, stride), (r // 2, r // 2))
    assert a.shape == b.shape and np.array_equal(a, b)
    # an off-centre embedding is a different function: the pin fails for it
    bad = np.zeros((4, 5, r, r))
    bad[:, :, 0, 0] = w[:, :, 0, 0]
    assert not np.array_equal(a, O.conv2d(x, bad, (stride, stride), (r // 2, r // 2)))


def test_groups_with_windows_on_resnet_and_rules():
    ops = nets.resnet18()
    names = [[ops[i].name for i in g] for g in OC.combine_groups(ops, windows=True)]
    assert names == [["l2.b0.conv1", "l2.b0.down"], ["l3.b0.conv1", "l3.b0.down"], ["l4.b0.conv1", "l4.b0.down"]]
    assert OC.combine_groups(nets.inception_block(), windows=True) == OC.combine_groups(nets.inception_block())
    assert OC.combine_groups(nets.mobilenet_v1(), windows=True) == []
    c = nets.conv
    ops = [c("a", "x", "a", 32, 8, 1, 2, 0, relu=False), c("b", "x", "b", 32, 16, 3, 2, 1),     # 1x1 + 3x3, stride 2
           c("c", "x", "c", 32, 16, 3, 1, 1),                                                    # other stride
           c("d", "x", "d", 32, 16, 5, 2, 2), c("e", "x", "e", 32, 16, 3, 2, 0),                 # wider window; not centred
           c("f", "x", "f", 32, 16, 3, 2, 1, relu=False)]
    # widest window (5x5, d) takes the 1x1 (a); the two 3x3/s2/p1 differ in relu and stay apart; e is not centred
    assert OC.combine_groups(ops, windows=True) == [[3, 0]]


def test_windowed_group_equals_its_members_exactly():
    ops = [nets.conv("t", "x", "t", 6, 5, 3, 2, 1), nets.conv("d", "x", "d", 6, 7, 1, 2, 0, relu=False)]
    members = [inputs.layer_params(op, 9, j, "f16") for j, op in enumerate(ops)]
    x = np.random.default_rng(60).standard_normal((2, 6, 9, 8)).astype(np.float16)
    outs = OC.combined_conv2d_windows(x, ops, members)
    for op, m, got in zip(ops, members, outs):
        want = O.fused_conv2d(x, m["w"], stride=(2, 2), pad=(op.pad, op.pad), scale=m["scale"], shift=m["shift"],
                              relu_flag=op.relu, out_dtype="f16")
        assert got.shape == want.shape and np.array_equal(got, want), op.name
    assert outs[1].min() < 0 <= outs[0].min()

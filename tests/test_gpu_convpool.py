"""GPU parity of the convolution that carries its 3x3 / stride 2 / pad 1 max pool in the same
launch (operator fusion, paper Section 4.1, taken one window operator further): against the
oracle's conv followed by its max pool, and bit for bit against the library's own two calls."""
import numpy as np
import pytest
import torch

import oracle as O
from workloads import inputs, nets

pytestmark = pytest.mark.gpu
TOL_F16 = 1e-2


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


def _oracle_f16(x, p, stride, pad, relu):
    y = O.fused_conv2d(x, p["w"], stride=(stride, stride), pad=(pad, pad), bias=p.get("bias"),
                       scale=p.get("scale"), shift=p.get("shift"), relu_flag=relu, out_dtype="f16")
    return O.maxpool2d(y, 3, 2, 1).astype(np.float16)


# (n, c, h, w, k, r, stride, pad, bias, bn, relu): conv outputs of 14a x 16b, several blocks per
# image in both directions, a ragged last channel tile, the first-layer geometry in both layouts
F16_CASES = [
    (2, 32, 28, 32, 64, 3, 1, 1, False, True, True),
    (1, 64, 14, 16, 72, 3, 1, 1, True, True, True),      # one block per image, 64 + 8 channels
    (3, 32, 28, 48, 136, 1, 1, 0, True, False, False),   # pointwise, no relu: negative maxima
    (2, 3, 56, 64, 64, 7, 2, 3, False, True, True),      # first layer
    (1, 32, 56, 32, 64, 3, 2, 1, False, True, True),     # strided conv: 28 x 16
]


@pytest.mark.parametrize("case", F16_CASES)
def test_fp16_conv_maxpool_one_launch(G, case):
    n, c, h, w, k, r, st, pd, bias, bn, relu = case
    op = nets.conv("c", "x", "y", c, k, r, st, pd, bias=bias, bn=bn, relu=relu)
    p = inputs.layer_params(op, 31, k + r, "f16")
    x = inputs.activation(31, c + h, (n, c, h, w), "f16")
    want = _oracle_f16(x, p, st, pd, relu)
    for nhwc4 in ((True,) if c <= 4 else (False,)):   # few-channel inputs come pre-padded
        got = G.run_conv_pool_f16(x, p["w"], st, pd, bias=p.get("bias"), scale=p.get("scale"), shift=p.get("shift"),
                                  relu=relu, nhwc4=nhwc4)
        assert got.shape == want.shape and got.dtype == np.float16
        assert not np.isnan(got).any()
        assert O.max_rel_err(got, want) <= TOL_F16, nhwc4
        two = G.run_conv_pool_f16(x, p["w"], st, pd, bias=p.get("bias"), scale=p.get("scale"), shift=p.get("shift"),
                                  relu=relu, nhwc4=nhwc4, fused=False)
        # same rounding of every conv output: the comparison commutes with nothing else
        assert int((got.view(np.uint16) != two.view(np.uint16)).sum()) == 0, nhwc4


I8_CASES = [
    (2, 64, 28, 32, 64, 3, 1, 1, True, True),
    (1, 64, 14, 16, 72, 3, 1, 1, False, False),   # no relu: negative maxima, the -127 clip
    (2, 3, 56, 64, 64, 7, 2, 3, True, True),      # first layer
    (1, 128, 28, 16, 200, 1, 1, 0, True, True),
]


@pytest.mark.parametrize("case", I8_CASES)
def test_int8_conv_maxpool_one_launch_bit_exact(G, case):
    n, c, h, w, k, r, st, pd, bias, relu = case
    op = nets.conv("c", "x", "y", c, k, r, st, pd, bn=False, relu=relu)
    p = inputs.layer_params(op, 32, k + r, "i8")
    x = inputs.activation(32, c + h, (n, c, h, w), "i8")
    b = inputs.rng_for(32, 77).integers(-2000, 2000, size=k).astype(np.int32) if bias else None
    rs = inputs.default_out_rshift(c * r * r)
    y = O.qconv2d_requant(x, p["w"], stride=(st, st), pad=(pd, pd), bias=b, out_rshift=rs, relu_flag=relu)
    want = O.maxpool2d(y, 3, 2, 1).astype(np.int8)
    for nhwc4 in ((True,) if c <= 4 else (False,)):   # few-channel inputs come pre-padded
        got = G.run_qconv_pool(x, p["w"], st, pd, bias=b, rshift=rs, relu=relu, nhwc4=nhwc4)
        assert got.shape == want.shape and int((got != want).sum()) == 0, nhwc4
    if not relu:
        assert (want < 0).any()


def test_pooled_border_takes_only_inside_values(G):
    """All conv outputs negative (no relu): a pad position counted as 0 would win every border window."""
    n, c, h, w, k = 1, 32, 14, 16, 64
    x = np.abs(inputs.activation(33, 1, (n, c, h, w), "f16"))
    wt = -np.abs(inputs.activation(33, 2, (k, c, 3, 3), "f16")) * np.float16(0.05)
    y = O.fused_conv2d(x, wt, stride=(1, 1), pad=(1, 1), out_dtype="f16")
    assert (y < 0).all()
    want = O.maxpool2d(y, 3, 2, 1).astype(np.float16)
    got = G.run_conv_pool_f16(x, wt, 1, 1)
    assert (got < 0).all() and O.max_rel_err(got, want) <= TOL_F16


def test_first_layer_at_full_size_equals_the_two_calls(G):
    """ResNet's first layer at batch 32, the launch the benchmark times: every pooled output equals
    conv-then-pool of the separate kernels (themselves held to the oracle on sampled outputs),
    and sampled pooled outputs equal the oracle's windows computed one by one."""
    n, c, h, w, k = 32, 3, 224, 224, 64
    op = nets.conv("c", "x", "y", c, k, 7, 2, 3, bn=True, relu=True)
    p = inputs.layer_params(op, 34, 0, "f16")
    x = inputs.image(34, n, c, h, w, "f16")
    got = G.run_conv_pool_f16(x, p["w"], 2, 3, scale=p["scale"], shift=p["shift"], relu=True)
    two = G.run_conv_pool_f16(x, p["w"], 2, 3, scale=p["scale"], shift=p["shift"], relu=True, fused=False)
    assert got.shape == (n, k, 56, 56) and int((got.view(np.uint16) != two.view(np.uint16)).sum()) == 0
    g = np.random.default_rng(5)
    for _ in range(24):
        i, oy, ox = int(g.integers(n)), int(g.integers(56)), int(g.integers(56))
        if _ < 8:   # the image corners and edges
            oy, ox = (0, 55)[_ & 1], (0, 55, int(g.integers(56)), 0)[_ >> 1]
        # the conv outputs under this pooled pixel: rows 2oy-1..2oy+1 -> input rows 4oy-5 .. 4oy+7
        r0, r1 = max(2 * oy - 1, 0), min(2 * oy + 1, 111)
        c0, c1 = max(2 * ox - 1, 0), min(2 * ox + 1, 111)
        # cut the padded input patch that produces conv rows r0..r1, columns c0..c1
        ph0, pw0 = 2 * r0 - 3, 2 * c0 - 3
        hh, ww = 2 * (r1 - r0) + 7, 2 * (c1 - c0) + 7
        xi = np.zeros((1, c, hh, ww), np.float16)
        for dy in range(hh):
            for dx in range(ww):
                yy, xx = ph0 + dy, pw0 + dx
                if 0 <= yy < h and 0 <= xx < w:
                    xi[0, :, dy, dx] = x[i, :, yy, xx]
        yc = O.fused_conv2d(xi, p["w"], stride=(2, 2), pad=(0, 0), scale=p["scale"], shift=p["shift"],
                            relu_flag=True, out_dtype="f16")
        want = yc.reshape(k, -1).max(axis=1).astype(np.float16)
        assert O.max_rel_err(got[i, :, oy, ox], want) <= TOL_F16, (i, oy, ox)


@pytest.mark.parametrize("fold_scale", [False, True])
def test_network_driver_takes_the_pooled_launch(G, fold_scale):
    """The first four functions of ResNet-18 (conv, max pool, one residual block) through the network
    driver, the pool inside the conv's launch and as its own: same bits both ways, and the oracle's
    values (on parameters folded by the oracle where the driver folds the scale into the filters)."""
    from oracle import combine as OC
    from oracle.stack import run_float
    from paper_1904_08368_amd.stack import FusedNet
    ops = nets.resnet18()[:4]
    params = inputs.net_params(ops, 3, "f16")
    x = inputs.image(35, 2, 3, 224, 224, "f16")
    ref = run_float(ops, [OC.fold_bn_into_conv(p, "f16") if (fold_scale and p) else p for p in params], x, "f16")
    outs = {}
    for pooled in (True, False):
        net = FusedNet(ops, params, 2, 224, 224, "f16", fold_scale=fold_scale, fuse_pool=pooled)
        assert ("conv1+maxpool" in net.call_names) == pooled and len(net.calls) == (4 if pooled else 5)
        net.load_input(x)
        net.run()
        torch.cuda.synchronize()
        outs[pooled] = {name: net.tensor(name) for name in (ops[1].dst, ops[-1].dst)}
        with pytest.raises(KeyError):
            net.tensor("c1") if pooled else net.tensor("no such tensor")
    for name in outs[True]:
        assert int((outs[True][name].view(np.uint16) != outs[False][name].view(np.uint16)).sum()) == 0, name
    assert O.max_rel_err(outs[True][ops[1].dst], ref[ops[1].dst]) <= TOL_F16
    assert O.max_rel_err(outs[True][ops[-1].dst], ref[ops[-1].dst]) <= 2e-2   # three layers deep: the chain tolerance of the network tests

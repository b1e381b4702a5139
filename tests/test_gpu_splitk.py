"""GPU parity of the reduction split over workgroups (the workspace path of the conv entry points):
against the oracle at forced split counts, against the unsplit kernel (int8 bit for bit), reuse of
one workspace across calls without clearing, and the library's own choice on the deep layers at
batch 1."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import quant as OQ
from workloads import inputs

pytestmark = pytest.mark.gpu
TOL_F16 = 1e-2


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


def _case(seed, n, c, h, w, k, r, mode):
    rng = np.random.default_rng(700 + seed)
    if mode == "f16":
        x = rng.standard_normal((n, c, h, w)).astype(np.float16)
        wt = (rng.standard_normal((k, c, r, r)) * np.sqrt(2.0 / (c * r * r))).astype(np.float16)
        res = rng.standard_normal((n, k, h, w)).astype(np.float16)
        sc = (1 + 0.1 * rng.standard_normal(k)).astype(np.float32)
        sf = (0.1 * rng.standard_normal(k)).astype(np.float32)
        return x, wt, res, sc, sf
    x = rng.integers(-127, 128, (n, c, h, w)).astype(np.int8)
    wt = rng.integers(-127, 128, (k, c, r, r)).astype(np.int8)
    res = rng.integers(-127, 128, (n, k, h, w)).astype(np.int8)
    bias = rng.integers(-5000, 5000, k).astype(np.int32)
    return x, wt, res, bias, None


@pytest.mark.parametrize("split", [2, 3, 9, 64])
@pytest.mark.parametrize("tile", [-1, 5, 10, 15, 9, 12])
def test_fp16_split_matches_oracle(G, split, tile):
    """128 -> 72 channels (a ragged channel tile), 3 images of 7x5 (a ragged pixel tile), residual and relu."""
    x, wt, res, sc, sf = _case(0, 3, 128, 7, 5, 72, 3, "f16")
    want = O.fused_conv2d(x, wt, stride=(1, 1), pad=(1, 1), scale=sc, shift=sf, residual=res, relu_flag=True,
                          out_dtype="f16")
    got = G.run_conv_f16(x, wt, 1, 1, scale=sc, shift=sf, residual=res, relu=True, tile=tile, split=split)
    assert O.max_rel_err(got, want) <= TOL_F16
    plain = G.run_conv_f16(x, wt, 1, 1, scale=sc, shift=sf, residual=res, relu=True, tile=tile)
    assert O.max_rel_err(got, plain) <= 2e-3           # same products, fp32 sums grouped differently


@pytest.mark.parametrize("split", [2, 5, 64])
@pytest.mark.parametrize("tile", [-1, 5, 10, 15])
def test_int8_split_is_bit_exact(G, split, tile):
    x, wt, res, bias, _ = _case(1, 2, 256, 6, 7, 80, 3, "i8")
    want = O.qconv2d_requant(x, wt, stride=(1, 1), pad=(1, 1), bias=bias, residual=res, residual_lshift=9,
                             out_rshift=13, relu_flag=False)
    got = G.run_qconv(x, wt, 1, 1, bias=bias, residual=res, lshift=9, rshift=13, tile=tile, split=split)
    assert np.array_equal(got, want)


def test_int8_split_with_stochastic_rounding(G):
    from paper_1904_08368_amd import binding as B
    x, wt, _, _, _ = _case(2, 1, 128, 7, 7, 64, 3, "i8")
    want = OQ.qconv2d_requant_mode(x, wt, stride=(1, 1), pad=(1, 1), out_rshift=14, mode=OQ.STOCHASTIC, seed=77)
    got = G.run_qconv(x, wt, 1, 1, rshift=14, split=4, round_mode=B.ROUND_STOCHASTIC, seed=77)
    assert np.array_equal(got, want)


def test_strided_and_pointwise_layers_split(G):
    x, wt, _, sc, sf = _case(3, 2, 256, 14, 14, 96, 3, "f16")
    want = O.fused_conv2d(x, wt, stride=(2, 2), pad=(1, 1), scale=sc, shift=sf, relu_flag=True, out_dtype="f16")
    assert O.max_rel_err(G.run_conv_f16(x, wt, 2, 1, scale=sc, shift=sf, relu=True, split=6), want) <= TOL_F16
    x, wt, _, sc, sf = _case(4, 1, 1024, 7, 7, 128, 1, "f16")
    want = O.fused_conv2d(x, wt, stride=(1, 1), pad=(0, 0), scale=sc, shift=sf, relu_flag=False, out_dtype="f16")
    assert O.max_rel_err(G.run_conv_f16(x, wt, 1, 0, scale=sc, shift=sf, split=8), want) <= TOL_F16


def test_workspace_is_reusable_without_clearing(G):
    """Three calls in a row on one buffer that is zeroed once: a split layer, a smaller one, the first
    again.  The arrival counts must be back at zero after every call."""
    state = {}
    big = _case(5, 2, 256, 7, 7, 128, 3, "f16")
    small = _case(6, 1, 128, 5, 5, 64, 3, "f16")
    for x, wt, res, sc, sf in (big, small, big):
        want = O.fused_conv2d(x, wt, stride=(1, 1), pad=(1, 1), scale=sc, shift=sf, relu_flag=True, out_dtype="f16")
        got = G.run_conv_f16(x, wt, 1, 1, scale=sc, shift=sf, relu=True, split=4, ws_state=state)
        assert O.max_rel_err(got, want) <= TOL_F16
        assert int(state["ws"][:256].to(torch.int32).abs().sum()) == 0


def test_library_splits_the_deep_layers_at_batch_1_only(G):
    from paper_1904_08368_amd import binding as B
    d = lambda n, c, hw, k: B.conv_desc(n, c, hw, hw, k, 3, 3, 1, 1, B.RELAY_F16, B.RELAY_NHWC, B.RELU)
    assert B.relay_workspace_bytes(d(1, 512, 7, 512)) > 0
    assert B.relay_workspace_bytes(d(1, 256, 14, 256)) == 0      # 18 chunks: measured faster unsplit
    assert B.relay_workspace_bytes(d(32, 64, 56, 64)) == 0
    assert B.relay_workspace_bytes(d(32, 128, 28, 128)) == 0
    # the layer the library splits by itself: parity at its real shape (sampled: the oracle's full conv
    # of this layer takes seconds, which is fine once)
    x, wt, _, sc, sf = _case(7, 1, 512, 7, 7, 512, 3, "f16")
    want = O.fused_conv2d(x, wt, stride=(1, 1), pad=(1, 1), scale=sc, shift=sf, relu_flag=True, out_dtype="f16")
    got = G.run_conv_f16(x, wt, 1, 1, scale=sc, shift=sf, relu=True, split=0)
    assert O.max_rel_err(got, want) <= TOL_F16


def test_resnet18_batch1_with_split_layers_matches_the_oracle(G):
    """Batch 1 is where the network driver hands workspaces to the deep layers: the chain against the
    oracle, eager and replayed from a HIP graph three times (the counters must come back to zero
    every time), fp16 and int8."""
    from oracle.stack import run_float, run_quantized
    from paper_1904_08368_amd.stack import FusedNet
    from workloads import nets
    ops = nets.resnet18()
    params = inputs.net_params(ops, 3, "f16")
    x = inputs.image(3, 1, 3, 224, 224, "f16")
    ref = run_float(ops, params, x, "f16")
    net = FusedNet(ops, params, 1, 224, 224, "f16")
    assert sum(1 for _, args in net.calls if len(args) == 9 and args[-1] is not None) >= 3     # layers given a workspace
    net.load_input(x)
    net.run()
    torch.cuda.synchronize()
    logits = net.tensor("logits").reshape(1, 1000)
    assert O.max_rel_err(logits, ref["logits"]) <= 2e-2
    assert O.max_rel_err(net.tensor("l4.b1.out"), ref["l4.b1.out"]) <= 2e-2
    net.capture()
    for _ in range(3):
        net.bufs["logits"].zero_()
        net.replay()
        torch.cuda.synchronize()
        assert np.array_equal(net.tensor("logits").reshape(1, 1000), logits)
    qops = nets.resnet18(with_dense=False)
    qp = inputs.net_params(qops, 4, "i8")
    sh = inputs.chain_shifts(qops)
    xq = inputs.image(4, 1, 3, 224, 224, "i8")
    qnet = FusedNet(qops, qp, 1, 224, 224, "i8", shifts=sh)
    qnet.load_input(xq)
    qnet.run()
    torch.cuda.synchronize()
    refq = run_quantized(qops, qp, sh, xq)
    assert np.array_equal(qnet.tensor(qops[-1].dst), refq[qops[-1].dst])

"""GPU parity of the quantization variants (paper Section 4.2): rounding strategies of the fused
requantization and the Q / simQ operators, bit for bit against the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import quant as OQ

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    from paper_1904_08368_amd import binding as B
    B.lib()
    assert torch.cuda.is_available()
    from tests import gpu_util
    return gpu_util


def _qconv_mode(G, x, w, stride, pad, *, bias=None, residual=None, lshift=0, rshift=0, relu=False, mode=0, seed=0):
    from paper_1904_08368_amd import binding as B
    n, c, h, ww = x.shape
    k, _, r, s = w.shape
    flags = B.flags_of(bias, None, residual, relu)
    d, xd = G._input(x, k, r, s, stride, pad, B.RELAY_I8, 16, flags, False)
    ho, wo = B.relay_conv2d_out_shape(d)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=G.DEV)
    B.relay_prepack_conv2d_weights(d, G.up(w), c, wp)
    y = torch.full((n, ho, wo, k), -128, dtype=torch.int8, device=G.DEV)
    res = G.to_nhwc(residual, k, B.RELAY_I8) if residual is not None else None
    B.relay_qconv2d_requant_rounding(d, xd, wp, G.up(bias) if bias is not None else None, res, lshift, rshift, mode, seed, y)
    torch.cuda.synchronize()
    return G.from_nhwc(y, k)


@pytest.mark.parametrize("mode", [OQ.NEAREST, OQ.FLOOR, OQ.CEIL, OQ.STOCHASTIC])
@pytest.mark.parametrize("shape", [(2, 64, 13, 17, 192), (1, 48, 9, 11, 37), (2, 128, 7, 7, 64)])
def test_qconv_rounding_modes_bit_exact(G, mode, shape):
    n, c, h, w, k = shape
    rng = np.random.default_rng(700 + c + mode)
    x = rng.integers(-127, 128, (n, c, h, w)).astype(np.int8)
    wt = rng.integers(-127, 128, (k, c, 3, 3)).astype(np.int8)
    res = rng.integers(-127, 128, (n, k, h, w)).astype(np.int8)
    b = rng.integers(-5000, 5000, k).astype(np.int32)
    for seed, s in ((0x1234_5678_9ABC_DEF0, 13), (7, 1), (99, 0)):
        ref = OQ.qconv2d_requant_mode(x, wt, stride=(1, 1), pad=(1, 1), bias=b, residual=res, residual_lshift=s,
                                      out_rshift=s, relu_flag=False, mode=mode, seed=seed)
        got = _qconv_mode(G, x, wt, 1, 1, bias=b, residual=res, lshift=s, rshift=s, mode=mode, seed=seed)
        assert np.array_equal(got, ref), (mode, s)
    # nearest through the new entry point is the old entry point
    if mode == OQ.NEAREST:
        assert np.array_equal(_qconv_mode(G, x, wt, 1, 1, rshift=12, relu=True), G.run_qconv(x, wt, 1, 1, rshift=12, relu=True))


@pytest.mark.parametrize("mode", [OQ.NEAREST, OQ.FLOOR, OQ.CEIL, OQ.STOCHASTIC])
def test_qconv_rounding_exact_for_shifts_up_to_31_and_sums_near_the_int32_limits(G, mode):
    """Biases push the sums to +-(2^30 .. 2^31): adding the rounding addend in 32 bits would wrap
    there (ceiling at s = 31 of acc = 1 would give -1); the library must still equal the oracle,
    whose arithmetic is 64-bit."""
    rng = np.random.default_rng(760 + mode)
    x = rng.integers(-127, 128, (1, 64, 9, 10)).astype(np.int8)
    wt = rng.integers(-127, 128, (72, 64, 3, 3)).astype(np.int8)
    top = (1 << 31) - 1 - 9 * 64 * 127 * 127                   # leaves room for the largest possible conv sum
    b = rng.integers(-top, top, 72).astype(np.int32)
    b[:8] = [top, -top, (1 << 30), -(1 << 30), 0, 1, -1, top - 1]
    for s in (31, 30, 24):
        for bias in (b, None):
            ref = OQ.qconv2d_requant_mode(x, wt, stride=(1, 1), pad=(1, 1), bias=bias, out_rshift=s, mode=mode, seed=11)
            for tile in (-1, 100):                               # the implicit-GEMM kernel and the halo kernel
                from paper_1904_08368_amd import binding as B
                B.relay_set_conv_tile(tile)
                try:
                    got = _qconv_mode(G, x, wt, 1, 1, bias=bias, rshift=s, mode=mode, seed=11)
                finally:
                    B.relay_set_conv_tile(-1)
                assert np.array_equal(got, ref), (mode, s, bias is None, tile)
    # the zero-weight layer: acc = bias exactly, every code decided by the rounding rule alone
    z = np.zeros_like(wt)
    small = np.array([1, -1, 0, 2, -2, (1 << 30) + 1, -(1 << 30) - 1, (1 << 31) - 1] * 9, dtype=np.int32)
    ref = OQ.qconv2d_requant_mode(x, z, stride=(1, 1), pad=(1, 1), bias=small, out_rshift=31, mode=mode, seed=11)
    got = _qconv_mode(G, x, z, 1, 1, bias=small, rshift=31, mode=mode, seed=11)
    assert np.array_equal(got, ref)
    if mode == OQ.CEIL:
        assert got[0, 0, 0, 0] == 1 and got[0, 1, 0, 0] == 0 and got[0, 5, 0, 0] == 1


def test_qconv_stochastic_depends_on_seed_and_position_only(G):
    """The same layer with a different tile shape, and as two half-batches, draws the same words."""
    from paper_1904_08368_amd import binding as B
    rng = np.random.default_rng(720)
    x = rng.integers(-127, 128, (2, 64, 12, 12)).astype(np.int8)
    wt = rng.integers(-127, 128, (64, 64, 3, 3)).astype(np.int8)
    ref = OQ.qconv2d_requant_mode(x, wt, stride=(1, 1), pad=(1, 1), out_rshift=14, mode=OQ.STOCHASTIC, seed=5)
    for tile in (4, 5, 0):
        B.relay_set_conv_tile(tile)
        try:
            got = _qconv_mode(G, x, wt, 1, 1, rshift=14, mode=OQ.STOCHASTIC, seed=5)
        finally:
            B.relay_set_conv_tile(-1)
        assert np.array_equal(got, ref), tile
    assert not np.array_equal(_qconv_mode(G, x, wt, 1, 1, rshift=14, mode=OQ.STOCHASTIC, seed=6), ref)


@pytest.mark.parametrize("mode", [OQ.NEAREST, OQ.FLOOR, OQ.CEIL, OQ.STOCHASTIC])
@pytest.mark.parametrize("src", ["f32", "f16"])
def test_quantize_and_sim_quantize_bit_exact(G, mode, src):
    from paper_1904_08368_amd import binding as B
    rng = np.random.default_rng(740 + mode)
    n = 2048 * 3 + 5                                     # whole blocks and a ragged tail
    x = (rng.standard_normal(n) * 3).astype(np.float32)
    x[:8] = [0.0, -0.0, 2.5 / 64, -2.5 / 64, 1e9, -1e9, 0.5 / 64, -0.5 / 64]   # ties and far out of range
    if src == "f16":
        x[4:6] = [60000, -60000]
        x = x.astype(np.float16)
    xd = G.up(x)
    for rho, beta, sigma in ((2.0, 8, 1), (6.5, 8, 1), (0.75, 4, 1), (16.0, 8, 0), (3.0, 5, 0)):   # sigma 0: unsigned codes
        y = torch.full((n,), -128, dtype=torch.int8, device=G.DEV)
        B.relay_quantize(n, B.RELAY_F16 if src == "f16" else B.RELAY_F32, xd, rho, beta, sigma, mode, 42, y)
        torch.cuda.synchronize()
        ref = OQ.Q(x, rho, beta, sigma, mode, 42)
        assert ref.dtype == (np.uint8 if sigma == 0 else np.int8)
        assert np.array_equal(y.cpu().numpy().view(np.uint8), ref.view(np.uint8)), (rho, beta)   # the same bytes
        if src == "f32":
            ys = torch.full((n,), float("nan"), dtype=torch.float32, device=G.DEV)
            B.relay_sim_quantize(n, xd, rho, beta, sigma, mode, 42, ys)
            torch.cuda.synchronize()
            refs = OQ.simQ(x, beta, sigma, rho, mode, 42)
            assert np.array_equal(ys.cpu().numpy().view(np.uint32), refs.view(np.uint32)), (rho, beta)


def test_quantized_input_feeds_the_int8_stack(G):
    """Q as the first operator of a realized network: fp16 image -> int8 codes -> int8 conv, the
    whole chain bit-exact against the oracle chain."""
    from paper_1904_08368_amd import binding as B
    rng = np.random.default_rng(760)
    img = (rng.standard_normal((2, 16, 10, 10))).astype(np.float16)
    wt = rng.integers(-127, 128, (32, 16, 3, 3)).astype(np.int8)
    codes_ref = OQ.Q(img, 4.0, 8, 1)
    ref = O.qconv2d_requant(codes_ref, wt, stride=(1, 1), pad=(1, 1), out_rshift=9, relu_flag=True)
    xq = torch.empty(img.size, dtype=torch.int8, device=G.DEV)
    B.relay_quantize(img.size, B.RELAY_F16, G.up(img), 4.0, 8, 1, B.ROUND_NEAREST, 0, xq)
    torch.cuda.synchronize()
    codes = xq.cpu().numpy().reshape(img.shape)
    assert np.array_equal(codes, codes_ref)
    assert np.array_equal(G.run_qconv(codes, wt, 1, 1, rshift=9, relu=True), ref)


def test_calibrate_realize_flow_on_resnet18(G):
    """fp16 ResNet-18 conv stack -> calibrated power-of-two ranges -> scale folded into the filters ->
    realized int8 network: ranges, filters, biases and shifts equal the oracle's; the realized network
    runs bit-exactly; its dequantized output follows the float network."""
    from oracle import realize as R
    from oracle.stack import run_float, run_quantized
    from paper_1904_08368_amd import quantize as PQ
    from paper_1904_08368_amd.stack import FusedNet
    from workloads import inputs, nets
    ops = nets.resnet18(with_dense=False)
    params = inputs.net_params(ops, 3, "f16")
    x = inputs.image(3, 2, 3, 224, 224, "f16")
    t = run_float(ops, params, x, "f16")
    rho_ref = R.calibrate(ops, t)
    rho = PQ.calibrate(ops, params, x)
    # the two float runs differ in the last bits: a maximum sitting on a power of two could flip a range
    assert sum(1 for k in rho_ref if rho[k] != rho_ref[k]) == 0, {k: (rho[k], rho_ref[k]) for k in rho if rho[k] != rho_ref[k]}
    qp_ref, sh_ref = R.realize(ops, params, rho_ref)
    qp, sh = PQ.realize(ops, params, rho)
    assert sh == sh_ref
    for a, b, op in zip(qp, qp_ref, ops):
        assert a.keys() == b.keys(), op.name
        for k in a:
            assert np.array_equal(a[k], b[k]), (op.name, k)
    xq = PQ.quantize_input(x, rho["x"])
    assert np.array_equal(xq, OQ.Q(x, rho_ref["x"], 8, 1))
    ref_q = run_quantized(ops, qp_ref, sh_ref, xq)
    net = FusedNet(ops, qp, 2, 224, 224, "i8", shifts=sh)
    net.load_input(xq)
    net.run()
    torch.cuda.synchronize()
    for op in ops:
        if op.dst in net.bufs:      # (a conv that runs with its max pool leaves no tensor of its own)
            assert np.array_equal(net.tensor(op.dst), ref_q[op.dst]), op.name
    last = ops[-1].dst
    ref = t[last].astype(np.float64)
    deq = R.dequantize(net.tensor(last), rho[last])
    sqnr = 10 * np.log10((ref ** 2).sum() / ((deq - ref) ** 2).sum())
    assert sqnr > 20, sqnr


def test_realize_conv_and_range_entry_points_against_the_oracle(G):
    """relay_realize_conv (device kernels) against oracle.realize (numpy): filters with the scale
    folded in, the bias with a conv bias in front of the scale, both shifts, the filter range, and
    the status bits; relay_calibrate_pow2_range against the oracle's rule, edge values included."""
    from oracle import realize as R
    from paper_1904_08368_amd import binding as B
    rng = np.random.default_rng(780)

    class Op:
        kind, name, src, dst, res = "conv", "c", "x", "y", "r"
    for k, c, r, with_bias, with_bn in ((24, 16, 3, True, True), (7, 5, 1, False, True), (9, 3, 7, True, False), (4, 8, 3, False, False)):
        w = (rng.standard_normal((k, c, r, r)) * 0.3).astype(np.float32)
        p = {"w": w}
        if with_bias:
            p["bias"] = rng.standard_normal(k).astype(np.float32)
        if with_bn:
            p["scale"] = (1 + 0.3 * rng.standard_normal(k)).astype(np.float32)
            p["shift"] = rng.standard_normal(k).astype(np.float32)
        rho = {"x": 4.0, "y": 16.0, "r": 8.0}
        qp_ref, sh_ref = R.realize([Op], [p], rho)
        wq = torch.full(w.shape, -128, dtype=torch.int8, device=G.DEV)
        bq = torch.full((k,), 12345, dtype=torch.int32, device=G.DEV) if (with_bias or with_bn) else None
        out = torch.zeros(4, dtype=torch.int32, device=G.DEV)
        ws = torch.empty(w.size * 4 + 16, dtype=torch.uint8, device=G.DEV)
        B.relay_realize_conv(k, c * r * r, G.up(w), G.up(p.get("bias")), G.up(p.get("scale")), G.up(p.get("shift")),
                             rho["x"], rho["y"], rho["r"], wq, bq, out, ws)
        torch.cuda.synchronize()
        rho_w_bits, s, l, status = out.cpu().tolist()
        rho_w = float(np.array([rho_w_bits], dtype=np.int32).view(np.float32)[0])
        wf = R.fold_scale(w, p.get("scale")).astype(np.float32)
        assert rho_w == R.pow2_range(float(np.abs(wf).max())) and status == 0
        assert {"s": s, "l": l} == sh_ref[0]
        assert np.array_equal(wq.cpu().numpy(), qp_ref[0]["w"])
        if bq is not None:
            assert np.array_equal(bq.cpu().numpy(), qp_ref[0]["bias"])
        else:
            assert "bias" not in qp_ref[0]
    # status bits: an output range too small for the accumulator scale, a range that is no power of two, a bias out of int32
    w = np.ones((4, 8, 3, 3), dtype=np.float32)
    for args, bit in (((4.0, 2.0 ** -12, 0.0), B.REALIZE_BAD_OUT_SHIFT), ((4.0, 3.0, 0.0), B.REALIZE_BAD_OUT_SHIFT),
                      ((4.0, 16.0, 2.0 ** 40), B.REALIZE_BAD_RES_SHIFT)):
        out = torch.zeros(4, dtype=torch.int32, device=G.DEV)
        wq = torch.empty(w.shape, dtype=torch.int8, device=G.DEV)
        ws = torch.empty(w.size * 4 + 16, dtype=torch.uint8, device=G.DEV)
        B.relay_realize_conv(4, 72, G.up(w), None, None, None, *args, wq, None, out, ws)
        torch.cuda.synchronize()
        assert out.cpu().tolist()[3] & bit, args
    out = torch.zeros(4, dtype=torch.int32, device=G.DEV)
    bq = torch.empty(4, dtype=torch.int32, device=G.DEV)
    B.relay_realize_conv(4, 72, G.up(w), G.up(np.array([1e9, 0, -1e9, 1], dtype=np.float32)), None, None, 2.0 ** -8, 2.0 ** -8, 0.0,
                         wq, bq, out, ws)
    torch.cuda.synchronize()
    assert out.cpu().tolist()[3] & B.REALIZE_BIAS_OVERFLOW
    # ranges
    cell = torch.empty(1, dtype=torch.int32, device=G.DEV)
    rho_d = torch.empty(1, dtype=torch.float32, device=G.DEV)
    for vals, dt in (([0.0, -0.0], "f32"), ([1.0, -0.25], "f32"), ([1.0001, 0.5], "f32"), ([-5.9, 3.0], "f16"), ([0.5], "f16"),
                     ([3e-4, -2e-4], "f32"), (rng.standard_normal(70001) * 37, "f32"), (rng.standard_normal(4099), "f16")):
        a = np.asarray(vals, dtype=np.float32 if dt == "f32" else np.float16)
        B.relay_calibrate_pow2_range(B.RELAY_F32 if dt == "f32" else B.RELAY_F16, a.size, G.up(a), rho_d, cell)
        torch.cuda.synchronize()
        assert float(rho_d.cpu()[0]) == R.pow2_range(float(np.max(np.abs(a.astype(np.float64))))), vals if len(vals) < 5 else dt

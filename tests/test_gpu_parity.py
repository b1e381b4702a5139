"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded
inputs.  Tolerances: fp32 1e-5, fp16 (fp32 accumulation) 1e-2 in the RMS-floored relative
error, int8 path bit-exact."""
import numpy as np
import pytest
import torch

import oracle as O
from workloads import inputs, nets

pytestmark = pytest.mark.gpu

TOL_F16, TOL_F32 = 1e-2, 1e-5


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


def _rng(i):
    return np.random.default_rng(inputs.BASE_SEED + 77000 + i)


def _h(a):
    return a.astype(np.float16)


# ------------------------------------------------------------------ config 1: fp32 NCHW
def test_config1_fp32_conv_bias_relu(G):
    from paper_1904_08368_amd import binding as B
    op = nets.conv("c", "x", "y", 3, 16, 3, 1, 1, bn=False, relu=True, bias=True)
    p = inputs.layer_params(op, 1, 0, "f32u")
    x = inputs.image(1, 1, 3, 32, 32, "f32")
    d = B.conv_desc(1, 3, 32, 32, 16, 3, 3, 1, 1, B.RELAY_F32, B.RELAY_NCHW, B.HAS_BIAS | B.RELU)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=G.DEV)
    B.relay_prepack_conv2d_weights(d, G.up(p["w"]), 3, wp)
    y = torch.full((1, 16, 32, 32), float("nan"), dtype=torch.float32, device=G.DEV)
    B.relay_fused_conv2d_bias_bn_relu(d, G.up(x), wp, G.up(p["bias"]), None, None, None, y)
    torch.cuda.synchronize()
    ref = O.fused_conv2d(x, p["w"], stride=(1, 1), pad=(1, 1), bias=p["bias"], relu_flag=True, out_dtype="f32")
    got = y.cpu().numpy()
    assert O.max_rel_err(got, ref) <= TOL_F32
    assert got.min() >= 0 and np.all(got[ref.astype(np.float64) < -1e-4] == 0)


def test_fp32_conv_all_epilogue_ops_and_strides(G):
    from paper_1904_08368_amd import binding as B
    g = _rng(1)
    x = g.uniform(-1, 1, (2, 5, 13, 11)).astype(np.float32)
    w = g.uniform(-1, 1, (7, 5, 3, 3)).astype(np.float32)
    b, sc, sf = (g.standard_normal(7).astype(np.float32) for _ in range(3))
    for st, pd in [(1, 1), (2, 1), (2, 0)]:
        d = B.conv_desc(2, 5, 13, 11, 7, 3, 3, st, pd, B.RELAY_F32, B.RELAY_NCHW, 15)
        ho, wo = B.relay_conv2d_out_shape(d)
        res = g.standard_normal((2, 7, ho, wo)).astype(np.float32)
        y = torch.empty((2, 7, ho, wo), dtype=torch.float32, device=G.DEV)
        B.relay_fused_conv2d_bias_bn_relu(d, G.up(x), G.up(w), G.up(b), G.up(sc), G.up(sf), G.up(res), y)
        torch.cuda.synchronize()
        ref = O.fused_conv2d(x, w, stride=(st, st), pad=(pd, pd), bias=b, scale=sc, shift=sf, residual=res,
                             relu_flag=True, out_dtype="f32")
        assert O.max_rel_err(y.cpu().numpy(), ref) <= TOL_F32


# ----------------------------------------------------------------------- fp16 MFMA conv
F16_CASES = [
    # n, c, h, w, k, r, stride, pad
    (1, 64, 20, 20, 64, 3, 1, 1),       # one ragged tile
    (2, 64, 29, 31, 128, 3, 1, 1),      # several tiles + ragged tail, fast path
    (2, 32, 17, 19, 96, 3, 2, 1),       # stride 2, channels not a multiple of 64
    (3, 128, 9, 9, 256, 1, 1, 0),       # 1x1
    (2, 64, 15, 15, 128, 1, 2, 0),      # 1x1 stride 2 (the ResNet shortcut)
    (2, 3, 37, 41, 64, 7, 2, 3),        # the stem: C=3 padded to 8, 7x7/s2/p3, generic tap decode
    (1, 24, 12, 12, 40, 3, 1, 1),       # C % 32 != 0 -> generic path; K % 64 != 0
    (1, 16, 10, 10, 30, 3, 1, 1),       # K % 4 != 0 -> scalar stores
    (1, 512, 7, 7, 512, 3, 1, 1),       # long reduction (4608), M=49
]


@pytest.mark.parametrize("case", F16_CASES)
def test_fp16_conv_full_epilogue(G, case):
    n, c, h, w, k, r, st, pd = case
    g = _rng(hash(case) % 1000)
    x = _h(g.standard_normal((n, c, h, w)))
    wt = _h(g.standard_normal((k, c, r, r)) * np.sqrt(2.0 / (c * r * r)))
    b = (g.standard_normal(k) * 0.1).astype(np.float32)
    sc = (1 + g.standard_normal(k) * 0.1).astype(np.float32)
    sf = (g.standard_normal(k) * 0.1).astype(np.float32)
    ho, wo = O.out_hw(h, r, st, pd), O.out_hw(w, r, st, pd)
    res = _h(g.standard_normal((n, k, ho, wo)))
    ref = O.fused_conv2d(x, wt, stride=(st, st), pad=(pd, pd), bias=b, scale=sc, shift=sf, residual=res, relu_flag=True)
    got = G.run_conv_f16(x, wt, st, pd, bias=b, scale=sc, shift=sf, residual=res, relu=True)
    assert got.shape == ref.shape and not np.isnan(got).any()
    assert O.max_rel_err(got, ref) <= TOL_F16
    pre = O.fused_conv2d(x, wt, stride=(st, st), pad=(pd, pd), bias=b, scale=sc, shift=sf, residual=res, out_dtype="f64")
    assert np.all(got[pre < -1e-2] == 0)                       # no sign leaks through the relu
    # no epilogue at all: the bare contraction
    ref0 = O.fused_conv2d(x, wt, stride=(st, st), pad=(pd, pd))
    assert O.max_rel_err(G.run_conv_f16(x, wt, st, pd), ref0) <= TOL_F16


@pytest.mark.parametrize("c", [64, 24, 128])     # 64, 128: direct-to-LDS kernel (128 admits every chunk length); 24: register-staged kernel
@pytest.mark.parametrize("tile", list(range(18)))
@pytest.mark.parametrize("n", [2, 5])            # filters larger than the activations, and the reverse: both tile orders
def test_fp16_conv_every_tile_shape(G, tile, c, n):
    g = _rng(50)
    h, w, k = 23, 27, 192
    x = _h(g.standard_normal((n, c, h, w)))
    wt = _h(g.standard_normal((k, c, 3, 3)) * np.sqrt(2.0 / (c * 9)))
    sc = (1 + g.standard_normal(k) * 0.1).astype(np.float32)
    sf = (g.standard_normal(k) * 0.1).astype(np.float32)
    ref = O.fused_conv2d(x, wt, stride=(1, 1), pad=(1, 1), scale=sc, shift=sf, relu_flag=True)
    got = G.run_conv_f16(x, wt, 1, 1, scale=sc, shift=sf, relu=True, tile=tile)
    assert O.max_rel_err(got, ref) <= TOL_F16


@pytest.mark.parametrize("case", [(2, 3, 37, 41, 64, 7, 2, 3), (1, 3, 20, 33, 32, 3, 2, 1), (2, 4, 9, 9, 16, 5, 1, 2),
                                  (1, 1, 12, 12, 8, 3, 1, 0)])
def test_first_layer_both_input_layouts(G, case):
    """<= 4 input channels: the pre-padded NHWC4 path and the channel-padded NHWC path agree
    with the oracle (fp16) and bit for bit (int8)."""
    n, c, h, w, k, r, st, pd = case
    g = _rng(60 + h)
    x = _h(g.standard_normal((n, c, h, w)))
    wt = _h(g.standard_normal((k, c, r, r)) * np.sqrt(2.0 / (c * r * r)))
    sc = (1 + g.standard_normal(k) * 0.1).astype(np.float32)
    sf = (g.standard_normal(k) * 0.1).astype(np.float32)
    ref = O.fused_conv2d(x, wt, stride=(st, st), pad=(pd, pd), scale=sc, shift=sf, relu_flag=True)
    for nhwc4 in (True, False):
        got = G.run_conv_f16(x, wt, st, pd, scale=sc, shift=sf, relu=True, nhwc4=nhwc4)
        assert got.shape == ref.shape and O.max_rel_err(got, ref) <= TOL_F16, nhwc4
    xi = g.integers(-127, 128, (n, c, h, w)).astype(np.int8)
    wi = g.integers(-127, 128, (k, c, r, r)).astype(np.int8)
    s = inputs.default_out_rshift(c * r * r)
    refq = O.qconv2d_requant(xi, wi, stride=(st, st), pad=(pd, pd), out_rshift=s, relu_flag=True)
    for nhwc4 in (True, False):
        assert np.array_equal(G.run_qconv(xi, wi, st, pd, rshift=s, relu=True, nhwc4=nhwc4), refq), nhwc4


def test_fp16_delta_kernel_reproduces_input(G):
    g = _rng(51)
    x = _h(g.standard_normal((1, 64, 14, 14)))
    wt = np.zeros((64, 64, 3, 3), dtype=np.float16)
    for i in range(64):
        wt[i, i, 1, 1] = 1
    assert np.array_equal(G.run_conv_f16(x, wt, 1, 1), x)
    wt = np.zeros((64, 64, 3, 3), dtype=np.float16)
    for i in range(64):
        wt[i, i, 0, 2] = 1                                      # off-centre: no flip, shift (-1, +1)
    got = G.run_conv_f16(x, wt, 1, 1)
    want = np.zeros_like(x)
    want[:, :, 1:, :-1] = x[:, :, :-1, 1:]
    assert np.array_equal(got, want)


# --------------------------------------------------------------------- int8 MFMA conv
I8_CASES = [
    (1, 64, 20, 20, 64, 3, 1, 1),
    (2, 64, 29, 31, 128, 3, 1, 1),
    (2, 32, 17, 19, 96, 3, 2, 1),
    (3, 128, 9, 9, 256, 1, 1, 0),
    (2, 64, 15, 15, 128, 1, 2, 0),
    (2, 3, 37, 41, 64, 7, 2, 3),
    (1, 48, 12, 12, 40, 3, 1, 1),
    (1, 16, 10, 10, 30, 3, 1, 1),
    (1, 512, 7, 7, 512, 3, 1, 1),
]


@pytest.mark.parametrize("case", I8_CASES)
def test_int8_qconv_bit_exact(G, case):
    n, c, h, w, k, r, st, pd = case
    g = _rng(100 + hash(case) % 1000)
    x = g.integers(-127, 128, (n, c, h, w)).astype(np.int8)
    wt = g.integers(-127, 128, (k, c, r, r)).astype(np.int8)
    ho, wo = O.out_hw(h, r, st, pd), O.out_hw(w, r, st, pd)
    res = g.integers(-127, 128, (n, k, ho, wo)).astype(np.int8)
    bias = g.integers(-20000, 20000, k)
    s = inputs.default_out_rshift(c * r * r)
    for kw in (dict(), dict(relu=True), dict(bias=bias, residual=res, lshift=s, relu=True),
               dict(bias=bias, residual=res, lshift=3, relu=False)):
        ref = O.qconv2d_requant(x, wt, stride=(st, st), pad=(pd, pd), bias=kw.get("bias"), residual=kw.get("residual"),
                                residual_lshift=kw.get("lshift", 0), out_rshift=s, relu_flag=kw.get("relu", False))
        got = G.run_qconv(x, wt, st, pd, rshift=s, **kw)
        assert got.dtype == np.int8 and np.array_equal(got, ref), kw.keys()
    # shift 0 (no rounding term) and a small shift that saturates almost everywhere
    for s2 in (0, 2, 31):
        ref = O.qconv2d_requant(x, wt, stride=(st, st), pad=(pd, pd), out_rshift=s2)
        assert np.array_equal(G.run_qconv(x, wt, st, pd, rshift=s2), ref)


@pytest.mark.parametrize("c", [64, 48, 256])     # 256 int8 channels admit every chunk length
@pytest.mark.parametrize("tile", list(range(18)))
def test_int8_every_tile_shape_and_repeatable(G, tile, c):
    g = _rng(150)
    x = g.integers(-127, 128, (2, c, 23, 27)).astype(np.int8)
    wt = g.integers(-127, 128, (192, c, 3, 3)).astype(np.int8)
    ref = O.qconv2d_requant(x, wt, stride=(1, 1), pad=(1, 1), out_rshift=12, relu_flag=True)
    for _ in range(3):
        assert np.array_equal(G.run_qconv(x, wt, 1, 1, rshift=12, relu=True, tile=tile), ref)


def test_int8_rounding_ties_through_the_kernel(G):
    # 1x1 conv with a single non-zero weight of 1 makes acc = x, so the epilogue is tested
    # on chosen accumulator values: ties at +-0.5 and the clip bounds.
    x = np.zeros((1, 16, 4, 4), dtype=np.int8)
    vals = np.array([-128, -127, -7, -6, -5, -3, -2, -1, 0, 1, 2, 3, 5, 6, 7, 127], dtype=np.int8)
    x[0, 0] = vals.reshape(4, 4)
    wt = np.zeros((4, 16, 1, 1), dtype=np.int8)
    wt[:, 0, 0, 0] = [1, -1, 127, -127]
    for s in (0, 1, 2, 3):
        ref = O.qconv2d_requant(x, wt, out_rshift=s)
        got = G.run_qconv(x, wt, 1, 0, rshift=s)
        assert np.array_equal(got, ref), s
    assert G.run_qconv(x, wt, 1, 0, rshift=1)[0, 0].ravel().tolist()[4:7] == [-2, -1, -1]   # -2.5->-2, -1.5->-1, -1->-1


# -------------------------------------------------------------------------- depthwise
@pytest.mark.parametrize("case", [(2, 32, 19, 23, 1), (2, 64, 19, 23, 2), (1, 8, 7, 7, 1), (3, 128, 14, 14, 2),
                                  (1, 1024, 7, 7, 1), (1, 40, 5, 9, 2),
                                  # rows of 28 pixels and more at stride 1: the LDS-staged kernel, exact and ragged tiles
                                  (2, 64, 30, 37, 1), (1, 96, 17, 28, 1), (2, 128, 56, 56, 1), (1, 32, 9, 61, 1)])
def test_dwconv_f16(G, case):
    n, c, h, w, st = case
    g = _rng(200 + c + st)
    x = _h(g.standard_normal((n, c, h, w)))
    wt = _h(g.standard_normal((c, 3, 3)) * np.sqrt(2.0 / 9))
    sc = (1 + g.standard_normal(c) * 0.1).astype(np.float32)
    sf = (g.standard_normal(c) * 0.1).astype(np.float32)
    b = (g.standard_normal(c) * 0.1).astype(np.float32)
    ref = O.fused_dwconv2d(x, wt, stride=(st, st), pad=(1, 1), scale=sc, shift=sf, relu_flag=True)
    got = G.run_dwconv_f16(x, wt, st, 1, scale=sc, shift=sf, relu=True)
    assert got.shape == ref.shape and O.max_rel_err(got, ref) <= TOL_F16
    ref = O.fused_dwconv2d(x, wt, stride=(st, st), pad=(1, 1), bias=b)
    assert O.max_rel_err(G.run_dwconv_f16(x, wt, st, 1, bias=b), ref) <= TOL_F16


# ------------------------------------------------------------------------------ dense
@pytest.mark.parametrize("m,n,k", [(1, 1000, 512), (32, 1000, 1024), (5, 37, 24), (9, 130, 2048), (32, 1000, 512), (17, 37, 192), (70, 136, 64)])
def test_dense(G, m, n, k):
    from paper_1904_08368_amd import binding as B
    g = _rng(300 + m)
    x = g.standard_normal((m, k))
    w = g.standard_normal((n, k)) * np.sqrt(2.0 / k)
    b = (g.standard_normal(n) * 0.1).astype(np.float32)
    for dt, npdt, tdt, tol in ((B.RELAY_F16, np.float16, torch.float16, TOL_F16), (B.RELAY_F32, np.float32, torch.float32, TOL_F32)):
        xx, ww = x.astype(npdt), w.astype(npdt)
        for act in (0, 1):
            y = torch.full((m, n), float("nan"), dtype=tdt, device=G.DEV)
            B.relay_fused_dense_bias_act(m, n, k, dt, G.up(xx), G.up(ww), G.up(b), act, y)
            torch.cuda.synchronize()
            ref = O.fused_dense(xx, ww, bias=b, relu_flag=bool(act), out_dtype="f16" if dt == B.RELAY_F16 else "f32")
            assert O.max_rel_err(y.cpu().numpy(), ref) <= tol


# ------------------------------------------------------------------------ glue kernels
def test_pools_and_layout(G):
    from paper_1904_08368_amd import binding as B
    g = _rng(400)
    x = _h(g.standard_normal((2, 16, 13, 15)))
    xd = G.to_nhwc(x, 16, B.RELAY_F16)
    assert np.array_equal(G.from_nhwc(xd, 16), x)
    xp = G.to_nhwc(x[:, :3], 8, B.RELAY_F16)
    assert np.array_equal(G.from_nhwc(xp, 3), x[:, :3]) and float(xp[..., 3:].abs().max()) == 0.0
    y = torch.empty((2, 7, 8, 16), dtype=torch.float16, device=G.DEV)
    B.relay_maxpool2d(B.RELAY_F16, 2, 16, 13, 15, 3, 2, 1, xd, y)
    torch.cuda.synchronize()
    assert np.array_equal(G.from_nhwc(y, 16), O.maxpool2d(x, 3, 2, 1).astype(np.float16))
    a = torch.empty((2, 1, 1, 16), dtype=torch.float16, device=G.DEV)
    B.relay_global_avgpool(B.RELAY_F16, 2, 16, 13 * 15, xd, a)
    torch.cuda.synchronize()
    assert O.max_rel_err(a.cpu().numpy().reshape(2, 16), O.cast_f16(O.global_avgpool(x))) <= TOL_F16
    xi = g.integers(-128, 128, (2, 16, 9, 9)).astype(np.int8)
    yi = torch.empty((2, 5, 5, 16), dtype=torch.int8, device=G.DEV)
    B.relay_maxpool2d(B.RELAY_I8, 2, 16, 9, 9, 3, 2, 1, G.to_nhwc(xi, 16, B.RELAY_I8), yi)
    torch.cuda.synchronize()
    assert np.array_equal(G.from_nhwc(yi, 16), O.maxpool2d(xi, 3, 2, 1).astype(np.int8))


@pytest.mark.parametrize("geom", [(3, 1, 1), (3, 2, 0), (3, 3, 2), (3, 2, 2), (2, 2, 0), (2, 1, 1), (5, 2, 2)])
def test_maxpool_window_stride_and_padding(G, geom):
    """Negative inputs next to the border: padding must never win the maximum, whichever kernel runs
    (3x3 windows: the branch-free one; other sizes: the general one)."""
    from paper_1904_08368_amd import binding as B
    r, st, pd = geom
    g = _rng(410 + r + st)
    n, c, h, w = 3, 24, 11, 14
    x = _h(g.standard_normal((n, c, h, w)) - 3.0)              # mostly negative
    ho, wo = (h + 2 * pd - r) // st + 1, (w + 2 * pd - r) // st + 1
    y = torch.empty((n, ho, wo, c), dtype=torch.float16, device=G.DEV)
    B.relay_maxpool2d(B.RELAY_F16, n, c, h, w, r, st, pd, G.to_nhwc(x, c, B.RELAY_F16), y)
    torch.cuda.synchronize()
    assert np.array_equal(G.from_nhwc(y, c), O.maxpool2d(x, r, st, pd).astype(np.float16))


# ------------------------------------------------------------- 3x3 kernel with one-time staging
HALO_SHAPES = [  # n, c, h, w, k
    (2, 64, 23, 27, 192), (1, 32, 9, 11, 37), (3, 128, 14, 14, 128), (1, 256, 7, 7, 64), (2, 64, 56, 56, 64),
    (5, 96, 5, 6, 72), (1, 64, 1, 1, 64), (2, 64, 2, 40, 24),
    # several 256-byte chunks (the 64 x 64 tile's long-chunk form), one chunk, a halo too wide for it
    (1, 512, 7, 7, 192), (2, 128, 9, 11, 72), (1, 384, 5, 20, 24), (1, 384, 5, 40, 24),
]


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("shape", HALO_SHAPES)
def test_fp16_halo_kernel(G, shape, variant):
    from paper_1904_08368_amd import binding as B
    n, c, h, w, k = shape
    g = _rng(900 + c + h)
    x = _h(g.standard_normal((n, c, h, w)))
    wt = _h(g.standard_normal((k, c, 3, 3)) * np.sqrt(2.0 / (c * 9)))
    sc = (1 + g.standard_normal(k) * 0.1).astype(np.float32)
    sf = (g.standard_normal(k) * 0.1).astype(np.float32)
    res = _h(g.standard_normal((n, k, h, w)))
    d = B.conv_desc(n, c, h, w, k, 3, 3, 1, 1, B.RELAY_F16, B.RELAY_NHWC, 0)
    B.relay_set_conv_tile(100 + variant)
    try:
        assert "halo" in B.relay_conv2d_kernel_name(d), "the forced variant does not take this shape"
    finally:
        B.relay_set_conv_tile(-1)
    ref = O.fused_conv2d(x, wt, stride=(1, 1), pad=(1, 1), scale=sc, shift=sf, residual=res, relu_flag=True)
    got = G.run_conv_f16(x, wt, 1, 1, scale=sc, shift=sf, residual=res, relu=True, tile=100 + variant)
    assert got.shape == ref.shape and not np.isnan(got).any()
    assert O.max_rel_err(got, ref) <= TOL_F16
    ref0 = O.fused_conv2d(x, wt, stride=(1, 1), pad=(1, 1))
    assert O.max_rel_err(G.run_conv_f16(x, wt, 1, 1, tile=100 + variant), ref0) <= TOL_F16


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("shape", [(2, 64, 23, 27, 192), (1, 128, 9, 11, 40), (2, 256, 14, 14, 64), (1, 64, 56, 56, 64), (1, 512, 7, 7, 136),
                                   (3, 768, 5, 6, 72)])
def test_int8_halo_kernel_bit_exact(G, shape, variant):
    n, c, h, w, k = shape
    g = _rng(950 + c + h)
    x = g.integers(-127, 128, (n, c, h, w)).astype(np.int8)
    wt = g.integers(-127, 128, (k, c, 3, 3)).astype(np.int8)
    res = g.integers(-127, 128, (n, k, h, w)).astype(np.int8)
    b = g.integers(-3000, 3000, k).astype(np.int32)
    ref = O.qconv2d_requant(x, wt, stride=(1, 1), pad=(1, 1), bias=b, residual=res, residual_lshift=12, out_rshift=12,
                            relu_flag=True)
    for _ in range(2):
        got = G.run_qconv(x, wt, 1, 1, bias=b, residual=res, lshift=12, rshift=12, relu=True, tile=100 + variant)
        assert np.array_equal(got, ref)


# -------------------------------------------------------------------------- maximum sizes
def _pattern(shape, dtype):
    """A cheap deterministic tensor (no generator can fill 2 GB in seconds): small signed values that
    depend on every coordinate."""
    n, c, h, w = shape
    v = (np.arange(n, dtype=np.int16).reshape(n, 1, 1, 1) * 7 + np.arange(c, dtype=np.int16).reshape(1, c, 1, 1) * 17 +
         np.arange(h, dtype=np.int16).reshape(1, 1, h, 1) * 131 + np.arange(w, dtype=np.int16).reshape(1, 1, 1, w) * 71)
    v = (v % 13 - 6).astype(np.int8)
    return v if dtype == np.int8 else (v.astype(np.float16) / np.float16(8))


@pytest.mark.parametrize("mode", ["f16", "i8"])
def test_conv_input_at_the_2_31_byte_limit(G, mode):
    """The largest input the 32-bit buffer offsets admit (2^31 - 1 bytes): outputs sampled near the
    far end of the tensor, where an offset that wrapped or lost its top bit would read elsewhere."""
    if mode == "f16":
        n, c, h, w, k = 3, 64, 2364, 2364, 16
        assert n * c * h * w * 2 <= 2 ** 31 - 1 < n * c * (h + 1) * (w + 1) * 2
    else:
        n, c, h, w, k = 2, 64, 4096, 4095, 16
        assert n * c * h * w <= 2 ** 31 - 1
    g = _rng(990)
    x = _pattern((n, c, h, w), np.int8 if mode == "i8" else np.float16)
    pts = [(n - 1, int(g.integers(0, k)), int(g.integers(h - 40, h)), int(g.integers(0, w))) for _ in range(120)]
    pts += [(n - 1, k - 1, h - 1, w - 1), (n - 1, 0, h - 1, 0), (0, 0, 0, 0), (n - 1, 3, h - 2, w - 1)]
    if mode == "f16":
        wt = _h(g.standard_normal((k, c, 3, 3)) * np.sqrt(2.0 / (c * 9)))
        got = G.run_conv_f16(x, wt, 1, 1, relu=True)
        acc = O.conv2d_points(x, wt, pts, (1, 1), (1, 1))
        want = O.cast_f16(np.maximum(acc, 0.0)).astype(np.float64)
        gv = np.array([got[t] for t in pts], dtype=np.float64)
        assert np.max(np.abs(gv - want) / np.maximum(np.abs(want), 0.05)) <= TOL_F16
        assert np.any(want > 0)
    else:
        wt = g.integers(-127, 128, (k, c, 3, 3)).astype(np.int8)
        got = G.run_qconv(x, wt, 1, 1, rshift=9)
        acc = O.conv2d_points(x, wt, pts, (1, 1), (1, 1), integer=True)
        want = O.requant_points(acc, out_rshift=9)
        assert np.array_equal(np.array([got[t] for t in pts]), want)


@pytest.mark.parametrize("stride", [1, 2])
def test_dwconv_input_at_the_2_31_byte_limit(G, stride):
    n, c, h, w = 1, 32, 5793, 5792
    assert n * c * h * w * 2 <= 2 ** 31 - 1 < n * c * (h + 1) * w * 2
    g = _rng(991 + stride)
    x = _pattern((n, c, h, w), np.float16)
    wt = _h(g.standard_normal((c, 3, 3)) * np.sqrt(2.0 / 9))
    got = G.run_dwconv_f16(x, wt, stride, 1, relu=True)
    ho, wo = got.shape[2], got.shape[3]
    pts = [(0, int(g.integers(0, c)), int(g.integers(ho - 30, ho)), int(g.integers(0, wo))) for _ in range(120)]
    pts += [(0, c - 1, ho - 1, wo - 1), (0, 0, ho - 1, 0), (0, 0, 0, 0), (0, 5, ho - 1, wo - 2)]
    acc = O.dwconv2d_points(x, wt, pts, (stride, stride), (1, 1))
    want = O.cast_f16(np.maximum(acc, 0.0)).astype(np.float64)
    gv = np.array([got[t] for t in pts], dtype=np.float64)
    assert np.max(np.abs(gv - want) / np.maximum(np.abs(want), 0.05)) <= TOL_F16
    assert np.any(want > 0)

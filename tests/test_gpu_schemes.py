"""GPU parity of the further quantization schemes (paper Section 4.2; the 8/16 and 16/32 rows of the
accuracy table of Section 5.4): general per-channel scales, the 16-bit accumulator, int16 operands,
unsigned activations -- every result bit for bit against oracle.schemes."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import schemes as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    from paper_1904_08368_amd import binding as B
    B.lib()
    assert torch.cuda.is_available()
    from tests import gpu_util
    return gpu_util


def _setup_i8(G, B, x, w, stride, pad, flags):
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    d = B.conv_desc(n, c, h, wd, k, r, s, stride, pad, B.RELAY_I8, B.RELAY_NHWC, flags)
    ho, wo = B.relay_conv2d_out_shape(d)
    xd = G.to_nhwc(x, c, B.RELAY_I8)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=G.DEV)
    B.relay_prepack_conv2d_weights(d, G.up(w), c, wp)
    return d, xd, wp, ho, wo


@pytest.mark.parametrize("tile", [-1, 100, 5])         # heuristics, the 3x3 stride-1 kernel, a forced implicit-GEMM tile
@pytest.mark.parametrize("shape", [(2, 64, 13, 17, 72, 3, 1, 1), (1, 48, 9, 11, 40, 3, 2, 1), (2, 128, 7, 7, 64, 1, 1, 0)])
def test_scaled_requant_per_channel_bit_exact(G, tile, shape):
    from paper_1904_08368_amd import binding as B
    n, c, h, w, k, r, stride, pad = shape
    g = np.random.default_rng(400 + c + k)
    x = g.integers(-127, 128, (n, c, h, w)).astype(np.int8)
    wt = g.integers(-127, 128, (k, c, r, r)).astype(np.int8)
    b = g.integers(-5000, 5000, k).astype(np.int32)
    ho, wo = O.out_hw(h, r, stride, pad), O.out_hw(w, r, stride, pad)
    res = g.integers(-127, 128, (n, k, ho, wo)).astype(np.int8)
    scales = 2.0 ** g.uniform(-15, -9, k)                       # general scales, one per output channel
    ms = [S.quantize_multiplier(float(v)) for v in scales]
    mult, rsh = np.array([m for m, _ in ms], dtype=np.int32), np.array([s for _, s in ms], dtype=np.int32)
    for use_res, relu in ((True, False), (False, True)):
        ref = S.qconv2d_requant_scaled(x, wt, stride=(stride, stride), pad=(pad, pad), bias=b, residual=res if use_res else None,
                                       residual_lshift=9, mult=mult, rshift=rsh, relu_flag=relu)
        d, xd, wp, _, _ = _setup_i8(G, B, x, wt, stride, pad, B.flags_of(b, None, res if use_res else None, relu))
        y = torch.full((n, ho, wo, k), -128, dtype=torch.int8, device=G.DEV)
        B.relay_set_conv_tile(tile)
        try:
            B.relay_qconv2d_requant_scaled(d, xd, wp, G.up(b), G.to_nhwc(res, k, B.RELAY_I8) if use_res else None, 9, G.up(mult), G.up(rsh), y)
        finally:
            B.relay_set_conv_tile(-1)
        torch.cuda.synchronize()
        assert np.array_equal(G.from_nhwc(y, k), ref), (shape, tile, use_res)
    # the multiplier 2^30 with shift s - 1 is the power-of-two entry point with shift s
    half = np.full(k, 1 << 30, dtype=np.int32)
    d, xd, wp, _, _ = _setup_i8(G, B, x, wt, stride, pad, B.flags_of(b, None, None, True))
    y = torch.empty((n, ho, wo, k), dtype=torch.int8, device=G.DEV)
    B.relay_qconv2d_requant_scaled(d, xd, wp, G.up(b), None, 0, G.up(half), G.up(np.full(k, 11, dtype=np.int32)), y)
    torch.cuda.synchronize()
    assert np.array_equal(G.from_nhwc(y, k), G.run_qconv(x, wt, stride, pad, bias=b, rshift=12, relu=True))


def test_library_multiplier_decomposition_equals_the_oracle(G):
    from paper_1904_08368_amd import binding as B
    g = np.random.default_rng(410)
    for v in list(2.0 ** g.uniform(-31.5, -1e-9, 500)) + [0.5, 0.75, 2.0 ** -20, 0.99999999999, 1.0 - 2.0 ** -33, 2.0 ** -31 * 1.5]:
        assert B.relay_quantize_multiplier(float(v)) == S.quantize_multiplier(float(v)), v
    for bad in (0.0, 1.0, -0.5, 2.0 ** -40, float("inf")):
        with pytest.raises(B.RelayError):
            B.relay_quantize_multiplier(bad)


@pytest.mark.parametrize("tile", [-1, 100])
def test_acc16_scheme_bit_exact_in_range_and_saturated(G, tile):
    from paper_1904_08368_amd import binding as B
    g = np.random.default_rng(420)
    for lim, fits in ((7, True), (127, False)):                 # 4-bit magnitudes keep the sums in 16 bits; full-range ones saturate
        x = g.integers(-lim, lim + 1, (2, 64, 9, 10)).astype(np.int8)
        wt = g.integers(-lim, lim + 1, (72, 64, 3, 3)).astype(np.int8)
        b = g.integers(-300, 300, 72).astype(np.int32)
        res = g.integers(-lim, lim + 1, (2, 72, 9, 10)).astype(np.int8)
        assert S.fits_int16(x, wt, pad=(1, 1), bias=b, residual=res, residual_lshift=3) == fits
        s = 5 if fits else 8
        ref = S.qconv2d_requant_acc16(x, wt, stride=(1, 1), pad=(1, 1), bias=b, residual=res, residual_lshift=3, out_rshift=s, relu_flag=False)
        d, xd, wp, ho, wo = _setup_i8(G, B, x, wt, 1, 1, B.flags_of(b, None, res, False))
        y = torch.full((2, ho, wo, 72), -128, dtype=torch.int8, device=G.DEV)
        B.relay_set_conv_tile(tile)
        try:
            B.relay_qconv2d_requant_acc16(d, xd, wp, G.up(b), G.to_nhwc(res, 72, B.RELAY_I8), 3, s, y)
        finally:
            B.relay_set_conv_tile(-1)
        torch.cuda.synchronize()
        got = G.from_nhwc(y, 72)
        assert np.array_equal(got, ref), (lim, tile)
        if fits:      # within its precondition the scheme equals 8/32
            assert np.array_equal(got, O.qconv2d_requant(x, wt, stride=(1, 1), pad=(1, 1), bias=b, residual=res, residual_lshift=3, out_rshift=s))
        else:
            assert (np.abs(got.astype(int)) == 127).mean() > 0.2


@pytest.mark.parametrize("shape", [(2, 16, 9, 11, 20, 3, 1, 1), (1, 24, 13, 8, 8, 3, 2, 1), (2, 8, 6, 6, 12, 1, 1, 0), (1, 8, 15, 15, 4, 7, 2, 3)])
def test_int16_scheme_bit_exact(G, shape):
    from paper_1904_08368_amd import binding as B
    n, c, h, w, k, r, stride, pad = shape
    g = np.random.default_rng(430 + c)
    x = g.integers(-2000, 2001, (n, c, h, w)).astype(np.int16)
    wt = g.integers(-2000, 2001, (k, c, r, r)).astype(np.int16)
    x[0, 0, 0, :3] = [32767, -32768, 32767]
    wt[0, 0, 0, 0] = -32768
    b = g.integers(-10 ** 6, 10 ** 6, k).astype(np.int32)
    for s, relu, bias in ((12, False, b), (0, True, None), (20, True, b)):
        ref = S.qconv2d_requant_i16(x, wt, stride=(stride, stride), pad=(pad, pad), bias=bias, out_rshift=s, relu_flag=relu)
        d = B.conv_desc(n, c, h, w, k, r, r, stride, pad, B.RELAY_I16, B.RELAY_NHWC, B.flags_of(bias, None, None, relu))
        ho, wo = B.relay_conv2d_out_shape(d)
        xd = G.to_nhwc(x, c, B.RELAY_I16)
        wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=G.DEV)
        B.relay_prepack_conv2d_weights(d, G.up(wt), c, wp)
        y = torch.full((n, ho, wo, k), -32768, dtype=torch.int16, device=G.DEV)
        B.relay_qconv2d_requant_i16(d, xd, wp, G.up(bias) if bias is not None else None, s, y)
        torch.cuda.synchronize()
        assert np.array_equal(G.from_nhwc(y, k), ref), (shape, s)


@pytest.mark.parametrize("shape", [(2, 64, 13, 17, 72, 3, 1, 1), (1, 16, 20, 21, 32, 7, 2, 3), (2, 128, 7, 7, 64, 1, 1, 0), (1, 48, 9, 11, 40, 3, 2, 1)])
def test_unsigned_activations_bit_exact(G, shape):
    from paper_1904_08368_amd import binding as B
    n, c, h, w, k, r, stride, pad = shape
    g = np.random.default_rng(440 + c)
    x = g.integers(0, 256, (n, c, h, w)).astype(np.uint8)
    x[0, 0, 0, :4] = [0, 255, 128, 127]
    wt = g.integers(-127, 128, (k, c, r, r)).astype(np.int8)
    b = g.integers(-5000, 5000, k).astype(np.int32)
    d = B.conv_desc(n, c, h, w, k, r, r, stride, pad, B.RELAY_I8, B.RELAY_NHWC, B.flags_of(b, None, None, True))
    ho, wo = B.relay_conv2d_out_shape(d)
    xd = torch.from_numpy(np.ascontiguousarray(x.transpose(0, 2, 3, 1))).to(G.DEV)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=G.DEV)
    B.relay_prepack_conv2d_weights(d, G.up(wt), c, wp)
    for bias in (b, None):
        bz = torch.empty(k, dtype=torch.int32, device=G.DEV)
        B.relay_fold_zero_point(k, c * r * r, G.up(wt), G.up(bias) if bias is not None else None, 128, bz)
        torch.cuda.synchronize()
        want_bz = (0 if bias is None else bias.astype(np.int64)) + 128 * wt.astype(np.int64).sum(axis=(1, 2, 3))
        assert np.array_equal(bz.cpu().numpy().astype(np.int64), want_bz)
        ws = torch.empty(B.relay_qconv2d_u8_workspace_bytes(d), dtype=torch.uint8, device=G.DEV)
        for out_unsigned in (False, True):
            s = int(np.log2(np.sqrt(c * r * r) * 128 * 74 / 60)) - 1      # codes that fill the 8-bit range without saturating everywhere
            ref = S.qconv2d_requant_u8(x, wt, stride=(stride, stride), pad=(pad, pad), bias=bias, out_rshift=s, relu_flag=True,
                                       out_unsigned=out_unsigned)
            y = torch.full((n, ho, wo, k), 77, dtype=torch.uint8, device=G.DEV)
            B.relay_qconv2d_requant_u8(d, xd, wp, bz, s, out_unsigned, y, ws)
            torch.cuda.synchronize()
            got = y.permute(0, 3, 1, 2).contiguous().cpu().numpy()
            got = got if out_unsigned else got.view(np.int8)
            assert np.array_equal(got, ref), (shape, out_unsigned)
            assert not out_unsigned or got.max() > 127           # the unsigned range is really used

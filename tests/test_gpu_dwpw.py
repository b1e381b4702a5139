"""The depthwise conv and its 1x1 conv as one launch (paper Sections 4.1 and 5.2), against the oracle's
two fused operators with the fp16 narrowing in between, and bit for bit against the two separate launches."""
import numpy as np
import pytest
import torch

import oracle as O
from workloads import inputs

pytestmark = pytest.mark.gpu

TOL_F16 = 1e-2
# stride of every kernel variant, in the library's order
VARIANT_STRIDE = (1, 1, 1, 1, 1, 2, 2, 2, 2, 2)
# variants that take one channel count only (the whole reduction is one chunk)
VARIANT_ONLY_C = {1: 32, 5: 64}
N_VARIANTS = len(VARIANT_STRIDE)


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


def _rng(i):
    return np.random.default_rng(inputs.BASE_SEED + 88000 + i)


def _h(a):
    return a.astype(np.float16)


def _params(g, c):
    return ((1 + g.standard_normal(c) * 0.1).astype(np.float32), (g.standard_normal(c) * 0.1).astype(np.float32),
            (g.standard_normal(c) * 0.1).astype(np.float32))


def _run(G, x, wd, wp, st, dw_tail, pw_tail, variant=-1):
    """dw_tail / pw_tail: (bias, scale, shift, relu).  Returns (fused, two launches) as NCHW fp16."""
    from paper_1904_08368_amd import binding as B
    n, c, h, w = x.shape
    k = wp.shape[0]
    db, dsc, dsf, drelu = dw_tail
    pb, psc, psf, prelu = pw_tail
    dd = B.conv_desc(n, c, h, w, c, 3, 3, st, 1, B.RELAY_F16, B.RELAY_NHWC, B.flags_of(db, dsc, None, drelu))
    ho, wo = B.relay_conv2d_out_shape(dd)
    pflags = B.flags_of(pb, psc, None, prelu)
    pd = B.conv_desc(n, c, ho, wo, k, 1, 1, 1, 0, B.RELAY_F16, B.RELAY_NHWC, pflags)
    xd = G.to_nhwc(x, c, B.RELAY_F16)
    wdd = torch.empty((9, c), dtype=torch.float16, device=G.DEV)
    B.relay_prepack_dwconv_weights(dd, G.up(wd), wdd)
    wpp = torch.empty(B.relay_packed_weight_bytes(pd), dtype=torch.uint8, device=G.DEV)
    B.relay_prepack_conv2d_weights(pd, G.up(wp.reshape(k, c, 1, 1)), c, wpp)
    y = torch.full((n, ho, wo, k), float("nan"), dtype=torch.float16, device=G.DEV)
    B.relay_set_conv_tile(-1 if variant < 0 else 300 + variant)
    try:
        B.relay_fused_dwconv_pwconv(dd, xd, wdd, G.up(db), G.up(dsc), G.up(dsf), k, pflags, wpp, G.up(pb), G.up(psc), G.up(psf), y)
    finally:
        B.relay_set_conv_tile(-1)
    t = torch.full((n, ho, wo, c), float("nan"), dtype=torch.float16, device=G.DEV)
    y2 = torch.full((n, ho, wo, k), float("nan"), dtype=torch.float16, device=G.DEV)
    B.relay_fused_dwconv_bias_relu(dd, xd, wdd, G.up(db), G.up(dsc), G.up(dsf), t)
    B.relay_fused_conv2d_bias_bn_relu(pd, t, wpp, G.up(pb), G.up(psc), G.up(psf), None, y2, None)
    torch.cuda.synchronize()
    return G.from_nhwc(y, k), G.from_nhwc(y2, k)


def _oracle(x, wd, wp, st, dw_tail, pw_tail):
    db, dsc, dsf, drelu = dw_tail
    pb, psc, psf, prelu = pw_tail
    t = O.fused_dwconv2d(x, wd, stride=(st, st), pad=(1, 1), bias=db, scale=dsc, shift=dsf, relu_flag=drelu)     # fp16
    return O.fused_conv2d(t, wp.reshape(wp.shape[0], -1, 1, 1), bias=pb, scale=psc, shift=psf, relu_flag=prelu)


def _case(G, seed, n, c, h, w, k, st, variant=-1, plain_tail=False):
    g = _rng(seed)
    x = _h(g.standard_normal((n, c, h, w)))
    wd = _h(g.standard_normal((c, 3, 3)) * np.sqrt(2.0 / 9))
    wp = _h(g.standard_normal((k, c)) * np.sqrt(2.0 / c))
    dsc, dsf, db = _params(g, c)
    psc, psf, pb = _params(g, k)
    dw_tail = (db, None, None, False) if plain_tail else (None, dsc, dsf, True)
    pw_tail = (None, None, None, False) if plain_tail else (pb, psc, psf, True)
    got, two = _run(G, x, wd, wp, st, dw_tail, pw_tail, variant)
    ref = _oracle(x, wd, wp, st, dw_tail, pw_tail)
    assert got.shape == ref.shape
    assert O.max_rel_err(got, ref) <= TOL_F16
    assert np.array_equal(got.view(np.uint16), two.view(np.uint16))     # same sums in the same order as the two launches


# the MobileNet block shapes at a small batch, and shapes whose rectangles are ragged on both sides
@pytest.mark.parametrize("case", [(2, 32, 112, 112, 64, 1), (1, 64, 112, 112, 128, 2), (2, 128, 56, 56, 128, 1),
                                  (2, 128, 56, 56, 256, 2), (2, 256, 28, 28, 256, 1), (2, 256, 28, 28, 512, 2),
                                  (3, 512, 14, 14, 512, 1), (3, 512, 14, 14, 1024, 2), (3, 1024, 7, 7, 1024, 1),
                                  (2, 64, 19, 23, 72, 1), (1, 96, 17, 31, 40, 2), (1, 32, 5, 9, 8, 1), (2, 160, 9, 6, 136, 2)])
def test_dwpw_default_variant(G, case):
    n, c, h, w, k, st = case
    _case(G, c + k + st, n, c, h, w, k, st)
    _case(G, c + k + st + 1, n, c, h, w, k, st, plain_tail=True)


@pytest.mark.parametrize("variant", range(N_VARIANTS))
def test_dwpw_every_variant_on_ragged_shapes(G, variant):
    """Every kernel variant on images that its rectangle does not divide, with channel counts that leave a
    partial channel tile (the fused kernel's masks, not only the shapes it was tuned for)."""
    st = VARIANT_STRIDE[variant]
    for i, (n, c, h, w, k) in enumerate([(2, 64, 17, 29, 72), (1, 128, 33, 15, 200), (2, 64, 8, 16, 128)]):
        c = VARIANT_ONLY_C.get(variant, c)
        _case(G, 100 + 10 * variant + i, n, c, h, w, k, st, variant=variant)


def test_variant_count_matches_library(G):
    """One past the last variant is refused by the library."""
    from paper_1904_08368_amd import binding as B
    g = _rng(7)
    x = _h(g.standard_normal((1, 64, 8, 8)))
    wd = _h(g.standard_normal((64, 3, 3)))
    wp = _h(g.standard_normal((64, 64)))
    with pytest.raises(Exception):
        _run(G, x, wd, wp, 1, (None, None, None, False), (None, None, None, False), variant=N_VARIANTS)

"""The allocation-free conv entry point (reduction-split scratch in a static device array of the
library) against the workspace form of the same call, through the C ABI: two calls in a row, the
second on a smaller layer, bit for bit; and against the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
from workloads import inputs

pytestmark = pytest.mark.gpu


def _layer(B, G, n, c, hw, k, seed, residual):
    g = np.random.default_rng(seed)
    x = g.standard_normal((n, c, hw, hw)).astype(np.float16)
    w = (g.standard_normal((k, c, 3, 3)) * np.sqrt(2.0 / (9 * c))).astype(np.float16)
    scale = (1 + 0.1 * g.standard_normal(k)).astype(np.float32)
    shift = (0.1 * g.standard_normal(k)).astype(np.float32)
    res = g.standard_normal((n, k, hw, hw)).astype(np.float16) if residual else None
    flags = B.flags_of(None, scale, res, True)
    d = B.conv_desc(n, c, hw, hw, k, 3, 3, 1, 1, B.RELAY_F16, B.RELAY_NHWC, flags)
    xd = G.to_nhwc(x, c, B.RELAY_F16)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=G.DEV)
    B.relay_prepack_conv2d_weights(d, G.up(w), c, wp)
    rd = None if res is None else G.to_nhwc(res, k, B.RELAY_F16)
    return dict(d=d, x=x, w=w, scale=scale, shift=shift, res=res, xd=xd, wp=wp, rd=rd, sc=G.up(scale), sf=G.up(shift), n=n, k=k, hw=hw)


def test_static_scratch_conv_equals_the_workspace_form():
    from paper_1904_08368_amd import binding as B
    from tests import gpu_util as G
    B.lib()
    assert torch.cuda.is_available()
    # deep layers at batch 1: few output tiles, long reductions -> the library splits the reduction
    big = _layer(B, G, 1, 512, 7, 512, 901, True)
    small = _layer(B, G, 1, 384, 7, 256, 902, False)
    for L in (big, small, big):       # in a row, the second smaller than the first, then the first again
        need = B.relay_workspace_bytes(L["d"])
        assert 0 < need <= (4 << 20), need          # the layer really uses scratch, within the static array
        ws = torch.zeros(need, dtype=torch.uint8, device=G.DEV)
        y_ws = torch.full((L["n"], L["hw"], L["hw"], L["k"]), float("nan"), dtype=torch.float16, device=G.DEV)
        B.relay_fused_conv2d_bias_bn_relu(L["d"], L["xd"], L["wp"], None, L["sc"], L["sf"], L["rd"], y_ws, ws)
        y_st = torch.full_like(y_ws, float("nan"))
        B.relay_fused_conv2d_bias_bn_relu_static(L["d"], L["xd"], L["wp"], None, L["sc"], L["sf"], L["rd"], y_st)
        torch.cuda.synchronize()
        a, b = G.from_nhwc(y_st, L["k"]), G.from_nhwc(y_ws, L["k"])
        assert not np.isnan(a).any()
        assert np.array_equal(a, b)
        ref = O.fused_conv2d(L["x"], L["w"], stride=(1, 1), pad=(1, 1), scale=L["scale"], shift=L["shift"], residual=L["res"],
                             relu_flag=True, out_dtype="f16")
        assert O.max_rel_err(a, ref) <= 1e-2
    # a layer that needs no scratch goes through the same call
    plain = _layer(B, G, 2, 64, 20, 64, 903, False)
    assert B.relay_workspace_bytes(plain["d"]) == 0
    y1 = torch.full((2, 20, 20, 64), float("nan"), dtype=torch.float16, device=G.DEV)
    y2 = torch.full_like(y1, float("nan"))
    B.relay_fused_conv2d_bias_bn_relu_static(plain["d"], plain["xd"], plain["wp"], None, plain["sc"], plain["sf"], None, y1)
    B.relay_fused_conv2d_bias_bn_relu(plain["d"], plain["xd"], plain["wp"], None, plain["sc"], plain["sf"], None, y2)
    torch.cuda.synchronize()
    assert np.array_equal(y1.cpu().numpy(), y2.cpu().numpy())


def test_static_scratch_conv_rejects_what_does_not_fit():
    """Host-side: a forced split whose partial tiles exceed the static array is refused, nothing launched."""
    from paper_1904_08368_amd import binding as B
    B.lib()
    d = B.conv_desc(8, 512, 14, 14, 512, 3, 3, 1, 1, B.RELAY_F16, B.RELAY_NHWC, 0)
    B.relay_set_conv_split(36)
    try:
        assert B.relay_workspace_bytes(d) > (4 << 20)
        with pytest.raises(B.RelayError) as e:
            B.relay_fused_conv2d_bias_bn_relu_static(d, _Fake(0x7F0000001000), _Fake(0x7F0000101000), None, None, None, None,
                                                     _Fake(0x7F0000201000))
        assert e.value.status == 6
    finally:
        B.relay_set_conv_split(0)


class _Fake:
    def __init__(self, p):
        self.p = p

    def data_ptr(self):
        return self.p

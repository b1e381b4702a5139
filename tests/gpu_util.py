"""Helpers of the GPU parity tests: move numpy NCHW tensors to the device in the layout the
library wants, call one entry point through the binding, bring the result back as NCHW."""
from __future__ import annotations

import numpy as np
import torch

from paper_1904_08368_amd import binding as B

DEV = "cuda:0"


def up(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_nhwc(x_nchw: np.ndarray, cpad: int, dtype: int) -> torch.Tensor:
    n, c, h, w = x_nchw.shape
    src = up(x_nchw)
    dst = torch.empty((n, h, w, cpad), dtype=src.dtype, device=DEV)
    B.relay_nchw_to_nhwc(dtype, n, c, h, w, cpad, src, dst)
    return dst


def from_nhwc(t: torch.Tensor, c: int) -> np.ndarray:
    return t[..., :c].permute(0, 3, 1, 2).contiguous().cpu().numpy()


def round_up(a, b):
    return (a + b - 1) // b * b


def _input(x, k, r, s, stride, pad, dtype, ve, flags, nhwc4):
    """Descriptor and device input: plain (channel-padded) NHWC, or the pre-padded NHWC4 form
    for inputs of at most 4 channels."""
    n, c, h, wd = x.shape
    if nhwc4 and c <= 4:
        d = B.conv_desc(n, c, h, wd, k, r, s, stride, pad, dtype, B.RELAY_NHWC4_PADDED, flags)
        hp, wp = B.relay_nhwc4_padded_shape(d)
        xd = torch.full((n, hp, wp, 4), 7, dtype=torch.float16 if dtype == B.RELAY_F16 else torch.int8, device=DEV)
        B.relay_pack_input_nhwc4(d, up(x), xd)
        return d, xd
    cp = round_up(c, ve)
    d = B.conv_desc(n, cp, h, wd, k, r, s, stride, pad, dtype, B.RELAY_NHWC, flags)
    return d, to_nhwc(x, cp, dtype)


def workspace_for(d, split, state=None):
    """Zeroed workspace of the size the library asks for under a forced split (None if it asks for none).
    state: a dict that keeps one buffer across calls, to exercise reuse without clearing."""
    B.relay_set_conv_split(split)
    need = B.relay_workspace_bytes(d)
    if need == 0:
        return None
    if state is not None:
        if state.get("ws") is None or state["ws"].numel() < need:
            state["ws"] = torch.zeros(need, dtype=torch.uint8, device=DEV)
        return state["ws"]
    return torch.zeros(need, dtype=torch.uint8, device=DEV)


def run_conv_f16(x, w, stride, pad, bias=None, scale=None, shift=None, residual=None, relu=False, tile=-1,
                 nhwc4=True, split=None, ws_state=None):
    """x [N,C,H,W] fp16, w [K,C,R,S] fp16 (numpy) -> y NCHW fp16 (numpy), via the C ABI."""
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    flags = B.flags_of(bias, scale, residual, relu)
    d, xd = _input(x, k, r, s, stride, pad, B.RELAY_F16, 8, flags, nhwc4)
    ho, wo = B.relay_conv2d_out_shape(d)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=DEV)
    B.relay_prepack_conv2d_weights(d, up(w), c, wp)
    rd = None if residual is None else to_nhwc(residual, k, B.RELAY_F16)
    y = torch.full((n, ho, wo, k), float("nan"), dtype=torch.float16, device=DEV)
    B.relay_set_conv_tile(tile)
    try:
        ws = None if split is None else workspace_for(d, split, ws_state)
        B.relay_fused_conv2d_bias_bn_relu(d, xd, wp, up(bias), up(scale), up(shift), rd, y, ws)
    finally:
        B.relay_set_conv_tile(-1)
        B.relay_set_conv_split(0)
    torch.cuda.synchronize()
    return from_nhwc(y, k)


def run_qconv(x, w, stride, pad, bias=None, residual=None, lshift=0, rshift=0, relu=False, tile=-1, nhwc4=True,
              split=None, ws_state=None, round_mode=None, seed=0):
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    flags = B.flags_of(bias, None, residual, relu)
    d, xd = _input(x, k, r, s, stride, pad, B.RELAY_I8, 16, flags, nhwc4)
    ho, wo = B.relay_conv2d_out_shape(d)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=DEV)
    B.relay_prepack_conv2d_weights(d, up(w), c, wp)
    rd = None if residual is None else to_nhwc(residual, k, B.RELAY_I8)
    y = torch.full((n, ho, wo, k), -128, dtype=torch.int8, device=DEV)
    bd = None if bias is None else up(np.asarray(bias, dtype=np.int32))
    B.relay_set_conv_tile(tile)
    try:
        ws = None if split is None else workspace_for(d, split, ws_state)
        if round_mode is None:
            B.relay_qconv2d_requant(d, xd, wp, bd, rd, lshift, rshift, y, ws)
        else:
            B.relay_qconv2d_requant_rounding(d, xd, wp, bd, rd, lshift, rshift, round_mode, seed, y, ws)
    finally:
        B.relay_set_conv_tile(-1)
        B.relay_set_conv_split(0)
    torch.cuda.synchronize()
    return from_nhwc(y, k)


def run_dwconv_f16(x, w, stride, pad, bias=None, scale=None, shift=None, relu=False):
    n, c, h, wd = x.shape
    flags = B.flags_of(bias, scale, None, relu)
    d = B.conv_desc(n, c, h, wd, c, 3, 3, stride, pad, B.RELAY_F16, B.RELAY_NHWC, flags)
    ho, wo = B.relay_conv2d_out_shape(d)
    xd = to_nhwc(x, c, B.RELAY_F16)
    wp = torch.empty((9, c), dtype=torch.float16, device=DEV)
    B.relay_prepack_dwconv_weights(d, up(w), wp)
    y = torch.full((n, ho, wo, c), float("nan"), dtype=torch.float16, device=DEV)
    B.relay_fused_dwconv_bias_relu(d, xd, wp, up(bias), up(scale), up(shift), y)
    torch.cuda.synchronize()
    return from_nhwc(y, c)


def run_first_layer_f16(x, w, bias=None, scale=None, shift=None, relu=False):
    """The first-layer entry point: NCHW image in, NHWC out (returned as NCHW)."""
    n, c, h, wd = x.shape
    k = w.shape[0]
    d = B.conv_desc(n, c, h, wd, k, 3, 3, 2, 1, B.RELAY_F16, B.RELAY_NCHW, B.flags_of(bias, scale, None, relu))
    ho, wo = B.relay_conv2d_out_shape(d)
    y = torch.full((n, ho, wo, k), float("nan"), dtype=torch.float16, device=DEV)
    wp = torch.empty(B.relay_first_layer_packed_weight_bytes(d), dtype=torch.uint8, device=DEV)
    B.relay_prepack_first_layer_weights(d, up(w), wp)
    B.relay_fused_conv2d_first_layer(d, up(x), wp, up(bias), up(scale), up(shift), y)
    torch.cuda.synchronize()
    return from_nhwc(y, k)


def run_conv_pool_f16(x, w, stride, pad, bias=None, scale=None, shift=None, relu=False, nhwc4=True, fused=True):
    """conv -> 3x3/s2/p1 max pool, fp16: one pooled launch (fused) or the two separate calls."""
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    flags = B.flags_of(bias, scale, None, relu)
    d, xd = _input(x, k, r, s, stride, pad, B.RELAY_F16, 8, flags, nhwc4)
    ho, wo = B.relay_conv2d_out_shape(d)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=DEV)
    B.relay_prepack_conv2d_weights(d, up(w), c, wp)
    hp, wpo = (ho - 1) // 2 + 1, (wo - 1) // 2 + 1
    yp = torch.full((n, hp, wpo, k), float("nan"), dtype=torch.float16, device=DEV)
    if fused:
        B.relay_fused_conv2d_bn_relu_maxpool(d, xd, wp, up(bias), up(scale), up(shift), yp)
    else:
        y = torch.full((n, ho, wo, k), float("nan"), dtype=torch.float16, device=DEV)
        B.relay_fused_conv2d_bias_bn_relu(d, xd, wp, up(bias), up(scale), up(shift), None, y)
        B.relay_maxpool2d(B.RELAY_F16, n, k, ho, wo, 3, 2, 1, y, yp)
    torch.cuda.synchronize()
    return from_nhwc(yp, k)


def run_qconv_pool(x, w, stride, pad, bias=None, rshift=0, relu=False, nhwc4=True, fused=True):
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    flags = B.flags_of(bias, None, None, relu)
    d, xd = _input(x, k, r, s, stride, pad, B.RELAY_I8, 16, flags, nhwc4)
    ho, wo = B.relay_conv2d_out_shape(d)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=DEV)
    B.relay_prepack_conv2d_weights(d, up(w), c, wp)
    hp, wpo = (ho - 1) // 2 + 1, (wo - 1) // 2 + 1
    yp = torch.full((n, hp, wpo, k), -128, dtype=torch.int8, device=DEV)
    bd = None if bias is None else up(np.asarray(bias, dtype=np.int32))
    if fused:
        B.relay_qconv2d_requant_maxpool(d, xd, wp, bd, rshift, yp)
    else:
        y = torch.full((n, ho, wo, k), -128, dtype=torch.int8, device=DEV)
        B.relay_qconv2d_requant(d, xd, wp, bd, None, 0, rshift, y)
        B.relay_maxpool2d(B.RELAY_I8, n, k, ho, wo, 3, 2, 1, y, yp)
    torch.cuda.synchronize()
    return from_nhwc(yp, k)

"""ctypes binding of librelayfused.so: argument marshalling only.

Each function has the name of the C entry point it calls (include/relay_fused.h) and
takes torch tensors on the GPU purely as (pointer, shape) carriers; PyTorch supplies device
memory and the stream, every step of the computation runs in the library's own kernels.
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librelayfused.so")

RELAY_F32, RELAY_F16, RELAY_I8, RELAY_I16 = 0, 1, 2, 3
RELAY_NCHW, RELAY_NHWC, RELAY_NHWC4_PADDED = 0, 1, 2
HAS_BIAS, HAS_BN, HAS_RESIDUAL, RELU = 1, 2, 4, 8

STATUS_NAMES = {0: "RELAY_OK", 1: "RELAY_ERR_NULL", 2: "RELAY_ERR_SHAPE", 3: "RELAY_ERR_DTYPE",
                4: "RELAY_ERR_UNSUPPORTED", 5: "RELAY_ERR_ALIGN", 6: "RELAY_ERR_WORKSPACE",
                7: "RELAY_ERR_DEVICE"}


class RelayError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w",
                                         "pad_h", "pad_w", "dtype", "layout")] + [("flags", C.c_uint32)]


_lib = None

# name -> argtypes; every symbol the header declares
_P, _I, _SZ = C.c_void_p, C.c_int32, C.c_size_t
_DP = C.POINTER(ConvDesc)
SIGNATURES = {
    "relay_conv2d_out_shape": [_DP, C.POINTER(_I), C.POINTER(_I)],
    "relay_workspace_bytes": [_DP, C.POINTER(_SZ)],
    "relay_packed_weight_bytes": [_DP, C.POINTER(_SZ)],
    "relay_prepack_conv2d_weights": [_DP, _P, _I, _P, _SZ, _P],
    "relay_fused_conv2d_bias_bn_relu": [_DP, _P, _P, _P, _P, _P, _P, _P, _P, _SZ, _P],
    "relay_fused_conv2d_bias_bn_relu_static": [_DP, _P, _P, _P, _P, _P, _P, _P, _P],
    "relay_qconv2d_requant": [_DP, _P, _P, _P, _P, _I, _I, _P, _P, _SZ, _P],
    "relay_qconv2d_requant_scaled": [_DP, _P, _P, _P, _P, _I, _P, _P, _P, _P, _SZ, _P],
    "relay_quantize_multiplier": [C.c_double, C.POINTER(_I), C.POINTER(_I)],
    "relay_qconv2d_requant_acc16": [_DP, _P, _P, _P, _P, _I, _I, _P, _P, _SZ, _P],
    "relay_qconv2d_requant_i16": [_DP, _P, _P, _P, _I, _P, _P],
    "relay_qconv2d_u8_workspace_bytes": [_DP, C.POINTER(_SZ)],
    "relay_fold_zero_point": [_I, C.c_int64, _P, _P, _I, _P, _P],
    "relay_qconv2d_requant_u8": [_DP, _P, _P, _P, _I, _I, _P, _P, _SZ, _P],
    "relay_prepack_dwconv_weights": [_DP, _P, _P, _P],
    "relay_fused_dwconv_bias_relu": [_DP, _P, _P, _P, _P, _P, _P, _P],
    "relay_fused_conv2d_first_layer": [_DP, _P, _P, _P, _P, _P, _P, _P],
    "relay_conv2d_first_layer_supported": [_DP, C.POINTER(C.c_int32)],
    "relay_first_layer_packed_weight_bytes": [_DP, C.POINTER(C.c_size_t)],
    "relay_prepack_first_layer_weights": [_DP, _P, _P, _P],
    "relay_dwconv_pwconv_fusion_pays": [_DP, C.c_int32, C.POINTER(C.c_int32)],
    "relay_fused_dwconv_pwconv": [_DP, _P, _P, _P, _P, _P, C.c_int32, C.c_uint32, _P, _P, _P, _P, _P, _P],
    "relay_fused_dense_bias_act": [_I, _I, _I, _I, _P, _P, _P, _I, _P, _P],
    "relay_maxpool2d": [_I, _I, _I, _I, _I, _I, _I, _I, _P, _P, _P],
    "relay_global_avgpool": [_I, _I, _I, _I, _P, _P, _P],
    "relay_nchw_to_nhwc": [_I, _I, _I, _I, _I, _I, _P, _P, _P],
    "relay_nhwc4_padded_shape": [_DP, C.POINTER(_I), C.POINTER(_I)],
    "relay_pack_input_nhwc4": [_DP, _P, _P, _P],
    "relay_elementwise_f16": [_I, C.c_int64, _I, _P, _P, _P, _P, _P, _P],
    "relay_fuse_extract": [_I, _P, _P, _P, _P, _P],
    "relay_qconv2d_requant_rounding": [_DP, _P, _P, _P, _P, _I, _I, _I, C.c_uint64, _P, _P, _SZ, _P],
    "relay_quantize": [C.c_int64, _I, _P, C.c_float, _I, _I, _I, C.c_uint64, _P, _P],
    "relay_sim_quantize": [C.c_int64, _P, C.c_float, _I, _I, _I, C.c_uint64, _P, _P],
    "relay_fused_conv2d_combined": [_DP, _P, _I, _P, _P, _P, _P, _I, _P, _P, _P, _P],
    "relay_fused_conv2d_combined_windows": [_DP, _P, _I, _P, _P, _P, _P, _I, _P, _P, _P, _P, _P, _P],
    "relay_qconv2d_combined": [_DP, _P, _I, _P, _P, _P, _P, _I, _I, _P, _P, _P, _P],
    "relay_fold_scale_axis": [_I, _I, _I, _I, _I, _P, _P, _P, _P],
    "relay_fold_bias": [_I, _P, _P, _P, _P, _P],
    "relay_conv2d_maxpool_fusable": [_DP, C.POINTER(_I)],
    "relay_conv2d_maxpool_kernel_name": [_DP, C.c_char_p, _SZ],
    "relay_fused_conv2d_bn_relu_maxpool": [_DP, _P, _P, _P, _P, _P, _P, _P],
    "relay_qconv2d_requant_maxpool": [_DP, _P, _P, _P, _I, _P, _P],
    "relay_calibrate_pow2_range": [_I, C.c_int64, _P, _P, _P, _P],
    "relay_realize_conv": [_I, C.c_int64, _P, _P, _P, _P, C.c_float, C.c_float, C.c_float, _P, _P, _P, _P, _SZ, _P],
    "relay_probe_mfma": [_I, _I, _I, _P, _P],
    "relay_probe_copy": [_P, _P, C.c_int64, _P],
    "relay_probe_grid_barrier": [_I, _I, C.c_uint32, _P, _P, _P],
    "relay_set_conv_tile": [_I],
    "relay_set_conv_split": [_I],
    "relay_set_conv_workgroups": [_I],
    "relay_conv2d_kernel_name": [_DP, C.c_char_p, _SZ],
    "relay_dwconv_pwconv_kernel_name": [_DP, C.c_int32, C.c_char_p, _SZ],
}


def lib():
    """Load the library (built in-tree by build.py); fail loudly if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        l = C.CDLL(LIB_PATH)
        for name, argtypes in SIGNATURES.items():
            fn = getattr(l, name)
            fn.argtypes = argtypes
            fn.restype = C.c_int
        l.relay_last_error.restype = C.c_char_p
        l.relay_last_error.argtypes = []
        _lib = l
    return _lib


def _check(status: int) -> None:
    if status != 0:
        raise RelayError(status, lib().relay_last_error().decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> Optional[int]:
    import torch
    return torch.cuda.current_stream().cuda_stream or None


def conv_desc(n, c, h, w, k, r, s, stride, pad, dtype, layout, flags) -> ConvDesc:
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return ConvDesc(n, c, h, w, k, r, s, sh, sw, ph, pw, dtype, layout, flags)


def flags_of(bias=None, bn_scale=None, residual=None, relu=False) -> int:
    return ((HAS_BIAS if bias is not None else 0) | (HAS_BN if bn_scale is not None else 0) |
            (HAS_RESIDUAL if residual is not None else 0) | (RELU if relu else 0))


# --------------------------------------------------------------------------- entry points
def relay_conv2d_out_shape(d: ConvDesc) -> Tuple[int, int]:
    ho, wo = _I(), _I()
    _check(lib().relay_conv2d_out_shape(C.byref(d), C.byref(ho), C.byref(wo)))
    return ho.value, wo.value


def relay_workspace_bytes(d: ConvDesc) -> int:
    b = _SZ()
    _check(lib().relay_workspace_bytes(C.byref(d), C.byref(b)))
    return b.value


def relay_packed_weight_bytes(d: ConvDesc) -> int:
    b = _SZ()
    _check(lib().relay_packed_weight_bytes(C.byref(d), C.byref(b)))
    return b.value


def relay_prepack_conv2d_weights(d: ConvDesc, w_oihw, c_src: int, w_packed) -> None:
    _check(lib().relay_prepack_conv2d_weights(C.byref(d), _ptr(w_oihw), c_src, _ptr(w_packed),
                                              w_packed.numel() * w_packed.element_size(), _stream()))


def relay_fused_conv2d_bias_bn_relu(d: ConvDesc, x, w_packed, bias, bn_scale, bn_shift, residual, y,
                                    workspace=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().relay_fused_conv2d_bias_bn_relu(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(bn_scale),
                                                 _ptr(bn_shift), _ptr(residual), _ptr(y), _ptr(workspace),
                                                 ws_bytes, _stream()))


def relay_fused_conv2d_bias_bn_relu_static(d: ConvDesc, x, w_packed, bias, bn_scale, bn_shift, residual, y) -> None:
    _check(lib().relay_fused_conv2d_bias_bn_relu_static(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(bn_scale),
                                                        _ptr(bn_shift), _ptr(residual), _ptr(y), _stream()))


def relay_qconv2d_requant(d: ConvDesc, x, w_packed, bias, residual, residual_lshift: int, out_rshift: int, y,
                          workspace=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().relay_qconv2d_requant(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(residual),
                                       residual_lshift, out_rshift, _ptr(y), _ptr(workspace), ws_bytes, _stream()))


def relay_conv2d_maxpool_fusable(d: ConvDesc) -> bool:
    out = C.c_int32(0)
    _check(lib().relay_conv2d_maxpool_fusable(C.byref(d), C.byref(out)))
    return bool(out.value)


def relay_fused_conv2d_bn_relu_maxpool(d: ConvDesc, x, w_packed, bias, bn_scale, bn_shift, y_pooled) -> None:
    _check(lib().relay_fused_conv2d_bn_relu_maxpool(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(bn_scale),
                                                    _ptr(bn_shift), _ptr(y_pooled), _stream()))


def relay_qconv2d_requant_maxpool(d: ConvDesc, x, w_packed, bias, out_rshift: int, y_pooled) -> None:
    _check(lib().relay_qconv2d_requant_maxpool(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias), out_rshift,
                                               _ptr(y_pooled), _stream()))


def relay_prepack_dwconv_weights(d: ConvDesc, w_crs, w_rsc) -> None:
    _check(lib().relay_prepack_dwconv_weights(C.byref(d), _ptr(w_crs), _ptr(w_rsc), _stream()))


def relay_fused_dwconv_bias_relu(d: ConvDesc, x, w_rsc, bias, bn_scale, bn_shift, y) -> None:
    _check(lib().relay_fused_dwconv_bias_relu(C.byref(d), _ptr(x), _ptr(w_rsc), _ptr(bias), _ptr(bn_scale),
                                              _ptr(bn_shift), _ptr(y), _stream()))


def relay_conv2d_first_layer_supported(d: ConvDesc) -> bool:
    ok = C.c_int32(0)
    _check(lib().relay_conv2d_first_layer_supported(C.byref(d), C.byref(ok)))
    return bool(ok.value)


def relay_first_layer_packed_weight_bytes(d: ConvDesc) -> int:
    n = C.c_size_t(0)
    _check(lib().relay_first_layer_packed_weight_bytes(C.byref(d), C.byref(n)))
    return n.value


def relay_prepack_first_layer_weights(d: ConvDesc, w_oihw, w_packed) -> None:
    _check(lib().relay_prepack_first_layer_weights(C.byref(d), _ptr(w_oihw), _ptr(w_packed), _stream()))


def relay_fused_conv2d_first_layer(d: ConvDesc, x_nchw, w_packed, bias, bn_scale, bn_shift, y_nhwc) -> None:
    _check(lib().relay_fused_conv2d_first_layer(C.byref(d), _ptr(x_nchw), _ptr(w_packed), _ptr(bias), _ptr(bn_scale),
                                                _ptr(bn_shift), _ptr(y_nhwc), _stream()))


def relay_dwconv_pwconv_fusion_pays(dw: ConvDesc, k: int) -> bool:
    pays = C.c_int32(0)
    _check(lib().relay_dwconv_pwconv_fusion_pays(C.byref(dw), k, C.byref(pays)))
    return bool(pays.value)


def relay_fused_dwconv_pwconv(dw: ConvDesc, x, dw_w_rsc, dw_bias, dw_scale, dw_shift, k: int, pw_flags: int, pw_w_packed,
                              pw_bias, pw_scale, pw_shift, y) -> None:
    _check(lib().relay_fused_dwconv_pwconv(C.byref(dw), _ptr(x), _ptr(dw_w_rsc), _ptr(dw_bias), _ptr(dw_scale), _ptr(dw_shift),
                                           k, pw_flags, _ptr(pw_w_packed), _ptr(pw_bias), _ptr(pw_scale), _ptr(pw_shift),
                                           _ptr(y), _stream()))


def relay_fused_dense_bias_act(m: int, n: int, k: int, dtype: int, x, w, bias, act: int, y) -> None:
    _check(lib().relay_fused_dense_bias_act(m, n, k, dtype, _ptr(x), _ptr(w), _ptr(bias), act, _ptr(y), _stream()))


def relay_maxpool2d(dtype, n, c, h, w, r, stride, pad, x, y) -> None:
    _check(lib().relay_maxpool2d(dtype, n, c, h, w, r, stride, pad, _ptr(x), _ptr(y), _stream()))


def relay_global_avgpool(dtype, n, c, hw, x, y) -> None:
    _check(lib().relay_global_avgpool(dtype, n, c, hw, _ptr(x), _ptr(y), _stream()))


def relay_nchw_to_nhwc(dtype, n, c, h, w, c_pad, x, y) -> None:
    _check(lib().relay_nchw_to_nhwc(dtype, n, c, h, w, c_pad, _ptr(x), _ptr(y), _stream()))


def relay_nhwc4_padded_shape(d: ConvDesc) -> Tuple[int, int]:
    hp, wp = _I(), _I()
    _check(lib().relay_nhwc4_padded_shape(C.byref(d), C.byref(hp), C.byref(wp)))
    return hp.value, wp.value


def relay_pack_input_nhwc4(d: ConvDesc, x_nchw, y) -> None:
    _check(lib().relay_pack_input_nhwc4(C.byref(d), _ptr(x_nchw), _ptr(y), _stream()))


ROUND_NEAREST, ROUND_FLOOR, ROUND_CEIL, ROUND_STOCHASTIC = 0, 1, 2, 3
EW_BIAS_ADD, EW_SCALE_SHIFT, EW_ADD, EW_RELU = 0, 1, 2, 3


def relay_elementwise_f16(op: int, n_pixels: int, c: int, x, p0, p1, other, y) -> None:
    _check(lib().relay_elementwise_f16(op, n_pixels, c, _ptr(x), _ptr(p0), _ptr(p1), _ptr(other), _ptr(y), _stream()))



def relay_qconv2d_requant_rounding(d: ConvDesc, x, w_packed, bias, residual, residual_lshift: int, out_rshift: int,
                                   round_mode: int, seed: int, y, workspace=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().relay_qconv2d_requant_rounding(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(residual),
                                                residual_lshift, out_rshift, round_mode, seed, _ptr(y), _ptr(workspace),
                                                ws_bytes, _stream()))


def relay_qconv2d_requant_scaled(d: ConvDesc, x, w_packed, bias, residual, residual_lshift: int, mult, rshift, y,
                                 workspace=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().relay_qconv2d_requant_scaled(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(residual), residual_lshift,
                                              _ptr(mult), _ptr(rshift), _ptr(y), _ptr(workspace), ws_bytes, _stream()))


def relay_quantize_multiplier(scale: float) -> Tuple[int, int]:
    m, s = _I(), _I()
    _check(lib().relay_quantize_multiplier(scale, C.byref(m), C.byref(s)))
    return m.value, s.value


def relay_qconv2d_requant_acc16(d: ConvDesc, x, w_packed, bias, residual, residual_lshift: int, out_rshift: int, y,
                                workspace=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().relay_qconv2d_requant_acc16(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(residual), residual_lshift,
                                             out_rshift, _ptr(y), _ptr(workspace), ws_bytes, _stream()))


def relay_qconv2d_requant_i16(d: ConvDesc, x, w_packed, bias, out_rshift: int, y) -> None:
    _check(lib().relay_qconv2d_requant_i16(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias), out_rshift, _ptr(y), _stream()))


def relay_qconv2d_u8_workspace_bytes(d: ConvDesc) -> int:
    b = _SZ()
    _check(lib().relay_qconv2d_u8_workspace_bytes(C.byref(d), C.byref(b)))
    return b.value


def relay_fold_zero_point(k: int, per_k: int, w, bias, zero_point: int, out) -> None:
    _check(lib().relay_fold_zero_point(k, per_k, _ptr(w), _ptr(bias), zero_point, _ptr(out), _stream()))


def relay_qconv2d_requant_u8(d: ConvDesc, x, w_packed, bias_zp, out_rshift: int, out_unsigned: bool, y, workspace) -> None:
    _check(lib().relay_qconv2d_requant_u8(C.byref(d), _ptr(x), _ptr(w_packed), _ptr(bias_zp), out_rshift, 1 if out_unsigned else 0,
                                          _ptr(y), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def relay_quantize(n_elems: int, src_dtype: int, x, rho: float, beta: int, sigma: int, round_mode: int, seed: int, y) -> None:
    _check(lib().relay_quantize(n_elems, src_dtype, _ptr(x), rho, beta, sigma, round_mode, seed, _ptr(y), _stream()))


def relay_sim_quantize(n_elems: int, x, rho: float, beta: int, sigma: int, round_mode: int, seed: int, y) -> None:
    _check(lib().relay_sim_quantize(n_elems, _ptr(x), rho, beta, sigma, round_mode, seed, _ptr(y), _stream()))


REALIZE_BAD_OUT_SHIFT, REALIZE_BAD_RES_SHIFT, REALIZE_BIAS_OVERFLOW = 1, 2, 4


def relay_calibrate_pow2_range(dtype: int, n_elems: int, x, rho_out, cell) -> None:
    """rho_out: device float32[1]; cell: device scratch of 4 bytes."""
    _check(lib().relay_calibrate_pow2_range(dtype, n_elems, _ptr(x), _ptr(rho_out), _ptr(cell), _stream()))


def relay_realize_conv(k: int, per_k: int, w, bias, scale, shift, rho_x: float, rho_y: float, rho_res: float, wq,
                       bias_q, out, workspace) -> None:
    """out: device int32[4] that receives (rho_w as float bits, out_rshift, residual_lshift, status)."""
    _check(lib().relay_realize_conv(k, per_k, _ptr(w), _ptr(bias), _ptr(scale), _ptr(shift), rho_x, rho_y, rho_res,
                                    _ptr(wq), _ptr(bias_q), _ptr(out), _ptr(workspace),
                                    0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


FOLD_OUT, FOLD_IN = 0, 1


def relay_fused_conv2d_combined(d: ConvDesc, x, x_ld: int, w_packed, bias, bn_scale, bn_shift,
                                seg_channels: Sequence[int], seg_y: Sequence, seg_ld: Sequence[int]) -> None:
    """seg_y: one tensor per segment whose data_ptr() is channel 0 of pixel 0 of that segment
    (a channel slice of a wider NHWC tensor is fine: its data_ptr() already carries the offset)."""
    n = len(seg_y)
    ch = (C.c_int32 * max(n, 1))(*seg_channels)
    ld = (C.c_int32 * max(n, 1))(*seg_ld)
    ys = (C.c_void_p * max(n, 1))(*[_ptr(t) for t in seg_y])
    _check(lib().relay_fused_conv2d_combined(C.byref(d), _ptr(x), x_ld, _ptr(w_packed), _ptr(bias), _ptr(bn_scale),
                                             _ptr(bn_shift), n, C.cast(ch, _P), C.cast(ys, _P), C.cast(ld, _P),
                                             _stream()))


WINDOW_FULL, WINDOW_CENTRE = 0, 1


def relay_qconv2d_combined(d: ConvDesc, x, x_ld: int, w_packed, bias, mult, rshift, out_rshift: int,
                           seg_channels: Sequence[int], seg_y: Sequence, seg_ld: Sequence[int]) -> None:
    n = len(seg_y)
    ch = (C.c_int32 * max(n, 1))(*seg_channels)
    ld = (C.c_int32 * max(n, 1))(*seg_ld)
    ys = (C.c_void_p * max(n, 1))(*[_ptr(t) for t in seg_y])
    _check(lib().relay_qconv2d_combined(C.byref(d), _ptr(x), x_ld, _ptr(w_packed), _ptr(bias), _ptr(mult), _ptr(rshift), out_rshift,
                                        n, C.cast(ch, _P), C.cast(ys, _P), C.cast(ld, _P), _stream()))


def relay_fused_conv2d_combined_windows(d: ConvDesc, x, x_ld: int, w_packed, bias, bn_scale, bn_shift,
                                        seg_channels: Sequence[int], seg_y: Sequence, seg_ld: Sequence[int],
                                        seg_window: Sequence[int], seg_relu: Sequence[int]) -> None:
    n = len(seg_y)
    arr = lambda v: (C.c_int32 * max(n, len(v), 1))(*v)
    ch, ld, win, rl = arr(seg_channels), arr(seg_ld), arr(seg_window), arr(seg_relu)
    ys = (C.c_void_p * max(n, 1))(*[_ptr(t) for t in seg_y])
    _check(lib().relay_fused_conv2d_combined_windows(C.byref(d), _ptr(x), x_ld, _ptr(w_packed), _ptr(bias),
                                                     _ptr(bn_scale), _ptr(bn_shift), n, C.cast(ch, _P), C.cast(ys, _P),
                                                     C.cast(ld, _P), C.cast(win, _P), C.cast(rl, _P), _stream()))


def relay_fold_scale_axis(dtype: int, k: int, c: int, rs: int, axis: int, w, scale, w_out) -> None:
    _check(lib().relay_fold_scale_axis(dtype, k, c, rs, axis, _ptr(w), _ptr(scale), _ptr(w_out), _stream()))


def relay_fold_bias(k: int, bias, scale, shift, out) -> None:
    _check(lib().relay_fold_bias(k, _ptr(bias), _ptr(scale), _ptr(shift), _ptr(out), _stream()))


def relay_fuse_extract(pattern: Sequence[int], in_offsets: Sequence[int], in_nodes: Sequence[int]):
    """Host-side call: returns (ipdom, group) as lists, one entry per operator."""
    n = len(pattern)
    arr = lambda v: (C.c_int32 * max(len(v), 1))(*v)
    pat, offs, ins = arr(pattern), arr(in_offsets), arr(in_nodes)
    ipdom, group = (C.c_int32 * n)(), (C.c_int32 * n)()
    _check(lib().relay_fuse_extract(n, C.cast(pat, _P), C.cast(offs, _P), C.cast(ins, _P) if len(in_nodes) else None,
                                    C.cast(ipdom, _P), C.cast(group, _P)))
    return list(ipdom), list(group)


def relay_conv2d_kernel_name(d: ConvDesc) -> str:
    buf = C.create_string_buffer(128)
    _check(lib().relay_conv2d_kernel_name(C.byref(d), buf, 128))
    return buf.value.decode()


def relay_dwconv_pwconv_kernel_name(dw: ConvDesc, k: int) -> str:
    buf = C.create_string_buffer(160)
    _check(lib().relay_dwconv_pwconv_kernel_name(C.byref(dw), k, buf, 160))
    return buf.value.decode()


def relay_conv2d_maxpool_kernel_name(d: ConvDesc) -> str:
    buf = C.create_string_buffer(128)
    _check(lib().relay_conv2d_maxpool_kernel_name(C.byref(d), buf, 128))
    return buf.value.decode()


def relay_probe_mfma(dtype: int, iters: int, workgroups: int, out) -> None:
    _check(lib().relay_probe_mfma(dtype, iters, workgroups, _ptr(out), _stream()))


def relay_probe_grid_barrier(workgroups: int, rounds: int, spin_limit: int, cells, data=None) -> None:
    _check(lib().relay_probe_grid_barrier(workgroups, rounds, spin_limit, _ptr(cells), _ptr(data), _stream()))


def relay_probe_copy(src, dst, nbytes: int) -> None:
    _check(lib().relay_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream()))


def relay_set_conv_tile(tile: int) -> None:
    _check(lib().relay_set_conv_tile(tile))


def relay_set_conv_workgroups(workgroups: int) -> None:
    _check(lib().relay_set_conv_workgroups(workgroups))


def relay_set_conv_split(split: int) -> None:
    _check(lib().relay_set_conv_split(split))

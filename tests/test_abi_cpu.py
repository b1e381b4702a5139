"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and
rejects bad arguments on the host before any HIP call (no compute call is made here: every
case below must fail validation, so nothing is ever launched)."""
import ctypes as C
import os
import re

import pytest

from paper_1904_08368_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000            # a non-NULL, 4096-byte aligned address that is never dereferenced


def _header_symbols():
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include")))
                   if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(relay_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _header_symbols()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/*.h but not exported"
    # and the binding wraps each of them under the same name
    for n in names:
        if n != "relay_last_error":
            assert hasattr(B, n), f"binding has no {n}"


def _d(**kw):
    base = dict(n=1, c=64, h=8, w=8, k=64, r=3, s=3, stride=1, pad=1, dtype=B.RELAY_F16, layout=B.RELAY_NHWC, flags=0)
    base.update(kw)
    return B.conv_desc(base["n"], base["c"], base["h"], base["w"], base["k"], base["r"], base["s"], base["stride"],
                       base["pad"], base["dtype"], base["layout"], base["flags"])


def _status(fn, *args):
    lib = B.lib()
    return getattr(lib, fn)(*args)


def test_out_shape_formula_exhaustive():
    for h in range(1, 12):
        for r in (1, 2, 3, 5, 7):
            for st in (1, 2, 3):
                for pd in range(0, r):
                    if h + 2 * pd < r:
                        with pytest.raises(B.RelayError) as e:
                            B.relay_conv2d_out_shape(_d(h=h, w=h, r=r, s=r, stride=st, pad=pd))
                        assert e.value.status == 2
                        continue
                    ho, wo = B.relay_conv2d_out_shape(_d(h=h, w=h + 3, r=r, s=r, stride=st, pad=pd))
                    assert ho == (h + 2 * pd - r) // st + 1 and wo == (h + 3 + 2 * pd - r) // st + 1


@pytest.mark.parametrize("kw,status", [
    (dict(n=0), 2), (dict(c=-1), 2), (dict(k=0), 2), (dict(stride=0), 2), (dict(pad=3), 2), (dict(pad=-1), 2),
    (dict(h=1, w=1, pad=0), 2), (dict(dtype=9), 3), (dict(layout=7), 4), (dict(flags=64), 4),
    (dict(n=40000, c=512, h=512, w=512), 2),
])
def test_geometry_is_validated(kw, status):
    with pytest.raises(B.RelayError) as e:
        B.relay_conv2d_out_shape(_d(**kw))
    assert e.value.status == status
    assert B.lib().relay_last_error()           # a message is left behind


def test_null_descriptor_and_outputs():
    i = C.c_int32()
    assert _status("relay_conv2d_out_shape", None, C.byref(i), C.byref(i)) == 1
    assert _status("relay_conv2d_out_shape", C.byref(_d()), None, C.byref(i)) == 1
    assert _status("relay_workspace_bytes", C.byref(_d()), None) == 1
    # a layer with many output tiles, or a short reduction, keeps its sums in registers; a deep layer at
    # batch 1 is split along its reduction: 36 chunks over 6 workgroups for each of the 8 tiles of 64 x 64,
    # behind one 256-byte counter line per tile
    assert B.relay_workspace_bytes(_d(n=32, h=56, w=56)) == 0
    assert B.relay_workspace_bytes(_d()) == 0
    deep = _d(c=512, k=512, h=7, w=7)
    assert B.relay_workspace_bytes(deep) == 8 * 256 + 8 * 6 * 64 * 64 * 4
    B.relay_set_conv_split(1)
    try:
        assert B.relay_workspace_bytes(deep) == 0
    finally:
        B.relay_set_conv_split(0)
    B.relay_set_conv_split(3)
    try:
        assert B.relay_workspace_bytes(_d()) == 256 + 3 * 64 * 64 * 4
    finally:
        B.relay_set_conv_split(0)
    with pytest.raises(B.RelayError):
        B.relay_set_conv_split(65)


def test_workspace_is_checked_before_any_launch():
    B.relay_set_conv_split(3)
    try:
        _workspace_checks()
    finally:
        B.relay_set_conv_split(0)


def _workspace_checks():
    need = B.relay_workspace_bytes(_d())
    assert need > 0
    ws = FAKE + (1 << 20)
    assert _status("relay_fused_conv2d_bias_bn_relu", C.byref(_d()), FAKE, FAKE, None, None, None, None, FAKE + 4096,
                   ws + 16, need, None) == 5                                   # not 256-byte aligned
    assert _status("relay_fused_conv2d_bias_bn_relu", C.byref(_d()), FAKE, FAKE, None, None, None, None, FAKE + 4096,
                   ws, need - 1, None) == 6                                    # too small
    assert _status("relay_qconv2d_requant", C.byref(_d(dtype=B.RELAY_I8)), FAKE, FAKE, None, None, 0, 8, FAKE + 4096,
                   ws, 16, None) == 6


def test_packed_weight_bytes_and_channel_alignment():
    assert B.relay_packed_weight_bytes(_d()) == 64 * 576 * 2                 # 576 is a whole number of 128-byte groups
    assert B.relay_packed_weight_bytes(_d(c=8)) == 64 * 128 * 2             # 72 halves -> 128 (two 128-byte groups)
    assert B.relay_packed_weight_bytes(_d(dtype=B.RELAY_I8, c=16)) == 64 * 256
    assert B.relay_packed_weight_bytes(_d(dtype=B.RELAY_F32, layout=B.RELAY_NCHW, c=3)) == 64 * 27 * 4
    assert B.relay_packed_weight_bytes(_d(c=3, r=7, s=7, pad=3, layout=B.RELAY_NHWC4_PADDED)) == 64 * 256 * 2
    for kw, status in [(dict(c=3), 5), (dict(dtype=B.RELAY_I8, c=8), 5), (dict(layout=B.RELAY_NCHW), 4),
                       (dict(dtype=B.RELAY_F32), 4), (dict(c=5, layout=B.RELAY_NHWC4_PADDED), 2),
                       (dict(c=3, r=9, s=9, pad=4, layout=B.RELAY_NHWC4_PADDED), 4)]:
        with pytest.raises(B.RelayError) as e:
            B.relay_packed_weight_bytes(_d(**kw))
        assert e.value.status == status, kw
    hp, wp = B.relay_nhwc4_padded_shape(_d(c=3, h=224, w=224, r=7, s=7, pad=3, stride=2, layout=B.RELAY_NHWC4_PADDED))
    assert (hp, wp) == (230, 232)


def _conv(d, x=FAKE, w=FAKE, bias=None, sc=None, sf=None, res=None, y=FAKE + 4096):
    return _status("relay_fused_conv2d_bias_bn_relu", C.byref(d), x, w, bias, sc, sf, res, y, None, 0, None)


def test_conv_argument_checks_fail_before_any_launch():
    assert _conv(_d(), x=None) == 1
    assert _conv(_d(), y=None) == 1
    assert _conv(_d(flags=B.HAS_BIAS)) == 1                       # flag set, pointer NULL
    assert _conv(_d(), bias=FAKE) == 1                            # pointer given, flag clear
    assert _conv(_d(flags=B.HAS_BN), sc=FAKE) == 1                # shift missing
    assert _conv(_d(flags=B.HAS_RESIDUAL)) == 1
    assert _conv(_d(dtype=B.RELAY_I8)) == 3                       # int8 has its own entry point
    assert _conv(_d(), y=FAKE) == 4                               # output aliases input
    assert _conv(_d(), x=FAKE + 2) == 5                           # misaligned
    assert _conv(_d(c=12)) == 5
    assert _conv(_d(layout=B.RELAY_NCHW)) == 4
    assert _conv(_d(dtype=B.RELAY_F32, layout=B.RELAY_NHWC)) == 4
    assert b"" != B.lib().relay_last_error()


def _q(d, x=FAKE, w=FAKE, bias=None, res=None, l=0, s=8, y=FAKE + 4096):
    return _status("relay_qconv2d_requant", C.byref(d), x, w, bias, res, l, s, y, None, 0, None)


def test_qconv_argument_checks():
    q = dict(dtype=B.RELAY_I8)
    assert _q(_d()) == 3                                          # not an int8 descriptor
    assert _q(_d(**q), s=-1) == 4 and _q(_d(**q), s=32) == 4
    assert _q(_d(**q), l=-1) == 4 and _q(_d(**q), l=24) == 4
    assert _q(_d(flags=B.HAS_BN, **q)) == 4
    assert _q(_d(flags=B.HAS_RESIDUAL, **q)) == 1
    assert _q(_d(**q), res=FAKE) == 1
    assert _q(_d(c=24, **q)) == 5
    assert _q(_d(**q), y=FAKE + 4) == 5
    assert _q(_d(**q), x=None) == 1


def test_dwconv_dense_and_glue_checks():
    dw = _status
    d = _d(c=32, k=32)
    assert dw("relay_fused_dwconv_bias_relu", C.byref(d), None, FAKE, None, None, None, FAKE + 4096, None) == 1
    assert dw("relay_fused_dwconv_bias_relu", C.byref(_d(c=32, k=64)), FAKE, FAKE, None, None, None, FAKE + 4096, None) == 2
    assert dw("relay_fused_dwconv_bias_relu", C.byref(_d(c=36, k=36)), FAKE, FAKE, None, None, None, FAKE + 4096, None) == 5
    assert dw("relay_fused_dwconv_bias_relu", C.byref(_d(c=32, k=32, r=5, s=5, pad=2)), FAKE, FAKE, None, None, None, FAKE + 4096, None) == 4
    assert dw("relay_fused_dwconv_bias_relu", C.byref(_d(c=32, k=32, stride=3)), FAKE, FAKE, None, None, None, FAKE + 4096, None) == 4
    assert dw("relay_fused_dwconv_bias_relu", C.byref(_d(c=32, k=32, dtype=B.RELAY_I8)), FAKE, FAKE, None, None, None, FAKE + 4096, None) == 3
    assert dw("relay_prepack_dwconv_weights", C.byref(d), None, FAKE, None) == 1
    de = "relay_fused_dense_bias_act"
    assert _status(de, 0, 10, 16, B.RELAY_F16, FAKE, FAKE, None, 0, FAKE + 4096, None) == 2
    assert _status(de, 1, 10, 12, B.RELAY_F16, FAKE, FAKE, None, 0, FAKE + 4096, None) == 5
    assert _status(de, 1, 10, 16, B.RELAY_I8, FAKE, FAKE, None, 0, FAKE + 4096, None) == 3
    assert _status(de, 1, 10, 16, B.RELAY_F16, FAKE, FAKE, None, 2, FAKE + 4096, None) == 4
    assert _status(de, 1, 10, 16, B.RELAY_F16, None, FAKE, None, 0, FAKE + 4096, None) == 1
    assert _status("relay_maxpool2d", B.RELAY_F16, 1, 12, 8, 8, 3, 2, 1, FAKE, FAKE + 4096, None) == 5
    assert _status("relay_maxpool2d", B.RELAY_F32, 1, 16, 8, 8, 3, 2, 1, FAKE, FAKE + 4096, None) == 3
    assert _status("relay_maxpool2d", B.RELAY_F16, 1, 16, 8, 8, 3, 2, 3, FAKE, FAKE + 4096, None) == 2
    assert _status("relay_global_avgpool", B.RELAY_I8, 1, 16, 4, FAKE, FAKE + 4096, None) == 3
    assert _status("relay_nchw_to_nhwc", B.RELAY_F16, 1, 3, 8, 8, 2, FAKE, FAKE + 4096, None) == 2
    assert _status("relay_nchw_to_nhwc", B.RELAY_F16, 1, 3, 8, 8, 8, FAKE, FAKE, None) == 4
    assert _status("relay_pack_input_nhwc4", C.byref(_d(c=3)), None, FAKE, None) == 1
    assert _status("relay_pack_input_nhwc4", C.byref(_d(c=8)), FAKE, FAKE + 4096, None) == 2
    assert _status("relay_set_conv_tile", 99) == 4
    assert _status("relay_set_conv_tile", -1) == 0
    buf = C.create_string_buffer(128)
    assert _status("relay_conv2d_kernel_name", C.byref(_d()), None, 0) == 1
    assert _status("relay_conv2d_kernel_name", C.byref(_d(n=32, h=56, w=56)), buf, 128) == 0
    assert buf.value.decode() == "conv3x3_halo_kernel<false, 4, 1, 2, 2, 2, 2>"   # 3x3 / stride 1, 64 channels, 813 tiles of 128: the 256 x 64 variant
    assert _status("relay_conv2d_kernel_name", C.byref(_d(n=16, h=56, w=56)), buf, 128) == 0
    assert buf.value.decode() == "conv3x3_halo_kernel<false, 2, 2, 2, 1, 2, 1>"   # 407 tiles: one round of 128 x 64 tiles
    assert _status("relay_conv2d_kernel_name", C.byref(_d(n=32, h=56, w=56, stride=2)), buf, 128) == 0
    assert buf.value.decode().startswith("igemm_dma_kernel<false")
    assert _status("relay_conv2d_kernel_name", C.byref(_d(c=24)), buf, 128) == 0
    assert buf.value.decode().startswith("igemm_conv_kernel<false")


def test_first_layer_checks():
    fl = "relay_fused_conv2d_first_layer"
    good = dict(c=3, k=32, h=32, w=32, stride=2, pad=1, layout=B.RELAY_NCHW)
    args = (FAKE, FAKE + 4096, None, None, None, FAKE + 8192, None)
    assert _status(fl, C.byref(_d(**good)), None, *args[1:]) == 1
    assert _status(fl, C.byref(_d(**{**good, "dtype": B.RELAY_I8})), *args) == 3
    assert _status(fl, C.byref(_d(**{**good, "layout": B.RELAY_NHWC})), *args) == 4
    for bad in (dict(c=4), dict(k=24), dict(k=256), dict(w=36), dict(h=31), dict(stride=1), dict(pad=0), dict(r=5, s=5, pad=2),
                dict(flags=B.HAS_RESIDUAL)):
        assert _status(fl, C.byref(_d(**{**good, **bad})), *args) == 4, bad
    assert _status(fl, C.byref(_d(**good)), FAKE + 2, *args[1:]) == 5
    assert _status(fl, C.byref(_d(**{**good, "flags": B.HAS_BIAS})), *args) == 1       # flag set, array missing
    nb = C.c_size_t(0)
    assert _status("relay_first_layer_packed_weight_bytes", C.byref(_d(**good)), C.byref(nb)) == 0 and nb.value == 32 * 14 * 4
    assert _status("relay_first_layer_packed_weight_bytes", C.byref(_d(**{**good, "k": 24})), C.byref(nb)) == 4
    assert _status("relay_prepack_first_layer_weights", C.byref(_d(**good)), None, FAKE, None) == 1
    assert _status("relay_prepack_first_layer_weights", C.byref(_d(**good)), FAKE, FAKE + 8, None) == 5
    ok = C.c_int32(-1)
    assert _status("relay_conv2d_first_layer_supported", C.byref(_d(**good)), C.byref(ok)) == 0 and ok.value == 1
    assert _status("relay_conv2d_first_layer_supported", C.byref(_d(**{**good, "c": 4})), C.byref(ok)) == 0 and ok.value == 0
    assert _status("relay_conv2d_first_layer_supported", C.byref(_d(**good)), None) == 1


def test_grid_barrier_probe_checks():
    gb = "relay_probe_grid_barrier"
    assert _status(gb, 0, 1, 10, FAKE, None, None) == 4
    assert _status(gb, 2048, 1, 10, FAKE, None, None) == 4        # more workgroups than are sure to be resident at once
    assert _status(gb, 64, -1, 10, FAKE, None, None) == 4
    assert _status(gb, 64, 1, 0, FAKE, None, None) == 4           # a wait that may not poll at all
    assert _status(gb, 64, 1, 10, None, None, None) == 1
    assert _status(gb, 64, 1, 10, FAKE + 2, None, None) == 5


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1904_08368_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in ("oracle/__init__.py", "oracle/stack.py", "oracle/oracle.c"):
        text = open(os.path.join(ROOT, f)).read()
        assert "paper_1904_08368_amd" not in text and "relay_fused" not in text


def test_quantize_and_elementwise_arguments_are_checked_on_the_host():
    """Every refusal below happens before any HIP call (FAKE is never dereferenced)."""
    lib = B.lib()
    q = lambda **kw: lib.relay_quantize(*[{**dict(n=64, src=B.RELAY_F32, x=FAKE, rho=2.0, beta=8, sigma=1, mode=0, seed=0,
                                                  y=FAKE + 4096, st=None), **kw}[k]
                                          for k in ("n", "src", "x", "rho", "beta", "sigma", "mode", "seed", "y", "st")])
    assert q(n=0) == 2 and q(x=None) == 1 and q(y=None) == 1
    assert q(src=B.RELAY_I8) == 3
    assert q(rho=0.0) == 2 and q(rho=-1.0) == 2 and q(rho=float("inf")) == 2 and q(rho=float("nan")) == 2
    assert q(beta=9) == 4 and q(beta=1) == 4 and q(sigma=9) == 4 and q(mode=4) == 4 and q(mode=-1) == 4
    assert q(x=FAKE + 4) == 5 and q(y=FAKE + 4096 + 4) == 5
    assert q(y=FAKE) == 4                                     # output aliases the input
    s = lambda **kw: lib.relay_sim_quantize(*[{**dict(n=64, x=FAKE, rho=2.0, beta=8, sigma=1, mode=0, seed=0, y=FAKE + 4096,
                                                      st=None), **kw}[k]
                                              for k in ("n", "x", "rho", "beta", "sigma", "mode", "seed", "y", "st")])
    assert s(beta=25) == 4 and s(beta=24, y=FAKE + 4096 + 8) == 5 and s(x=None) == 1 and s(n=-5) == 2
    e = lambda **kw: lib.relay_elementwise_f16(*[{**dict(op=B.EW_RELU, n=10, c=64, x=FAKE, p0=None, p1=None, other=None,
                                                         y=FAKE + 4096, st=None), **kw}[k]
                                                 for k in ("op", "n", "c", "x", "p0", "p1", "other", "y", "st")])
    assert e(op=7) == 4 and e(n=0) == 2 and e(c=12) == 5 and e(x=None) == 1
    assert e(p0=FAKE) == 1                                    # relu takes no parameters
    assert e(op=B.EW_BIAS_ADD) == 1 and e(op=B.EW_SCALE_SHIFT, p0=FAKE) == 1 and e(op=B.EW_ADD) == 1
    assert e(op=B.EW_ADD, other=FAKE + 2) == 5
    assert b"op" in lib.relay_last_error() or lib.relay_last_error()


def test_rounding_entry_point_checks_mode_and_shifts():
    lib = B.lib()
    d = _d(dtype=B.RELAY_I8, c=64)
    call = lambda mode=0, s=5, l=0: lib.relay_qconv2d_requant_rounding(C.byref(d), FAKE, FAKE + 4096, None, None, l, s, mode, 1,
                                                                       FAKE + 8192, None, 0, None)
    assert call(mode=4) == 4 and call(mode=-1) == 4 and call(s=32) == 4 and call(s=-1) == 4 and call(l=24) == 4


def _comb(d, x=FAKE, x_ld=None, w=FAKE, bias=None, sc=None, sf=None, ch=(32, 32), ys=(FAKE + 4096, FAKE + 8192),
          ld=None, arrays=True):
    n = len(ch)
    cha = (C.c_int32 * max(n, 1))(*ch)
    lda = (C.c_int32 * max(n, 1))(*(ld if ld is not None else ch))
    ya = (C.c_void_p * max(n, len(ys), 1))(*ys)
    P = C.c_void_p
    return _status("relay_fused_conv2d_combined", C.byref(d), x, d.c if x_ld is None else x_ld, w, bias, sc, sf, n,
                   C.cast(cha, P) if arrays else None, C.cast(ya, P), C.cast(lda, P), None)


def test_combined_conv_argument_checks():
    """Every case fails validation on the host; nothing is launched."""
    assert _comb(_d(), x=None) == 1
    assert _comb(_d(), arrays=False) == 1
    assert _comb(_d(), ys=(FAKE + 4096, None)) == 1
    assert _comb(_d(flags=B.HAS_BIAS)) == 1                                   # flag set, pointer NULL
    assert _comb(_d(), sc=FAKE) == 1                                          # pointer given, flag clear
    assert _comb(_d(dtype=B.RELAY_I8)) == 3
    assert _comb(_d(layout=B.RELAY_NCHW)) == 4
    assert _comb(_d(flags=B.HAS_RESIDUAL)) == 4
    assert _comb(_d(), ch=()) == 2                                            # nseg outside 1..4
    assert _comb(_d(), ch=(16,) * 5, ys=(FAKE + 4096,) * 5) == 2
    assert _comb(_d(), ch=(32, 24)) == 2                                      # segments do not add up to k
    assert _comb(_d(), ch=(60, 4)) == 2                                       # not multiples of 8
    assert _comb(_d(), ld=(32, 24)) == 2                                      # pitch below the segment
    assert _comb(_d(), ld=(32, 36)) == 2                                      # pitch not a multiple of 8
    assert _comb(_d(), x_ld=56) == 2 and _comb(_d(), x_ld=68) == 2            # below c / not a multiple of 8
    assert _comb(_d(), ys=(FAKE + 4096, FAKE + 4096)) == 4                    # two segments at one address
    assert _comb(_d(), ys=(FAKE, FAKE + 4096)) == 4                           # output aliases the input
    assert _comb(_d(), ys=(FAKE + 4096, FAKE + 8200)) == 5                    # misaligned
    assert _comb(_d(c=48, k=64)) == 4                                         # c % 32: no direct-to-LDS kernel
    assert _comb(_d(n=4096, h=64, w=64, c=64), x_ld=256) == 2                 # view beyond 2^31-1 elements


def _qcomb(d, x=FAKE, x_ld=None, bias=None, mult=None, rsh=None, s=7, ch=(32, 32), ys=(FAKE + 4096, FAKE + 8192), ld=None):
    n = len(ch)
    P = C.c_void_p
    cha = (C.c_int32 * max(n, 1))(*ch)
    lda = (C.c_int32 * max(n, 1))(*(ld if ld is not None else ch))
    ya = (C.c_void_p * max(n, 1))(*ys)
    return _status("relay_qconv2d_combined", C.byref(d), x, d.c if x_ld is None else x_ld, FAKE, bias, mult, rsh, s, n,
                   C.cast(cha, P), C.cast(ya, P), C.cast(lda, P), None)


def test_quantized_combined_conv_argument_checks():
    """The 8-bit combination validates on the host like the fp16 one, plus its requantization arguments."""
    q = lambda **kw: _d(dtype=B.RELAY_I8, c=64, **kw)
    assert _qcomb(_d(c=64)) == 3                                               # fp16 descriptor
    assert _qcomb(q(), mult=FAKE) == 1 and _qcomb(q(), rsh=FAKE) == 1          # multiplier and shift come together
    assert _qcomb(q(), s=32) == 4 and _qcomb(q(), s=-1) == 4
    assert _qcomb(q(), mult=FAKE + 2, rsh=FAKE) == 5
    assert _qcomb(q(flags=B.HAS_BN)) == 4
    assert _qcomb(q(flags=B.HAS_BIAS)) == 1
    assert _qcomb(q(), x_ld=72) == 2                                           # input pitch not a multiple of 16
    assert _qcomb(q(), ys=(FAKE + 4096, FAKE + 8196)) == 5                     # an 8-byte store would straddle
    assert _qcomb(q(), ch=(32, 24)) == 2
    assert _qcomb(_d(dtype=B.RELAY_I8, c=32)) == 4                             # c % 64: no direct-to-LDS kernel


def test_fused_depthwise_pointwise_argument_checks():
    """The one-launch depthwise + 1x1 entry point and its profitability query validate on the host."""
    lib = B.lib()
    dw = lambda **kw: _d(**{**dict(c=64, k=64, r=3, s=3, pad=1, h=56, w=56), **kw})
    call = lambda d, k=128, pf=0, x=FAKE, w=FAKE + 4096, pw=FAKE + 8192, y=FAKE + (1 << 20), pb=None: \
        lib.relay_fused_dwconv_pwconv(C.byref(d), x, w, None, None, None, k, pf, pw, pb, None, None, y, None)
    assert call(dw(pad=0)) == 4 and call(dw(c=40, k=40)) == 4              # padding 1 only; c % 32
    assert call(dw(dtype=B.RELAY_I8)) == 3
    assert call(dw(), k=12) == 2 and call(dw(), k=0) == 2
    assert call(dw(), pf=B.HAS_RESIDUAL) == 4
    assert call(dw(), pf=B.HAS_BIAS) == 1 and call(dw(), pb=FAKE) == 1      # flag and pointer disagree
    assert call(dw(), x=None) == 1 and call(dw(), y=FAKE) == 4             # output aliases the input
    assert call(dw(), pw=FAKE + 8200) == 5
    assert call(dw(flags=B.HAS_BN)) == 1                                   # dw_scale missing
    pays = C.c_int32(-1)
    q = lambda d, k: (lib.relay_dwconv_pwconv_fusion_pays(C.byref(d), k, C.byref(pays)), pays.value)
    assert q(dw(n=32, c=128, k=128), 128) == (0, 1)                        # streams from memory: one launch pays
    assert q(dw(n=32, c=1024, k=1024, h=7, w=7), 1024) == (0, 0)           # deepest layer: two launches are faster
    assert q(dw(n=1, c=128, k=128), 128) == (0, 0)                         # too few pixels
    assert q(dw(pad=0), 128)[0] == 4 and lib.relay_dwconv_pwconv_fusion_pays(C.byref(dw()), 128, None) == 1


def test_scale_folding_argument_checks():
    f = lambda *a: _status("relay_fold_scale_axis", *a)
    assert f(B.RELAY_I8, 8, 8, 9, 0, FAKE, FAKE, FAKE, None) == 3
    assert f(B.RELAY_F16, 0, 8, 9, 0, FAKE, FAKE, FAKE, None) == 2
    assert f(B.RELAY_F16, 1 << 16, 1 << 16, 9, 0, FAKE, FAKE, FAKE, None) == 2
    assert f(B.RELAY_F16, 8, 8, 9, 2, FAKE, FAKE, FAKE, None) == 4
    assert f(B.RELAY_F16, 8, 8, 9, 0, None, FAKE, FAKE, None) == 1
    assert f(B.RELAY_F32, 8, 8, 9, 1, FAKE + 2, FAKE, FAKE, None) == 5
    g = lambda *a: _status("relay_fold_bias", *a)
    assert g(0, None, FAKE, FAKE, FAKE, None) == 2
    assert g(8, None, None, FAKE, FAKE, None) == 1
    assert g(8, FAKE + 1, FAKE, FAKE, FAKE, None) == 5


def _pool(d, x=FAKE, w=FAKE, bias=None, sc=None, sf=None, y=FAKE + 4096):
    return _status("relay_fused_conv2d_bn_relu_maxpool", C.byref(d), x, w, bias, sc, sf, y, None)


def _qpool(d, x=FAKE, w=FAKE, bias=None, s=8, y=FAKE + 4096):
    return _status("relay_qconv2d_requant_maxpool", C.byref(d), x, w, bias, s, y, None)


def test_pooled_conv_argument_checks():
    ok = dict(h=14, w=16)                                         # conv output 14 x 16: one block of pooled outputs
    assert B.relay_conv2d_maxpool_fusable(_d(**ok))
    assert B.relay_conv2d_maxpool_fusable(_d(c=3, h=224, w=224, r=7, s=7, stride=2, pad=3, layout=B.RELAY_NHWC4_PADDED))
    assert B.relay_conv2d_maxpool_fusable(_d(dtype=B.RELAY_I8, **ok))
    for bad in (_d(), _d(h=14, w=24), _d(h=21, w=16), _d(k=60, **ok), _d(c=8, **ok), _d(flags=B.HAS_RESIDUAL, **ok),
                _d(dtype=B.RELAY_F32, layout=B.RELAY_NCHW, **ok), _d(dtype=B.RELAY_I8, flags=B.HAS_BN, **ok)):
        assert not B.relay_conv2d_maxpool_fusable(bad)
    assert _pool(_d()) == 4                                       # 8 x 8 conv output: no whole block
    assert _pool(_d(h=14, w=24)) == 4 and _pool(_d(h=21, w=16)) == 4
    assert _pool(_d(flags=B.HAS_RESIDUAL, **ok)) == 4
    assert _pool(_d(dtype=B.RELAY_I8, **ok)) == 3
    assert _pool(_d(**ok), x=None) == 1 and _pool(_d(**ok), y=None) == 1
    assert _pool(_d(flags=B.HAS_BN, **ok), sc=FAKE) == 1
    assert _pool(_d(**ok), bias=FAKE) == 1
    assert _pool(_d(**ok), y=FAKE) == 4
    assert _pool(_d(**ok), y=FAKE + 4096 + 8) == 5
    q = dict(dtype=B.RELAY_I8, **ok)
    assert _qpool(_d(**ok)) == 3
    assert _qpool(_d(**q), s=-1) == 4 and _qpool(_d(**q), s=32) == 4
    assert _qpool(_d(flags=B.HAS_BN, **q)) == 4
    assert _qpool(_d(**q), x=None) == 1
    assert _qpool(_d(**q), y=FAKE + 4) == 5
    assert _qpool(_d(flags=B.HAS_BIAS, **q)) == 1
    assert _status("relay_conv2d_maxpool_fusable", C.byref(_d()), None) == 1
    assert B.relay_conv2d_maxpool_kernel_name(_d(**ok)) == "igemm_dma_kernel<false, 4, 1, 2, 2, 2, 1, 1, false, false, true>"
    assert _status("relay_conv2d_maxpool_kernel_name", C.byref(_d()), C.create_string_buffer(64), 64) == 4


def _combw(d, ch, win, relu, arrays=True):
    n = len(ch)
    P = C.c_void_p
    mk = lambda v: (C.c_int32 * max(len(v), 1))(*v)
    cha, lda, wa, ra = mk(ch), mk(ch), mk(win), mk(relu)
    ya = (C.c_void_p * max(n, 1))(*[FAKE + 4096 * (i + 1) for i in range(n)])
    return _status("relay_fused_conv2d_combined_windows", C.byref(d), FAKE, d.c, FAKE, None, None, None, n, C.cast(cha, P),
                   C.cast(ya, P), C.cast(lda, P), C.cast(wa, P) if arrays else None, C.cast(ra, P), None)


def test_combined_windows_argument_checks():
    """The per-segment window / relu arrays are validated on the host like everything else."""
    s2 = dict(stride=2, k=256, flags=B.RELU)
    assert _combw(_d(**s2), (128, 128), (0, 1), (1, 0), arrays=False) == 1
    assert _combw(_d(**s2), (128, 128), (0, 2), (1, 0)) == 4                  # not a relay_segment_window
    assert _combw(_d(**s2), (128, 128), (0, 1), (1, 2)) == 4                  # relu is 0 or 1
    assert _combw(_d(stride=2, k=256), (128, 128), (0, 1), (1, 0)) == 4      # seg_relu without RELAY_RELU
    assert _combw(_d(**s2), (64, 192), (0, 1), (1, 0)) == 2                   # centre segment off the 128-channel grid
    assert _combw(_d(stride=2, k=192, flags=B.RELU), (128, 64), (0, 1), (1, 0)) == 2
    assert _combw(_d(pad=0, **s2), (128, 128), (0, 1), (1, 0)) == 4           # window not padded by half its size
    assert _combw(_d(r=4, s=4, pad=2, **s2), (128, 128), (0, 1), (1, 0)) == 4  # even window: no centre tap
    # (a valid request is not tried here: it would launch)


def test_realize_and_calibrate_validate_on_the_host():
    f = C.c_float
    ok = dict(k=4, per_k=72, w=FAKE, bias=None, scale=None, shift=None, rx=f(4.0), ry=f(16.0), rr=f(0.0), wq=FAKE + 4096,
              bq=None, out=FAKE + 8192, ws=FAKE + 16384, wsb=4 * 72 * 4 + 16)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return _status("relay_realize_conv", a["k"], a["per_k"], a["w"], a["bias"], a["scale"], a["shift"], a["rx"], a["ry"],
                       a["rr"], a["wq"], a["bq"], a["out"], a["ws"], a["wsb"], None)
    assert call(k=0) == 2 and call(per_k=0) == 2 and call(k=1 << 20, per_k=1 << 20) == 2
    assert call(w=None) == 1 and call(wq=None) == 1 and call(out=None) == 1 and call(ws=None) == 1
    assert call(scale=FAKE) == 1 and call(shift=FAKE) == 1            # scale and shift come together
    assert call(bias=FAKE) == 1                                       # a bias needs bias_q
    assert call(rx=f(0.0)) == 2 and call(ry=f(-1.0)) == 2 and call(rr=f(-1.0)) == 2 and call(rx=f(float("inf"))) == 2
    assert call(wsb=4 * 72 * 4) == 6
    assert call(ws=FAKE + 16384 + 8) == 5 and call(w=FAKE + 2) == 5
    assert call(wq=FAKE) == 4                                          # output aliases the input
    cal = lambda dtype=B.RELAY_F32, n=10, x=FAKE, rho=FAKE + 64, cell=FAKE + 128: _status(
        "relay_calibrate_pow2_range", dtype, n, x, rho, cell, None)
    assert cal(dtype=B.RELAY_I8) == 3 and cal(n=0) == 2 and cal(x=None) == 1 and cal(rho=None) == 1 and cal(cell=None) == 1
    assert cal(rho=FAKE + 2) == 5


def test_tuning_overrides_are_thread_local():
    """A tile forced by one thread must not change what another thread's calls choose."""
    import threading
    d = _d(n=32, c=128, h=28, w=28, k=128)
    B.relay_set_conv_tile(-1)
    default = B.relay_conv2d_kernel_name(d)
    seen = {}

    def other():
        B.relay_set_conv_tile(5)
        seen["forced"] = B.relay_conv2d_kernel_name(d)
    t = threading.Thread(target=other)
    t.start()
    t.join()
    assert seen["forced"] != default and "igemm_dma_kernel" in seen["forced"]
    assert B.relay_conv2d_kernel_name(d) == default          # this thread still has its own setting


def test_every_entry_point_declaration_cites_its_source():
    """Each declared function sits behind a comment that names the passage defining the operation
    (a section of the paper) or, for the allocation-free variant, the callers it is for."""
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include")))
                   if f.endswith(".h"))
    missing = []
    for m in re.finditer(r"\brelay_status\s+(relay_[a-z0-9_]+)\s*\(|const char\*\s+(relay_last_error)\s*\(", text):
        name = m.group(1) or m.group(2)
        head = text[:m.start()]
        comment = head[head.rfind("/*"):]
        if "Section" not in comment and "cannot allocate" not in comment:
            missing.append(name)
    assert not missing, missing


def test_scheme_entry_points_validate_on_the_host():
    d8 = _d(dtype=B.RELAY_I8, flags=B.HAS_BIAS)
    by = C.byref
    # general scale: the per-channel arrays are required
    assert _status("relay_qconv2d_requant_scaled", by(d8), FAKE, FAKE + 4096, FAKE + 8192, None, 0, None, FAKE, FAKE + 65536, None, 0, None) == 1
    assert _status("relay_qconv2d_requant_scaled", by(d8), FAKE, FAKE + 4096, FAKE + 8192, None, 0, FAKE + 2, FAKE, FAKE + 65536, None, 0, None) == 5
    # 16-bit accumulator: same argument rules as the plain quantized conv
    assert _status("relay_qconv2d_requant_acc16", by(d8), FAKE, FAKE + 4096, FAKE + 8192, None, 0, 32, FAKE + 65536, None, 0, None) == 4
    assert _status("relay_qconv2d_requant_acc16", by(_d(dtype=B.RELAY_F16)), FAKE, FAKE + 4096, None, None, 0, 3, FAKE + 65536, None, 0, None) == 3
    # 16/32
    d16 = _d(dtype=B.RELAY_I16, flags=0)
    assert _status("relay_qconv2d_requant_i16", by(_d(dtype=B.RELAY_I8)), FAKE, FAKE + 4096, None, 3, FAKE + 65536, None) == 3
    assert _status("relay_qconv2d_requant_i16", by(_d(dtype=B.RELAY_I16, c=12)), FAKE, FAKE + 4096, None, 3, FAKE + 65536, None) == 5
    assert _status("relay_qconv2d_requant_i16", by(_d(dtype=B.RELAY_I16, k=6)), FAKE, FAKE + 4096, None, 3, FAKE + 65536, None) == 5
    assert _status("relay_qconv2d_requant_i16", by(_d(dtype=B.RELAY_I16, flags=B.HAS_BN)), FAKE, FAKE + 4096, None, 3, FAKE + 65536, None) == 4
    assert _status("relay_qconv2d_requant_i16", by(d16), FAKE, FAKE + 4096, None, 40, FAKE + 65536, None) == 4
    assert _status("relay_qconv2d_requant_i16", by(d16), None, FAKE + 4096, None, 3, FAKE + 65536, None) == 1
    assert B.relay_packed_weight_bytes(d16) == 64 * 576 * 2                 # packed like the other 2-byte type
    # the other entry points do not take the 16-bit integer type
    assert _status("relay_fused_conv2d_bias_bn_relu", by(d16), FAKE, FAKE + 4096, None, None, None, None, FAKE + 65536, None, 0, None) == 3
    assert _status("relay_qconv2d_requant", by(d16), FAKE, FAKE + 4096, None, None, 0, 3, FAKE + 65536, None, 0, None) == 3
    # unsigned activations
    need = B.relay_qconv2d_u8_workspace_bytes(d8)
    assert need == 1 * 10 * 10 * 64
    call = lambda d=d8, x=FAKE, ws=FAKE + (1 << 20), wsb=need, s=5, ou=1, bz=FAKE + 8192: _status(
        "relay_qconv2d_requant_u8", by(d), x, FAKE + 4096, bz, s, ou, FAKE + 65536, ws, wsb, None)
    assert call(wsb=need - 1) == 6 and call(ws=None) == 1 and call(x=None) == 1 and call(ou=2) == 4 and call(s=32) == 4
    assert call(d=_d(dtype=B.RELAY_I8, flags=0)) == 1                      # the zero-point term needs the bias operand
    assert call(d=_d(dtype=B.RELAY_I8, flags=B.HAS_BIAS | B.HAS_RESIDUAL)) == 4
    assert call(d=_d(dtype=B.RELAY_I8, c=24, flags=B.HAS_BIAS)) == 5 and call(d=_d(dtype=B.RELAY_F16, flags=B.HAS_BIAS)) == 3
    assert _status("relay_fold_zero_point", 0, 72, FAKE, None, 128, FAKE + 4096, None) == 2
    assert _status("relay_fold_zero_point", 4, 72, None, None, 128, FAKE + 4096, None) == 1
    assert _status("relay_fold_zero_point", 4, 72, FAKE, None, 300, FAKE + 4096, None) == 4
    # the multiplier decomposition is host code: 0.5 = 2^30 / 2^31, 3/16 = 0.75 * 2^-2
    assert B.relay_quantize_multiplier(0.5) == (1 << 30, 0) and B.relay_quantize_multiplier(0.1875) == (3 << 29, 2)
    m, s = B.relay_quantize_multiplier(1e-3)
    assert abs(m / 2.0 ** (31 + s) - 1e-3) < 1e-12 and (1 << 30) <= m < (1 << 31)
    for bad in (0.0, 1.0, 2.0 ** -40):
        with pytest.raises(B.RelayError) as e:
            B.relay_quantize_multiplier(bad)
        assert e.value.status == 2

"""A network as a sequence of fused primitive functions called one after another on
preallocated buffers (paper Section 3.3: operator invocations replaced by calls to the
compiled operators, inputs and outputs preallocated).

Set-up (filter packing, channel padding of filters, buffer allocation) is compile-time
work and happens once in the constructor; ``run()`` only enqueues kernels of the library
on torch's current stream, so it can also be captured into a HIP graph.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as B


def _round_up(a: int, b: int) -> int:
    return (a + b - 1) // b * b


class FusedNet:
    """mode 'f16': fp16 NHWC, fp32 accumulation.  mode 'i8': int8 NHWC, int32 accumulation,
    ``shifts[i] = {'s': out_rshift, 'l': residual_lshift}`` per conv."""

    def __init__(self, ops, params: List[dict], batch: int, h: int, w: int, mode: str = "f16",
                 shifts: Optional[List[dict]] = None, in_channels: int = 3, device: str = "cuda:0",
                 overlap_shortcuts: bool = False, fused: bool = True, combine: bool = False,
                 fold_scale: bool = False, fuse_pool: bool = True, fuse_dwpw: bool = True,
                 first_layer_direct: bool = True):
        assert mode in ("f16", "i8")
        assert fused or mode == "f16"
        # combine: convs that share input, window and tail run as one launch ("windows": also a 1x1 conv
        # beside a wider odd window of the same stride, and tails that differ in relu); fold_scale: the
        # batch-norm scale is multiplied into the filters ahead of time (paper Section 4.4, both)
        assert not (combine or fold_scale) or (mode == "f16" and fused)
        self.fold_scale = fold_scale
        # fuse_pool: a conv whose only reader is a 3x3 / stride 2 / pad 1 max pool runs with it as one
        # launch where the library takes the shape; the conv's own output tensor then does not exist
        self.fuse_pool = fuse_pool and fused
        # fuse_dwpw: a depthwise conv whose only reader is a plain 1x1 conv runs with it as one launch where
        # the library expects that to be faster; the depthwise output tensor then does not exist
        # ("always": wherever the library has a kernel for the shape, profitable or not)
        self.fuse_dwpw = fuse_dwpw if (fused and mode == "f16" and not fold_scale) else False
        # fused=False launches every elementwise operator behind a contraction as a kernel of its
        # own on a tensor of its own: the pipeline of a framework without operator fusion, kept
        # for the fusion ablation (paper Section 5.2)
        self.fused = fused
        self.ops, self.mode, self.batch = ops, mode, batch
        self.dev = torch.device(device)
        self.dtype = B.RELAY_F16 if mode == "f16" else B.RELAY_I8
        self.tdtype = torch.float16 if mode == "f16" else torch.int8
        self.ve = 8 if mode == "f16" else 16
        self.calls = []                      # (callable, args) in execution order
        self.call_names: List[str] = []
        self.bufs: Dict[str, torch.Tensor] = {}
        self.shape: Dict[str, tuple] = {}    # name -> (C_logical, H, W), physical C = padded
        self.keep = []                       # parameter tensors kept alive

        cpad = _round_up(in_channels, self.ve)
        self.x_nchw = torch.zeros((batch, in_channels, h, w), dtype=self.tdtype, device=self.dev)
        self.shape["x"] = (in_channels, h, w)
        first = ops[0]
        only_reader = first.kind == "conv" and first.src == "x" and \
            sum(1 for o in ops if o.src == "x" or o.res == "x") == 1
        # a first-layer conv the library reads straight from the NCHW image (3 channels, 3x3 / stride 2): no
        # converted or padded copy of the image at all
        self.stem_direct = False
        if only_reader and fused and mode == "f16" and not (combine or fold_scale) and first_layer_direct and \
                not first.res:
            d0 = B.conv_desc(batch, in_channels, h, w, first.cout, first.r, first.r, first.stride, first.pad,
                             self.dtype, B.RELAY_NCHW, 0)
            try:
                self.stem_direct = B.relay_conv2d_first_layer_supported(d0)
            except B.RelayError:
                self.stem_direct = False
        # a first-layer conv on <= 4 channels reads the pre-padded NHWC4 form of the image
        self.stem_nhwc4 = only_reader and in_channels <= 4 and not self.stem_direct
        if self.stem_direct:
            self.bufs["x"] = self.x_nchw
        elif self.stem_nhwc4:
            d0 = B.conv_desc(batch, in_channels, h, w, first.cout, first.r, first.r, first.stride, first.pad,
                             self.dtype, B.RELAY_NHWC4_PADDED, 0)
            hp, wp = B.relay_nhwc4_padded_shape(d0)
            self.bufs["x"] = torch.zeros((batch, hp, wp, 4), dtype=self.tdtype, device=self.dev)
            self._add("pack_input_nhwc4", B.relay_pack_input_nhwc4, (d0, self.x_nchw, self.bufs["x"]))
            self.keep.append(d0)
        else:
            self.bufs["x"] = torch.zeros((batch, h, w, cpad), dtype=self.tdtype, device=self.dev)
            self._add("nchw_to_nhwc", B.relay_nchw_to_nhwc,
                      (self.dtype, batch, in_channels, h, w, cpad, self.x_nchw, self.bufs["x"]))

        from .fusion import combine_parallel
        group_of = {min(g): g for g in (combine_parallel(ops, windows=(combine == "windows")) if combine else [])}
        absorbed = {j for i, g in group_of.items() for j in g if j != i}
        self._plan_concats(ops, batch, h, w, in_channels, cpad)

        for i, (op, p) in enumerate(zip(ops, params)):
            if i in absorbed:
                continue
            cin_l, hi, wi = self.shape[op.src]
            src = self.bufs[op.src]
            cin_p = src.shape[-1]
            if op.kind == "concat":
                # nothing to launch: every producer has already written its channel range
                assert all(self.view_of.get(s_, (None,))[0] == op.dst for s_ in op.srcs)
                self.shape[op.dst] = (self.bufs[op.dst].shape[-1], hi, wi)
            elif op.kind == "conv" and (i in group_of or op.dst in self.view_of or not src.is_contiguous()):
                idxs = group_of.get(i, [i])
                self._emit_conv_views([ops[j] for j in idxs], [params[j] for j in idxs], batch)
            elif op.kind == "conv" and i == 0 and self.stem_direct:
                flags = B.flags_of(p.get("bias"), p.get("scale"), None, op.relu)
                d = B.conv_desc(batch, cin_l, hi, wi, op.cout, op.r, op.r, op.stride, op.pad, self.dtype, B.RELAY_NCHW, flags)
                ho, wo = B.relay_conv2d_out_shape(d)
                wsrc = torch.from_numpy(np.ascontiguousarray(p["w"])).to(self.dev)
                y = torch.empty((batch, ho, wo, op.cout), dtype=self.tdtype, device=self.dev)
                bias, sc, sf = (self._f32(p.get(k)) for k in ("bias", "scale", "shift"))
                wp = torch.empty(B.relay_first_layer_packed_weight_bytes(d), dtype=torch.uint8, device=self.dev)
                B.relay_prepack_first_layer_weights(d, wsrc, wp)
                self._add(op.name, B.relay_fused_conv2d_first_layer, (d, src, wp, bias, sc, sf, y))
                self.keep += [wp, d]
                self.bufs[op.dst], self.shape[op.dst] = y, (op.cout, ho, wo)
            elif op.kind == "conv":
                flags = B.flags_of(p.get("bias"), p.get("scale"), op.res, op.relu)
                if i == 0 and self.stem_nhwc4:
                    d = B.conv_desc(batch, cin_l, hi, wi, op.cout, op.r, op.r, op.stride, op.pad, self.dtype,
                                    B.RELAY_NHWC4_PADDED, flags)
                else:
                    d = B.conv_desc(batch, cin_p, hi, wi, op.cout, op.r, op.r, op.stride, op.pad, self.dtype,
                                    B.RELAY_NHWC, flags)
                ho, wo = B.relay_conv2d_out_shape(d)
                wsrc = torch.from_numpy(np.ascontiguousarray(p["w"])).to(self.dev)
                wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=self.dev)
                B.relay_prepack_conv2d_weights(d, wsrc, cin_l, wp)
                pool = self._pool_behind(ops, i) if self.fuse_pool and B.relay_conv2d_maxpool_fusable(d) else None
                if pool is not None:
                    absorbed.add(pool)
                    y = torch.empty((batch, ho // 2, wo // 2, op.cout), dtype=self.tdtype, device=self.dev)
                    name = op.name + "+" + ops[pool].name
                    if mode == "f16" and fold_scale and p.get("scale") is not None:
                        bias = self._fold(op, p, wsrc, cin_l)
                        B.relay_prepack_conv2d_weights(d, wsrc, cin_l, wp)
                        d = B.conv_desc(d.n, d.c, d.h, d.w, d.k, d.r, d.s, d.stride_h, d.pad_h, self.dtype, d.layout,
                                        B.flags_of(True, None, None, op.relu))
                        self._add(name, B.relay_fused_conv2d_bn_relu_maxpool, (d, src, wp, bias, None, None, y))
                    elif mode == "f16":
                        bias, sc, sf = (self._f32(p.get(k)) for k in ("bias", "scale", "shift"))
                        self._add(name, B.relay_fused_conv2d_bn_relu_maxpool, (d, src, wp, bias, sc, sf, y))
                    else:
                        qb = None
                        if p.get("bias") is not None:
                            qb = torch.from_numpy(np.ascontiguousarray(p["bias"], dtype=np.int32)).to(self.dev)
                            self.keep.append(qb)
                        self._add(name, B.relay_qconv2d_requant_maxpool, (d, src, wp, qb, int(shifts[i]["s"]), y))
                    self.keep += [wp, d]
                    self.bufs[ops[pool].dst], self.shape[ops[pool].dst] = y, (op.cout, ho // 2, wo // 2)
                    continue
                y = torch.empty((batch, ho, wo, op.cout), dtype=self.tdtype, device=self.dev)
                res = self.bufs[op.res] if op.res else None
                ws = self._workspace(d)     # None for most layers
                if mode == "f16" and not fused and flags:
                    d0 = B.conv_desc(d.n, d.c, d.h, d.w, d.k, d.r, d.s, d.stride_h, d.pad_h, self.dtype, d.layout, 0)
                    raw = torch.empty_like(y)
                    self._add(op.name, B.relay_fused_conv2d_bias_bn_relu, (d0, src, wp, None, None, None, None, raw))
                    self.keep.append(d0)
                    y = self._unfused_tail(op, p, raw, batch * ho * wo, op.cout, res)
                elif mode == "f16" and fold_scale and p.get("scale") is not None:
                    # the filters were packed unscaled above: pack the folded ones over them
                    bias = self._fold(op, p, wsrc, cin_l)
                    B.relay_prepack_conv2d_weights(d, wsrc, cin_l, wp)
                    d1 = B.conv_desc(d.n, d.c, d.h, d.w, d.k, d.r, d.s, d.stride_h, d.pad_h, self.dtype, d.layout,
                                     B.flags_of(True, None, op.res, op.relu))
                    self._add(op.name, B.relay_fused_conv2d_bias_bn_relu, (d1, src, wp, bias, None, None, res, y, ws))
                    self.keep.append(d1)
                elif mode == "f16":
                    bias, sc, sf = (self._f32(p.get(k)) for k in ("bias", "scale", "shift"))
                    self._add(op.name, B.relay_fused_conv2d_bias_bn_relu, (d, src, wp, bias, sc, sf, res, y, ws))
                else:
                    sh = shifts[i]
                    qb = None
                    if p.get("bias") is not None:
                        qb = torch.from_numpy(np.ascontiguousarray(p["bias"], dtype=np.int32)).to(self.dev)
                        self.keep.append(qb)
                    self._add(op.name, B.relay_qconv2d_requant,
                              (d, src, wp, qb, res, int(sh.get("l", 0)), int(sh["s"]), y, ws))
                self.keep += [wp, d]
                self.bufs[op.dst], self.shape[op.dst] = y, (op.cout, ho, wo)
            elif op.kind == "dwconv":
                flags = B.flags_of(p.get("bias"), p.get("scale"), None, op.relu)
                d = B.conv_desc(batch, cin_p, hi, wi, cin_p, op.r, op.r, op.stride, op.pad, self.dtype,
                                B.RELAY_NHWC, flags)
                ho, wo = B.relay_conv2d_out_shape(d)
                wsrc = torch.from_numpy(np.ascontiguousarray(p["w"])).to(self.dev)
                wp = torch.empty((op.r * op.r, cin_p), dtype=self.tdtype, device=self.dev)
                B.relay_prepack_dwconv_weights(d, wsrc, wp)
                pw = self._pointwise_behind(ops, i, group_of, absorbed) if self.fuse_dwpw and op.r == 3 and op.pad == 1 \
                    and cin_p % 32 == 0 and src.is_contiguous() else None
                if pw is not None and (self.fuse_dwpw == "always" or B.relay_dwconv_pwconv_fusion_pays(d, ops[pw].cout)):
                    q, pp = ops[pw], params[pw]
                    pflags = B.flags_of(pp.get("bias"), pp.get("scale"), None, q.relu)
                    pd = B.conv_desc(batch, cin_p, ho, wo, q.cout, 1, 1, 1, 0, self.dtype, B.RELAY_NHWC, pflags)
                    pwp = torch.empty(B.relay_packed_weight_bytes(pd), dtype=torch.uint8, device=self.dev)
                    B.relay_prepack_conv2d_weights(pd, torch.from_numpy(np.ascontiguousarray(pp["w"])).to(self.dev), cin_l, pwp)
                    y = torch.empty((batch, ho, wo, q.cout), dtype=self.tdtype, device=self.dev)
                    bias, sc, sf = (self._f32(p.get(k)) for k in ("bias", "scale", "shift"))
                    pb, psc, psf = (self._f32(pp.get(k)) for k in ("bias", "scale", "shift"))
                    self._add(op.name + "+" + q.name, B.relay_fused_dwconv_pwconv,
                              (d, src, wp, bias, sc, sf, q.cout, pflags, pwp, pb, psc, psf, y))
                    absorbed.add(pw)
                    self.keep += [wp, d, pwp, pd]
                    self.bufs[q.dst], self.shape[q.dst] = y, (q.cout, ho, wo)
                    continue
                y = torch.empty((batch, ho, wo, cin_p), dtype=self.tdtype, device=self.dev)
                if not fused and flags:
                    d0 = B.conv_desc(d.n, d.c, d.h, d.w, d.k, d.r, d.s, d.stride_h, d.pad_h, self.dtype, d.layout, 0)
                    raw = torch.empty_like(y)
                    self._add(op.name, B.relay_fused_dwconv_bias_relu, (d0, src, wp, None, None, None, raw))
                    self.keep.append(d0)
                    y = self._unfused_tail(op, p, raw, batch * ho * wo, cin_p, None)
                else:
                    bias, sc, sf = (self._f32(p.get(k)) for k in ("bias", "scale", "shift"))
                    self._add(op.name, B.relay_fused_dwconv_bias_relu, (d, src, wp, bias, sc, sf, y))
                self.keep += [wp, d]
                self.bufs[op.dst], self.shape[op.dst] = y, (op.cout, ho, wo)
            elif op.kind == "maxpool":
                ho = (hi + 2 * op.pad - op.r) // op.stride + 1
                wo = (wi + 2 * op.pad - op.r) // op.stride + 1
                y = torch.empty((batch, ho, wo, cin_p), dtype=self.tdtype, device=self.dev)
                self._add(op.name, B.relay_maxpool2d, (self.dtype, batch, cin_p, hi, wi, op.r, op.stride, op.pad, src, y))
                self.bufs[op.dst], self.shape[op.dst] = y, (cin_l, ho, wo)
            elif op.kind == "avgpool":
                y = torch.empty((batch, 1, 1, cin_p), dtype=self.tdtype, device=self.dev)
                self._add(op.name, B.relay_global_avgpool, (self.dtype, batch, cin_p, hi * wi, src, y))
                self.bufs[op.dst], self.shape[op.dst] = y, (cin_l, 1, 1)
            elif op.kind == "dense":
                wd = torch.from_numpy(np.ascontiguousarray(p["w"])).to(self.dev)
                if hi * wi > 1:
                    # a dense layer over a [C, H, W] tensor: its filters are given for (channel, row, column)
                    # order; the NHWC buffer holds (row, column, channel), so the columns are permuted once here
                    if cin_p != cin_l or op.cin != cin_l * hi * wi:
                        raise ValueError(f"{op.name}: dense over a padded or mismatched [{cin_l},{hi},{wi}] tensor")
                    wd = wd.reshape(op.cout, cin_l, hi, wi).permute(0, 2, 3, 1).reshape(op.cout, op.cin).contiguous()
                bias = self._f32(p.get("bias"))
                y = torch.empty((batch, 1, 1, op.cout), dtype=self.tdtype, device=self.dev)
                if not fused and mode == "f16" and (bias is not None or op.relu) and op.cout % 8 == 0:
                    raw = torch.empty_like(y)
                    self._add(op.name, B.relay_fused_dense_bias_act,
                              (batch, op.cout, op.cin, self.dtype, src, wd, None, 0, raw))
                    y = self._unfused_tail(op, p, raw, batch, op.cout, None)
                else:
                    self._add(op.name, B.relay_fused_dense_bias_act,
                              (batch, op.cout, op.cin, self.dtype, src, wd, bias, 1 if op.relu else 0, y))
                self.keep += [wd]
                self.bufs[op.dst], self.shape[op.dst] = y, (op.cout, 1, 1)
            else:
                raise ValueError(op.kind)
        # calls that may run beside their predecessor: a conv that reads the same tensor as the
        # conv before it and whose output is first needed as a residual.  Off by default: with the
        # fork placed in front of the sibling conv the two kernels really do overlap, and the whole
        # ResNet-18 stack is then slower than the serial order (batch 32: 0.322 against 0.303 ms per
        # step, batch 1: 0.191 against 0.161 ms, replayed from a HIP graph)
        self.side_calls, self.join_before = set(), set()
        self.side = None
        if overlap_shortcuts and fused:   # (the unfused tails would have to follow their conv onto the side stream)
            idx_of = {name: i for i, name in enumerate(self.call_names)}
            for j in range(1, len(ops)):
                a0, a1 = ops[j - 1], ops[j]
                if a0.kind == "conv" and a1.kind == "conv" and a0.src == a1.src and not a1.res and not a0.res:
                    users = [o for o in ops if o.src == a1.dst or o.res == a1.dst]
                    if len(users) == 1 and users[0].res == a1.dst and a1.name in idx_of and users[0].name in idx_of \
                            and idx_of.get(a0.name) == idx_of[a1.name] - 1:
                        self.side_calls.add(idx_of[a1.name])
                        self.join_before.add(idx_of[users[0].name])
            if self.side_calls:
                self.side = torch.cuda.Stream(device=self.dev)
        torch.cuda.synchronize(self.dev)
        self.graph = None

    def _pointwise_behind(self, ops, i, group_of, absorbed):
        """Index of the plain 1x1 / stride 1 conv that is the only reader of depthwise conv i's output, or None."""
        op = ops[i]
        users = [j for j, o in enumerate(ops) if o.src == op.dst or o.res == op.dst or op.dst in (getattr(o, "srcs", None) or ())]
        if len(users) != 1 or users[0] != i + 1:
            return None
        q = ops[users[0]]
        plain = q.kind == "conv" and q.src == op.dst and q.r == 1 and q.stride == 1 and q.pad == 0 and not q.res
        if not plain or users[0] in group_of or users[0] in absorbed or q.dst in self.view_of or op.dst in self.view_of:
            return None
        return users[0]

    @staticmethod
    def _pool_behind(ops, i):
        """Index of the 3x3 / stride 2 / pad 1 max pool that is the only reader of conv i's output, or None."""
        op = ops[i]
        if op.res:
            return None
        users = [j for j, o in enumerate(ops) if o.src == op.dst or o.res == op.dst or op.dst in (o.srcs or ())]
        if len(users) != 1 or users[0] != i + 1:
            return None
        q = ops[users[0]]
        return users[0] if (q.kind == "maxpool" and q.src == op.dst and (q.r, q.stride, q.pad) == (3, 2, 1)) else None

    def _plan_concats(self, ops, batch, h, w, in_channels, cpad):
        """A channel concatenation is free when every tensor it joins is written by a conv: the
        conv stores straight into its channel range of the joined tensor.  Allocates those joined
        tensors and records view_of[name] = (joined tensor, first channel)."""
        self.view_of: Dict[str, tuple] = {}
        if not any(o.kind == "concat" for o in ops):
            return
        if self.mode != "f16" or not self.fused:
            raise ValueError("concatenation needs the fp16 fused pipeline")
        phys, hw = {"x": cpad}, {"x": (h, w)}      # physical channels and spatial size of every tensor
        producer = {}
        for o in ops:
            hi, wi = hw[o.src]
            out = lambda e: (e + 2 * o.pad - o.r) // o.stride + 1
            if o.kind in ("conv", "dwconv", "maxpool"):
                phys[o.dst] = o.cout if o.kind == "conv" else phys[o.src]
                hw[o.dst] = (out(hi), out(wi))
            elif o.kind in ("avgpool", "dense"):
                phys[o.dst], hw[o.dst] = (phys[o.src] if o.kind == "avgpool" else o.cout), (1, 1)
            elif o.kind == "concat":
                phys[o.dst], hw[o.dst] = sum(phys[s_] for s_ in o.srcs), hw[o.srcs[0]]
                off = 0
                for s_ in o.srcs:
                    if producer.get(s_) != "conv" or s_ in self.view_of or phys[s_] % 8 or hw[s_] != hw[o.dst]:
                        raise ValueError(f"concat {o.name}: {s_} must be a conv output of the same size, used in one "
                                         "concatenation, with a multiple of 8 channels")
                    self.view_of[s_] = (o.dst, off)
                    off += phys[s_]
                self.bufs[o.dst] = torch.empty((batch, *hw[o.dst], off), dtype=self.tdtype, device=self.dev)
            producer[o.dst] = o.kind

    def _emit_conv_views(self, members, mparams, batch):
        """One launch for one or more fp16 convs over the same input (a channel range of a wider
        tensor or a plain one), each storing into its own tensor or channel range."""
        op0 = members[0]          # (a member with the widest window: combine_parallel lists those first)
        cin_l, hi, wi = self.shape[op0.src]
        src = self.bufs[op0.src]
        cin_p = src.shape[-1]
        if any(m.res for m in members):
            raise ValueError(f"{op0.name}: a conv with a residual operand cannot store into a view")
        has_bias = mparams[0].get("bias") is not None
        has_bn = mparams[0].get("scale") is not None
        fold = self.fold_scale and has_bn
        any_relu = any(m.relu for m in members)
        mixed = any(m.r != op0.r or m.relu != any_relu for m in members)   # needs the per-segment windows / tails
        flags = B.flags_of(True if (has_bias or fold) else None, None if fold or not has_bn else True, None, any_relu)
        ktot = sum(m.cout for m in members)
        d = B.conv_desc(batch, cin_p, hi, wi, ktot, op0.r, op0.r, op0.stride, op0.pad, self.dtype, B.RELAY_NHWC, flags)
        ho, wo = B.relay_conv2d_out_shape(d)
        wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=self.dev)
        consts = {k: [] for k in ("bias", "scale", "shift")}
        ys, off = [], 0
        for m, p in zip(members, mparams):
            dm = B.conv_desc(batch, cin_p, hi, wi, m.cout, op0.r, op0.r, m.stride, op0.pad, self.dtype, B.RELAY_NHWC, flags)
            nbytes = B.relay_packed_weight_bytes(dm)
            wsrc = torch.from_numpy(np.ascontiguousarray(p["w"])).to(self.dev)
            if fold:
                consts["bias"].append(self._fold(m, p, wsrc, cin_l))
            else:
                consts["bias"].append(self._f32(p.get("bias")))
                consts["scale"].append(self._f32(p.get("scale")))
                consts["shift"].append(self._f32(p.get("shift")))
            if m.r != op0.r:      # a 1x1 member: its filters at the centre tap of the group's window, zeros around
                assert m.r == 1 and m.pad == 0 and op0.r % 2 == 1 and op0.pad == op0.r // 2 and m.stride == op0.stride
                wide = torch.zeros((m.cout, wsrc.shape[1], op0.r, op0.r), dtype=wsrc.dtype, device=self.dev)
                wide[:, :, op0.r // 2, op0.r // 2] = wsrc[:, :, 0, 0]
                wsrc = wide
            B.relay_prepack_conv2d_weights(dm, wsrc, cin_l, wp[off:off + nbytes])
            off += nbytes
            if m.dst in self.view_of:
                cat, c0 = self.view_of[m.dst]
                y = self.bufs[cat][..., c0:c0 + m.cout]
            else:
                y = torch.empty((batch, ho, wo, m.cout), dtype=self.tdtype, device=self.dev)
            assert tuple(y.shape) == (batch, ho, wo, m.cout)
            ys.append(y)
            self.bufs[m.dst], self.shape[m.dst] = y, (m.cout, ho, wo)
            self.keep.append(dm)
        joined = {k: (torch.cat(v) if v and v[0] is not None else None) for k, v in consts.items()}
        name = "+".join(m.name for m in members)
        if mixed:
            self._add(name, B.relay_fused_conv2d_combined_windows,
                      (d, src, src.stride(2), wp, joined["bias"], joined["scale"], joined["shift"],
                       [m.cout for m in members], ys, [y.stride(2) for y in ys],
                       [B.WINDOW_FULL if m.r == op0.r else B.WINDOW_CENTRE for m in members],
                       [1 if m.relu else 0 for m in members]))
        else:
            self._add(name, B.relay_fused_conv2d_combined,
                      (d, src, src.stride(2), wp, joined["bias"], joined["scale"], joined["shift"],
                       [m.cout for m in members], ys, [y.stride(2) for y in ys]))
        self.keep += [wp, d, joined]

    def _workspace(self, d):
        """Zeroed scratch of a conv whose reduction the library splits over workgroups (the deep
        layers at small batch), one buffer per conv so that convs on forked streams cannot share one."""
        need = B.relay_workspace_bytes(d)
        if need == 0:
            return None
        ws = torch.zeros(need, dtype=torch.uint8, device=self.dev)
        self.keep.append(ws)
        return ws

    def _fold(self, op, p, wsrc, cin_l):
        """Axis scale folding: multiplies the OIHW filters on the device by the conv's batch-norm
        scale, in place, and returns the bias that replaces "add bias, scale, shift"."""
        sc, sf = self._f32(p["scale"]), self._f32(p["shift"])
        B.relay_fold_scale_axis(self.dtype, op.cout, cin_l, op.r * op.r, B.FOLD_OUT, wsrc, sc, wsrc)
        folded = torch.empty(op.cout, dtype=torch.float32, device=self.dev)
        B.relay_fold_bias(op.cout, self._f32(p.get("bias")), sc, sf, folded)
        self.keep.append(folded)
        return folded

    def _f32(self, a):
        if a is None:
            return None
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev)
        self.keep.append(t)
        return t

    def _unfused_tail(self, op, p, cur, npix, c, res):
        """bias add, scale/shift, residual add, relu as separate launches, each into a new tensor."""
        def step(tag, ew, p0, p1, other):
            nonlocal cur
            nxt = torch.empty_like(cur)
            self._add(f"{op.name}.{tag}", B.relay_elementwise_f16, (ew, npix, c, cur, p0, p1, other, nxt))
            cur = nxt
        if p.get("bias") is not None:
            step("bias_add", B.EW_BIAS_ADD, self._f32(p["bias"]), None, None)
        if p.get("scale") is not None:
            step("scale_shift", B.EW_SCALE_SHIFT, self._f32(p["scale"]), self._f32(p["shift"]), None)
        if res is not None:
            step("add", B.EW_ADD, None, None, res)
        if op.relu:
            step("relu", B.EW_RELU, None, None, None)
        return cur

    def _add(self, name, fn, args):
        self.calls.append((fn, args))
        self.call_names.append(name)

    def load_input(self, x_nchw: np.ndarray) -> None:
        self.x_nchw.copy_(torch.from_numpy(np.ascontiguousarray(x_nchw)).to(self.dev))

    def run(self) -> None:
        """Enqueue the whole network on the current stream (layout conversion included).

        A conv whose output is only used as a later residual (the 1x1 shortcut of a ResNet
        block) is launched on a side stream between two events, so that it overlaps the block's
        first conv: both read the block input, neither reads the other.  The fork event is
        recorded BEFORE that first conv is enqueued, so the side stream waits only for the
        producer of the block input."""
        if not self.side_calls:
            for fn, args in self.calls:
                fn(*args)
            return
        main = torch.cuda.current_stream()
        pending = fork = None
        for i, (fn, args) in enumerate(self.calls):
            if i + 1 in self.side_calls:      # the next call runs beside this one
                fork = torch.cuda.Event()
                fork.record(main)
            if i in self.side_calls:
                self.side.wait_event(fork)
                with torch.cuda.stream(self.side):
                    fn(*args)
                    pending = torch.cuda.Event()
                    pending.record(self.side)
                continue
            if pending is not None and i in self.join_before:
                main.wait_event(pending)
                pending = None
            fn(*args)
        if pending is not None:
            main.wait_event(pending)

    def capture(self) -> None:
        """Record run() into a HIP graph (kernel launches only; nothing in it clears memory)."""
        self.run()
        torch.cuda.synchronize(self.dev)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.run()
        self.graph = g

    def replay(self) -> None:
        self.graph.replay()

    def tensor(self, name: str) -> np.ndarray:
        """Download a named tensor as NCHW with the logical channel count."""
        if name == "x":
            return self.x_nchw.cpu().numpy()
        if name not in self.bufs:
            raise KeyError(f"{name} is not stored: its producer runs fused with the operator that reads it")
        c, _, _ = self.shape[name]
        t = self.bufs[name][..., :c].permute(0, 3, 1, 2).contiguous().cpu().numpy()
        return t

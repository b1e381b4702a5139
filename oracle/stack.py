"""CPU oracle -- TEST INFRASTRUCTURE ONLY: a whole network run through the oracle operators.

The tensor handed from one primitive function to the next is stored in the working type
(fp16, fp32 or int8), so every layer output is narrowed before the next layer reads it;
that is the model's semantics (paper, Section 3.3: operators are called one after another
on preallocated buffers), not an approximation.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import (fused_conv2d, fused_dense, fused_dwconv2d, global_avgpool, maxpool2d,
               qconv2d_requant, _narrow)


def run_float(ops, params: List[dict], x: np.ndarray, out_dtype: str = "f16") -> Dict[str, np.ndarray]:
    """Returns every named tensor (NCHW; dense/pool outputs [N, C]) in the working dtype."""
    t: Dict[str, np.ndarray] = {"x": x}
    for op, p in zip(ops, params):
        src = t[op.src]
        if op.kind == "conv":
            t[op.dst] = fused_conv2d(src, p["w"], stride=(op.stride, op.stride), pad=(op.pad, op.pad),
                                     bias=p.get("bias"), scale=p.get("scale"), shift=p.get("shift"),
                                     residual=t[op.res] if op.res else None, relu_flag=op.relu,
                                     out_dtype=out_dtype)
        elif op.kind == "dwconv":
            t[op.dst] = fused_dwconv2d(src, p["w"], stride=(op.stride, op.stride), pad=(op.pad, op.pad),
                                       bias=p.get("bias"), scale=p.get("scale"), shift=p.get("shift"),
                                       relu_flag=op.relu, out_dtype=out_dtype)
        elif op.kind == "maxpool":
            t[op.dst] = _narrow(maxpool2d(src, op.r, op.stride, op.pad), out_dtype)
        elif op.kind == "avgpool":
            t[op.dst] = _narrow(global_avgpool(src), out_dtype)
        elif op.kind == "dense":
            # a dense layer over a [C, H, W] tensor reads it flattened in (channel, row, column) order
            t[op.dst] = fused_dense(src.reshape(src.shape[0], -1), p["w"], bias=p.get("bias"), relu_flag=op.relu,
                                    out_dtype=out_dtype)
        elif op.kind == "concat":
            t[op.dst] = np.concatenate([t[s] for s in op.srcs], axis=1)   # channel axis of NCHW
        else:
            raise ValueError(op.kind)
    return t


def run_quantized(ops, params: List[dict], shifts: List[dict], x: np.ndarray) -> Dict[str, np.ndarray]:
    """int8 network: every conv is qconv2d_requant with that layer's (out_rshift, residual_lshift)."""
    t: Dict[str, np.ndarray] = {"x": x}
    for op, p, sh in zip(ops, params, shifts):
        src = t[op.src]
        if op.kind == "conv":
            t[op.dst] = qconv2d_requant(src, p["w"], stride=(op.stride, op.stride), pad=(op.pad, op.pad),
                                        bias=p.get("bias"), residual=t[op.res] if op.res else None,
                                        residual_lshift=sh.get("l", 0), out_rshift=sh["s"],
                                        relu_flag=op.relu)
        elif op.kind == "maxpool":
            # max of int8 values is exact in double
            t[op.dst] = maxpool2d(src, op.r, op.stride, op.pad).astype(np.int8)
        else:
            raise ValueError(op.kind)
    return t


def run_float_unfused(ops, params: List[dict], x: np.ndarray) -> Dict[str, np.ndarray]:
    """The same network with operator fusion switched off: every elementwise operator behind a
    contraction is an operator call of its own whose result is stored in fp16 before the next one
    reads it (paper Section 5.2 compares fusion against such a pipeline)."""
    import oracle as O
    h = O.cast_f16
    t: Dict[str, np.ndarray] = {"x": x}
    for op, p in zip(ops, params):
        src = t[op.src]
        if op.kind in ("conv", "dwconv", "dense"):
            if op.kind == "conv":
                y = h(O.conv2d(src, p["w"], (op.stride, op.stride), (op.pad, op.pad)))
            elif op.kind == "dwconv":
                y = h(O.dwconv2d(src, p["w"], (op.stride, op.stride), (op.pad, op.pad)))
            else:
                y = h(O.dense(src.reshape(src.shape[0], -1), p["w"]))
            if p.get("bias") is not None:
                y = h(O.bias_add(y.astype(np.float64), p["bias"]))
            if p.get("scale") is not None:
                y = h(O.scale_shift(y.astype(np.float64), p["scale"], p["shift"]))
            if op.res:
                y = h(O.add(y.astype(np.float64), t[op.res]))
            if op.relu:
                y = h(O.relu(y.astype(np.float64)))
            t[op.dst] = y
        elif op.kind == "maxpool":
            t[op.dst] = _narrow(maxpool2d(src, op.r, op.stride, op.pad), "f16")
        elif op.kind == "avgpool":
            t[op.dst] = _narrow(global_avgpool(src), "f16")
        else:
            raise ValueError(op.kind)
    return t

"""Compile-time half of the quantization flow (paper Section 4.2; axis scale folding from
Section 4.4) for a stack of fused conv layers: calibrate power-of-two ranges on a float run,
fold the batch-norm scale into the filters, realize int8 filters / int32 biases / shifts.

Argument marshalling only: the float run (FusedNet in fp16), the ranges
(relay_calibrate_pow2_range) and the realization of every conv (relay_realize_conv) execute in
the library's kernels; this module uploads parameters, calls the entry points and reads the few
result words back.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np
import torch

from . import binding as B
from .stack import FusedNet


def calibrate(ops, params: Sequence[dict], x_f16: np.ndarray, global_scale: bool = False,
              device: str = "cuda:0") -> Dict[str, float]:
    """Ranges of the input and of every layer output: the smallest power of two not exceeded on the
    calibration batch (one common range when global_scale, the paper's first strategy)."""
    n, c, h, w = x_f16.shape
    net = FusedNet(ops, params, n, h, w, "f16", in_channels=c, device=device, fuse_pool=False)   # every tensor stays readable
    net.load_input(x_f16)
    net.run()
    names = ["x"] + [op.dst for op in ops]
    rho_d = torch.empty(len(names), dtype=torch.float32, device=device)
    cell = torch.empty(1, dtype=torch.int32, device=device)
    for i, name in enumerate(names):
        t = net.x_nchw if name == "x" else net.bufs[name]         # (channel padding holds zeros: no effect on a maximum)
        B.relay_calibrate_pow2_range(B.RELAY_F16, t.numel(), t, rho_d[i:i + 1], cell)
    vals = rho_d.cpu().tolist()
    if global_scale:
        vals = [max(vals)] * len(vals)
    return dict(zip(names, vals))


def realize(ops, params: Sequence[dict], rho: Dict[str, float], device: str = "cuda:0") -> Tuple[List[dict], List[dict]]:
    """int8 filters (scale folded in), int32 biases, and the (out_rshift, residual_lshift) of every
    conv, all computed by relay_realize_conv.  Raises when a shift or a bias leaves its range."""
    def up(a):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    qparams: List[dict] = []
    shifts: List[dict] = []
    for op, p in zip(ops, params):
        if op.kind != "conv":
            if op.kind != "maxpool":
                raise ValueError(f"no quantized form of {op.kind}")
            qparams.append({})
            shifts.append({})
            continue
        w = up(p["w"])
        k, per_k = w.shape[0], w[0].numel()
        bias, scale, shift = up(p.get("bias")), up(p.get("scale")), up(p.get("shift"))
        wq = torch.empty(w.shape, dtype=torch.int8, device=device)
        bq = torch.empty(k, dtype=torch.int32, device=device) if (bias is not None or shift is not None) else None
        out = torch.empty(4, dtype=torch.int32, device=device)
        ws = torch.empty(k * per_k * 4 + 16, dtype=torch.uint8, device=device)
        B.relay_realize_conv(k, per_k, w, bias, scale, shift, rho[op.src], rho[op.dst],
                             rho[op.res] if op.res else 0.0, wq, bq, out, ws)
        _, s, l, status = out.cpu().tolist()
        if status:
            raise ValueError(f"{op.name}: realization failed (status bits {status}: shifts s={s} l={l})")
        q = {"w": wq.cpu().numpy()}
        if bq is not None:
            q["bias"] = bq.cpu().numpy()
        qparams.append(q)
        shifts.append({"s": int(s), "l": int(l)})
    return qparams, shifts


def quantize_input(x_f16: np.ndarray, rho_x: float, device: str = "cuda:0") -> np.ndarray:
    xd = torch.from_numpy(np.ascontiguousarray(x_f16)).to(device)
    xq = torch.empty(x_f16.shape, dtype=torch.int8, device=device)
    B.relay_quantize(x_f16.size, B.RELAY_F16, xd, rho_x, 8, 1, B.ROUND_NEAREST, 0, xq)
    return xq.cpu().numpy()

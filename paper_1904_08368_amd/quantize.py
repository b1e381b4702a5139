"""Compile-time half of the quantization flow (paper Section 4.2; axis scale folding from
Section 4.4) for a stack of fused conv layers: calibrate power-of-two ranges on a float run,
fold the batch-norm scale into the filters, realize int8 filters / int32 biases / shifts.
The float run and the filter quantization execute in the library's kernels (FusedNet in fp16,
relay_quantize); what is left on the host is a handful of scalars per layer.

Scheme (8-bit signed, power-of-two ranges, "no overflow" calibration): a tensor with range rho
holds code * rho / 2^7.  One count of a conv's int32 accumulator is worth rho_x * rho_w / 2^14,
which fixes the realized bias and the two shifts of relay_qconv2d_requant.
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence, Tuple

import numpy as np
import torch

from . import binding as B
from .stack import FusedNet


def _range_of(max_abs: float) -> float:
    return 2.0 ** math.ceil(math.log2(max_abs)) if max_abs > 0 else 2.0 ** -20


def calibrate(ops, params: Sequence[dict], x_f16: np.ndarray, global_scale: bool = False,
              device: str = "cuda:0") -> Dict[str, float]:
    """Ranges of the input and of every layer output: the smallest power of two not exceeded on the
    calibration batch (one common range when global_scale, the paper's first strategy)."""
    n, c, h, w = x_f16.shape
    net = FusedNet(ops, params, n, h, w, "f16", in_channels=c, device=device, fuse_pool=False)   # every tensor is read back
    net.load_input(x_f16)
    net.run()
    torch.cuda.synchronize()
    names = ["x"] + [op.dst for op in ops]
    rho = {}
    for name in names:
        rho[name] = _range_of(float(np.abs(net.tensor(name).astype(np.float32)).max()))
    if global_scale:
        top = max(rho.values())
        rho = {k: top for k in rho}
    return rho


def realize(ops, params: Sequence[dict], rho: Dict[str, float], device: str = "cuda:0") -> Tuple[List[dict], List[dict]]:
    """int8 filters (scale folded in, quantized by relay_quantize), int32 biases, and the
    (out_rshift, residual_lshift) of every conv.  Raises when a shift leaves its range."""
    qparams: List[dict] = []
    shifts: List[dict] = []
    for op, p in zip(ops, params):
        if op.kind != "conv":
            if op.kind != "maxpool":
                raise ValueError(f"no quantized form of {op.kind}")
            qparams.append({})
            shifts.append({})
            continue
        w = np.asarray(p["w"], dtype=np.float64)
        if p.get("scale") is not None:                            # axis scale folding
            w = w * np.asarray(p["scale"], dtype=np.float64)[:, None, None, None]
        w32 = np.ascontiguousarray(w, dtype=np.float32)
        rho_w = _range_of(float(np.abs(w32).max()))
        wd = torch.from_numpy(w32).to(device)
        wq = torch.empty(w32.shape, dtype=torch.int8, device=device)
        B.relay_quantize(w32.size, B.RELAY_F32, wd, rho_w, 8, 1, B.ROUND_NEAREST, 0, wq)
        count = rho[op.src] * rho_w / 16384.0                     # real value of one accumulator count
        q = {"w": wq.cpu().numpy()}
        add = p.get("shift") if p.get("shift") is not None else p.get("bias")
        if add is not None:
            b = np.floor(np.asarray(add, dtype=np.float64) / count + 0.5)
            if np.abs(b).max() >= 2 ** 31:
                raise ValueError(f"{op.name}: realized bias does not fit int32")
            q["bias"] = b.astype(np.int32)
        s = math.log2(rho[op.dst] / 128.0 / count)
        l = math.log2(rho[op.res] / 128.0 / count) if op.res else 0.0
        if s != int(s) or not 0 <= s <= 31 or l != int(l) or not 0 <= l <= 23:
            raise ValueError(f"{op.name}: shifts s={s} l={l} outside what the quantized conv takes")
        qparams.append(q)
        shifts.append({"s": int(s), "l": int(l)})
    return qparams, shifts


def quantize_input(x_f16: np.ndarray, rho_x: float, device: str = "cuda:0") -> np.ndarray:
    xd = torch.from_numpy(np.ascontiguousarray(x_f16)).to(device)
    xq = torch.empty(x_f16.shape, dtype=torch.int8, device=device)
    B.relay_quantize(x_f16.size, B.RELAY_F16, xd, rho_x, 8, 1, B.ROUND_NEAREST, 0, xq)
    return xq.cpu().numpy()

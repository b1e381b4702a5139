"""CPU oracle -- TEST INFRASTRUCTURE ONLY: calibration and realization of the paper's generic
quantization flow (Section 4.2) for a stack of fused conv layers, plus axis scale folding
(Section 4.4), in plain numpy.

Flow (one reading of the section; its choices are listed in the design notes):
  annotate   every conv input, weight tensor and conv output is to be quantized to 8 bits
             (beta = 8, sigma = 1) with a power-of-two range rho;
  calibrate  "no overflow": rho of a tensor is the smallest power of two that its largest
             magnitude on the calibration batch does not exceed (optionally one global rho
             for all activations, the paper's first strategy; weights always per layer);
  fold       the per-channel scale behind a conv moves into its weights (axis scale folding):
             w'[k] = w[k] * scale[k]; the shift stays as a bias;
  realize    x_q = Q(x, rho_x); w_q = Q(w', rho_w); with real = code * rho / 2^7 the int32
             accumulator of a conv is in units of rho_x * rho_w / 2^14, hence
               bias_q[k] = round((bias[k] * scale[k] + shift[k]) * 2^14 / (rho_x * rho_w))
               s = log2(2^7 * rho_y / (rho_x * rho_w))        (output requantization shift)
               l = log2(2^7 * rho_r / (rho_x * rho_w))        (residual alignment shift)
             all integers because every rho is a power of two.
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence

import numpy as np

from . import quant as OQ


def pow2_range(max_abs: float) -> float:
    """Smallest power of two >= max_abs (a tensor of zeros gets 2^-20, any value would do)."""
    if not max_abs > 0:
        return 2.0 ** -20
    return 2.0 ** math.ceil(math.log2(max_abs))


def calibrate(ops, tensors: Dict[str, np.ndarray], global_scale: bool = False) -> Dict[str, float]:
    """rho per activation tensor from a float run of the network on the calibration batch."""
    names = ["x"] + [op.dst for op in ops]
    rho = {n: pow2_range(float(np.max(np.abs(tensors[n].astype(np.float64))))) for n in names}
    if global_scale:
        g = max(rho.values())
        rho = {n: g for n in names}
    return rho


def fold_scale(w: np.ndarray, scale) -> np.ndarray:
    """Axis scale folding: the per-output-channel multiply behind a conv becomes part of its filters."""
    w = np.asarray(w, dtype=np.float64)
    if scale is None:
        return w
    return w * np.asarray(scale, dtype=np.float64).reshape(-1, 1, 1, 1)


def realize(ops, params: Sequence[dict], rho: Dict[str, float]):
    """Returns (qparams, shifts): int8 filters and int32 biases per conv, (s, l) per layer."""
    qparams: List[dict] = []
    shifts: List[dict] = []
    for op, p in zip(ops, params):
        if op.kind != "conv":
            assert op.kind == "maxpool"          # max commutes with a positive scale: the range passes through
            assert rho[op.dst] <= rho[op.src]
            qparams.append({})
            shifts.append({})
            continue
        wf = fold_scale(p["w"], p.get("scale")).astype(np.float32)
        rho_w = pow2_range(float(np.max(np.abs(wf))))
        wq = OQ.Q(wf, rho_w, 8, 1)
        unit = rho[op.src] * rho_w / 2.0 ** 14          # real value of one accumulator count
        q = {"w": wq}
        # additive term of the float tail in its order bias -> scale, shift:
        # (acc + bias) * scale + shift = acc * scale + (bias * scale + shift)
        shift = None
        if p.get("bias") is not None:
            shift = np.asarray(p["bias"], dtype=np.float64)
        if p.get("scale") is not None:
            shift = (shift if shift is not None else 0.0) * np.asarray(p["scale"], dtype=np.float64) \
                + np.asarray(p["shift"], dtype=np.float64)
        if shift is not None:
            b = np.floor(np.asarray(shift, dtype=np.float64) / unit + 0.5)
            assert np.all(np.abs(b) < 2 ** 31)
            q["bias"] = b.astype(np.int32)
        s = math.log2(rho[op.dst] / 2.0 ** 7 / unit)
        assert s == int(s) and 0 <= s <= 31, (op.name, s)
        sh = {"s": int(s), "l": 0}
        if op.res:
            l = math.log2(rho[op.res] / 2.0 ** 7 / unit)
            assert l == int(l) and 0 <= l <= 23, (op.name, l)
            sh["l"] = int(l)
        qparams.append(q)
        shifts.append(sh)
    return qparams, shifts


def dequantize(codes: np.ndarray, rho: float) -> np.ndarray:
    return codes.astype(np.float64) * rho / 2.0 ** 7

"""Seeded synthetic inputs and parameters (host numpy arrays, NCHW / OIHW).

The paper times its vision models on random inputs (Section 5.1, methodology), so
random tensors of the real shapes stand in for images and trained weights.  This
module only draws numbers; it performs none of the method's arithmetic and is the
one module the CPU oracle's tests and the GPU path's tests both import.

Seed of a tensor group = BASE_SEED + 1000*config + layer_index.
"""
from __future__ import annotations

import math
from typing import Dict, List

import numpy as np

from .nets import Op

BASE_SEED = 190408368


def rng_for(config: int, layer: int) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + 1000 * config + layer)


def fan_in(op: Op) -> int:
    if op.kind == "dwconv":
        return op.r * op.r
    if op.kind == "dense":
        return op.cin
    return op.cin * op.r * op.r


def default_out_rshift(k_red: int) -> int:
    """Per-layer right shift for a conv fed with uniform int8 values: 7 + ceil(log2(K)/2)."""
    return 7 + int(math.ceil(math.log2(k_red) / 2.0))


def chain_out_rshift(k_red: int) -> int:
    """Right shift of a conv inside a chained int8 network: round(log2(sigma_w * sqrt(K))) with
    sigma_w = 73.3, the standard deviation of U{-127..127}.  The accumulator of a conv over
    zero-mean weights has rms = sigma_w * sqrt(K) * rms(x), so this shift hands the next layer
    activations of about the same rms as it received (a closed-form stand-in for the paper's
    calibration sweep, which needs real activations)."""
    return int(round(math.log2(73.3 * math.sqrt(k_red))))


def chain_shifts(ops: List[Op]) -> List[dict]:
    """Per-op {'s': out_rshift, 'l': residual_lshift} for a chained int8 network; the residual
    carries the output's scale, so l = s."""
    out = []
    for op in ops:
        if op.kind == "conv":
            s = chain_out_rshift(op.cin * op.r * op.r)
            out.append({"s": s, "l": s if op.res else 0})
        else:
            out.append({})
    return out


def image(config: int, n: int, c: int, h: int, w: int, mode: str) -> np.ndarray:
    """Network input, NCHW.  mode: 'f32' U[-1,1) | 'f16' N(0,1) rounded to fp16 | 'i8' U{-127..127}."""
    g = rng_for(config, 999)
    if mode == "f32":
        return g.uniform(-1.0, 1.0, size=(n, c, h, w)).astype(np.float32)
    if mode == "f16":
        return g.standard_normal(size=(n, c, h, w), dtype=np.float32).astype(np.float16)
    if mode == "i8":
        return g.integers(-127, 128, size=(n, c, h, w), dtype=np.int64).astype(np.int8)
    raise ValueError(mode)


def activation(config: int, layer: int, shape, mode: str) -> np.ndarray:
    """A fresh per-layer input of a given shape (for per-layer measurements and tests)."""
    g = rng_for(config, 500 + layer)
    if mode == "f32":
        return g.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    if mode == "f16":
        return g.standard_normal(size=shape, dtype=np.float32).astype(np.float16)
    if mode == "i8":
        return g.integers(-127, 128, size=shape, dtype=np.int64).astype(np.int8)
    raise ValueError(mode)


def layer_params(op: Op, config: int, layer: int, mode: str) -> Dict[str, np.ndarray]:
    """Parameters of one fused primitive function.

    float modes: w ~ N(0, 2/fan_in) (He-normal) in the working dtype, bias ~ N(0, 0.1^2),
    bn scale ~ N(1, 0.1^2), bn shift ~ N(0, 0.1^2) (fp32).  mode 'f32u' draws w ~ U[-1,1)
    as the smallest configuration asks.  'i8': w ~ U{-127..127}, no bias.
    """
    g = rng_for(config, layer)
    p: Dict[str, np.ndarray] = {}
    if op.kind == "dwconv":
        wshape = (op.cin, op.r, op.r)
    elif op.kind == "dense":
        wshape = (op.cout, op.cin)
    elif op.kind == "conv":
        wshape = (op.cout, op.cin, op.r, op.r)
    else:
        return p
    if mode == "i8":
        p["w"] = g.integers(-127, 128, size=wshape, dtype=np.int64).astype(np.int8)
        return p
    if mode == "f32u":
        p["w"] = g.uniform(-1.0, 1.0, size=wshape).astype(np.float32)
    else:
        std = math.sqrt(2.0 / fan_in(op))
        w = (g.standard_normal(size=wshape, dtype=np.float32) * np.float32(std))
        p["w"] = w.astype(np.float16 if mode == "f16" else np.float32)
    if op.bias:
        p["bias"] = (g.standard_normal(size=(op.cout,), dtype=np.float32) * np.float32(0.1))
    if op.bn:
        p["scale"] = (np.float32(1.0) + g.standard_normal(size=(op.cout,), dtype=np.float32) * np.float32(0.1))
        p["shift"] = (g.standard_normal(size=(op.cout,), dtype=np.float32) * np.float32(0.1))
    return p


def net_params(ops: List[Op], config: int, mode: str) -> List[Dict[str, np.ndarray]]:
    return [layer_params(op, config, i, mode) for i, op in enumerate(ops)]

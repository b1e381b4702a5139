"""CPU oracle -- TEST INFRASTRUCTURE ONLY: the two graph-level rewrites of paper Section 4.4
that change which kernels run without changing what they compute.

Axis scale folding: a multiplication by a per-channel constant next to a convolution is moved
into the convolution's constant filters, so no multiplication is left at run time.
    after the conv  (axis "out"):  conv(x, w)[:, k] * s[k]  ==  conv(x, w')   with w'[k, c, r, q] = w[k, c, r, q] * s[k]
    before the conv (axis "in"):   conv(x * s[c], w)        ==  conv(x, w')   with w'[k, c, r, q] = w[k, c, r, q] * s[c]
(zero padding commutes with the scaling, so the second identity holds at the border too.)

Parallel convolution combination: convolutions that read the same tensor with the same window
become one convolution whose filters are the members' filters stacked along the output-channel
axis; every member's result is a channel slice of the combined result.  Output channels of a
convolution do not interact, so the slices equal the members' own results exactly.

Everything here is written from those definitions with numpy in fp64; nothing is shared with
the GPU library.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

from . import _narrow, fused_conv2d


def fold_scale_axis(w: np.ndarray, scale, axis: str, out_dtype: str) -> np.ndarray:
    """w: OIHW filters.  Product in fp64, narrowed once to the working type."""
    w64 = np.asarray(w, dtype=np.float64)
    s = np.asarray(scale, dtype=np.float64)
    if axis == "out":
        assert s.shape == (w64.shape[0],)
        out = w64 * s[:, None, None, None]
    elif axis == "in":
        assert s.shape == (w64.shape[1],)
        out = w64 * s[None, :, None, None]
    else:
        raise ValueError(axis)
    return _narrow(out, out_dtype)


def fold_bn_into_conv(p: Dict[str, np.ndarray], out_dtype: str) -> Dict[str, np.ndarray]:
    """Parameters of conv -> (+bias) -> *scale + shift rewritten as conv' -> +bias' with
    w' = w * scale[k] and bias' = bias * scale + shift (fp64, narrowed to fp32 like any bias)."""
    if p.get("scale") is None:
        return dict(p)
    sc = np.asarray(p["scale"], dtype=np.float64)
    b = np.asarray(p["bias"], dtype=np.float64) if p.get("bias") is not None else 0.0
    q = {k: v for k, v in p.items() if k not in ("scale", "shift", "bias")}
    q["w"] = fold_scale_axis(p["w"], sc, "out", out_dtype)
    q["bias"] = (b * sc + np.asarray(p["shift"], dtype=np.float64)).astype(np.float32)
    return q


def embed_centre(w: np.ndarray, r: int) -> np.ndarray:
    """A 1x1 filter bank [K, C, 1, 1] as an r x r one (r odd) that is zero except at the centre tap.
    With the same stride, conv(x, w, pad 0) == conv(x, embed_centre(w, r), pad r // 2): output pixel
    (p, q) of the padded r x r window starts at input (p*stride - r//2, q*stride - r//2), so its
    centre tap reads input (p*stride, q*stride), the pixel the 1x1 convolution reads, and every
    other tap is multiplied by zero."""
    w = np.asarray(w)
    assert w.ndim == 4 and w.shape[2:] == (1, 1) and r % 2 == 1
    out = np.zeros(w.shape[:2] + (r, r), dtype=w.dtype)
    out[:, :, r // 2, r // 2] = w[:, :, 0, 0]
    return out


def signature(op) -> tuple:
    """What two convolutions must share, besides their input, to be combined: the window and
    the elementwise tail fused behind them (so the per-channel constants can be stacked too)."""
    return (op.src, op.cin, op.r, op.stride, op.pad, bool(op.bias), bool(op.bn), bool(op.relu))


def combine_groups(ops: Sequence, windows: bool = False) -> List[List[int]]:
    """Indices of the convs to merge, one list per combined conv (lists of length >= 2, members
    in program order, lists ordered by first member).  A conv with a residual operand is left
    alone: its tail reads a second tensor.

    windows=True: convs over the same input with the same stride whose windows are odd and padded
    by half their size are also merged when one kind is 1x1 and the other the widest window of
    the set (embed_centre), whatever their relu; the wide members are listed first."""
    if not windows:
        found: Dict[tuple, List[int]] = {}
        for i, op in enumerate(ops):
            if op.kind == "conv" and not op.res:
                found.setdefault(signature(op), []).append(i)
        return sorted((g for g in found.values() if len(g) >= 2), key=lambda g: g[0])
    convs = [i for i, op in enumerate(ops) if op.kind == "conv" and not op.res]
    is_centred = lambda op: op.r % 2 == 1 and op.pad == op.r // 2
    out: List[List[int]] = []
    # convs that are not centred windows, and centred ones of middle sizes, merge as without `windows`
    buckets: Dict[tuple, List[int]] = {}
    for i in convs:
        op = ops[i]
        buckets.setdefault((op.src, op.cin, op.stride, bool(op.bias), bool(op.bn)) if is_centred(op) else (None,) + signature(op), []).append(i)
    for key, members in buckets.items():
        if key[0] is None:
            if len(members) >= 2:
                out.append(members)
            continue
        widest = max(ops[i].r for i in members)
        if widest == 1:
            for relu in (True, False):
                same = [i for i in members if bool(ops[i].relu) == relu]
                if len(same) >= 2:
                    out.append(same)
            continue
        merged = [i for i in members if ops[i].r == widest] + [i for i in members if ops[i].r == 1]
        if len(merged) >= 2:
            out.append(merged)
        for r in sorted({ops[i].r for i in members} - {1, widest}):
            for relu in (True, False):
                same = [i for i in members if ops[i].r == r and bool(ops[i].relu) == relu]
                if len(same) >= 2:
                    out.append(same)
    return sorted(out, key=min)


def combined_conv2d_windows(x, ops: Sequence, members: Sequence[Dict[str, np.ndarray]], out_dtype: str = "f16") -> List[np.ndarray]:
    """A group found with windows=True evaluated as ONE conv: the 1x1 members' filters embedded at the
    centre of the widest window, filters and per-channel constants stacked, no relu in the conv;
    then every member's channel slice gets that member's relu (relu of the narrowed value equals the
    narrowed relu: narrowing is monotone and keeps zero)."""
    r = max(op.r for op in ops)
    ws = [np.asarray(m["w"]) if op.r == r else embed_centre(m["w"], r) for op, m in zip(ops, members)]
    def stack(key):
        if members[0].get(key) is None:
            assert all(m.get(key) is None for m in members)
            return None
        return np.concatenate([np.asarray(m[key]) for m in members], axis=0)
    st = ops[0].stride
    y = fused_conv2d(x, np.concatenate(ws, axis=0), stride=(st, st), pad=(r // 2, r // 2), bias=stack("bias"),
                     scale=stack("scale"), shift=stack("shift"), relu_flag=False, out_dtype=out_dtype)
    outs, k0 = [], 0
    for op, m in zip(ops, members):
        k = m["w"].shape[0]
        part = y[:, k0:k0 + k]
        outs.append(np.maximum(part, 0).astype(part.dtype) if op.relu else part)
        k0 += k
    return outs


def combined_conv2d(x, members: Sequence[Dict[str, np.ndarray]], *, stride, pad, relu_flag,
                    out_dtype: str = "f16") -> List[np.ndarray]:
    """The combined conv evaluated as ONE conv over stacked filters and stacked per-channel
    constants, then sliced; returns the members' outputs in order."""
    def stack(key):
        if members[0].get(key) is None:
            assert all(m.get(key) is None for m in members)
            return None
        return np.concatenate([np.asarray(m[key]) for m in members], axis=0)
    y = fused_conv2d(x, stack("w"), stride=stride, pad=pad, bias=stack("bias"), scale=stack("scale"),
                     shift=stack("shift"), relu_flag=relu_flag, out_dtype=out_dtype)
    outs, k0 = [], 0
    for m in members:
        k = m["w"].shape[0]
        outs.append(y[:, k0:k0 + k])
        k0 += k
    return outs

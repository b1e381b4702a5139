"""Layer tables of the vision networks the paper evaluates (Section 5, "vision" workloads).

The paper names ResNet-18 and MobileNet but does not list their layers; the tables
here are the standard published definitions of those architectures (shapes only).
A network is a list of op records over named tensors.  A record holds shapes and
which elementwise operators are fused behind the contraction -- no arithmetic.

Every conv record describes one *fused primitive function* in the sense of the
paper's operator-fusion section: the contraction plus the elementwise operators
that post-dominate it (bias add, folded batch-norm scale/shift, residual add, relu).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional


@dataclass(frozen=True)
class Op:
    kind: str                 # "conv" | "dwconv" | "dense" | "maxpool" | "avgpool" | "concat"
    name: str
    src: str                  # input tensor name
    dst: str                  # output tensor name
    cin: int = 0
    cout: int = 0
    r: int = 1                # square kernel
    stride: int = 1
    pad: int = 0
    bias: bool = False
    bn: bool = False
    relu: bool = False
    res: Optional[str] = None  # tensor added before relu (residual), or None
    srcs: tuple = ()          # concat only: the tensors joined along the channel axis, in order (src = srcs[0])


def conv(name, src, dst, cin, cout, r, stride, pad, *, bn=True, relu=True, res=None, bias=False):
    return Op("conv", name, src, dst, cin, cout, r, stride, pad, bias, bn, relu, res)


def resnet18(with_dense: bool = True) -> List[Op]:
    """20 fused convs (+ maxpool, global average pool and the 512->1000 dense)."""
    ops: List[Op] = [
        conv("conv1", "x", "c1", 3, 64, 7, 2, 3),
        Op("maxpool", "maxpool", "c1", "s1.in", cin=64, cout=64, r=3, stride=2, pad=1),
    ]
    cin = 64
    cur = "s1.in"
    for stage, cout in enumerate((64, 128, 256, 512), start=1):
        for blk in range(2):
            stride = 2 if (stage > 1 and blk == 0) else 1
            p = f"l{stage}.b{blk}"
            ops.append(conv(f"{p}.conv1", cur, f"{p}.t", cin, cout, 3, stride, 1))
            if stride != 1 or cin != cout:
                ops.append(conv(f"{p}.down", cur, f"{p}.d", cin, cout, 1, stride, 0, relu=False))
                shortcut = f"{p}.d"
            else:
                shortcut = cur
            ops.append(conv(f"{p}.conv2", f"{p}.t", f"{p}.out", cout, cout, 3, 1, 1, res=shortcut))
            cur = f"{p}.out"
            cin = cout
    if with_dense:
        ops.append(Op("avgpool", "avgpool", cur, "pooled", cin=512, cout=512))
        ops.append(Op("dense", "fc", "pooled", "logits", cin=512, cout=1000, bias=True))
    return ops


MOBILENET_V1_BLOCKS = (
    # (cin, cout, depthwise stride)
    (32, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1), (256, 512, 2),
    (512, 512, 1), (512, 512, 1), (512, 512, 1), (512, 512, 1), (512, 512, 1),
    (512, 1024, 2), (1024, 1024, 1),
)


def mobilenet_v1(with_dense: bool = True) -> List[Op]:
    """3x3/s2 stem, 13 depthwise-separable blocks, global average pool, 1024->1000 dense."""
    ops: List[Op] = [conv("stem", "x", "b0.out", 3, 32, 3, 2, 1)]
    cur = "b0.out"
    for i, (cin, cout, s) in enumerate(MOBILENET_V1_BLOCKS, start=1):
        ops.append(Op("dwconv", f"b{i}.dw", cur, f"b{i}.t", cin=cin, cout=cin, r=3, stride=s,
                      pad=1, bn=True, relu=True))
        ops.append(conv(f"b{i}.pw", f"b{i}.t", f"b{i}.out", cin, cout, 1, 1, 0))
        cur = f"b{i}.out"
    if with_dense:
        ops.append(Op("avgpool", "avgpool", cur, "pooled", cin=1024, cout=1024))
        ops.append(Op("dense", "fc", "pooled", "logits", cin=1024, cout=1000, bias=True))
    return ops


def basic_block(c: int = 64) -> List[Op]:
    """One ResNet basic block at constant width (the two-conv diamond with a residual edge)."""
    return [
        conv("blk.conv1", "x", "blk.t", c, c, 3, 1, 1),
        conv("blk.conv2", "blk.t", "blk.out", c, c, 3, 1, 1, res="x"),
    ]


# VGG-16 (configuration D of its paper): 3x3 convs with bias and relu, no batch norm; "M" = 2x2 / stride 2 max pool
VGG16_CONV = (64, 64, "M", 128, 128, "M", 256, 256, 256, "M", 512, 512, 512, "M", 512, 512, 512, "M")


def vgg16_convs() -> List[Op]:
    """The 13 fused conv + bias + relu layers and 5 pools of VGG-16 (the paper's second large vision
    model, Section 5); the three dense layers behind them are left out."""
    ops, cur, cin, blk, j = [], "x", 3, 1, 1
    for v in VGG16_CONV:
        if v == "M":
            ops.append(Op("maxpool", f"pool{blk}", cur, f"p{blk}", cin=cin, cout=cin, r=2, stride=2, pad=0))
            cur, blk, j = f"p{blk}", blk + 1, 1
        else:
            ops.append(conv(f"conv{blk}_{j}", cur, f"c{blk}_{j}", cin, v, 3, 1, 1, bn=False, bias=True))
            cur, cin, j = f"c{blk}_{j}", v, j + 1
    return ops


# Width table of one Inception block: input channels, 1x1 branch, 3x3 reduce -> 3x3, 5x5 reduce -> 5x5,
# pool projection.  (256, 128, 128, 192, 32, 96, 64) are the published widths of GoogLeNet's second
# block at 28x28, chosen because every reduction length is a multiple of 32 channels.
INCEPTION_WIDTHS = (256, 128, 128, 192, 32, 96, 64)


def inception_block(widths=INCEPTION_WIDTHS) -> List[Op]:
    """Four branches reading the same tensor, joined along the channel axis: the pattern the
    paper's parallel convolution combination was written for (Section 4.4).  conv + folded BN +
    relu throughout."""
    cin, c1, c3r, c3, c5r, c5, cp = widths
    return [
        conv("b1", "x", "b1.out", cin, c1, 1, 1, 0),
        conv("b3r", "x", "b3r.out", cin, c3r, 1, 1, 0),
        conv("b3", "b3r.out", "b3.out", c3r, c3, 3, 1, 1),
        conv("b5r", "x", "b5r.out", cin, c5r, 1, 1, 0),
        conv("b5", "b5r.out", "b5.out", c5r, c5, 5, 1, 2),
        Op("maxpool", "pool", "x", "pool.out", cin, cin, 3, 1, 1),
        conv("bp", "pool.out", "bp.out", cin, cp, 1, 1, 0),
        Op("concat", "cat", "b1.out", "cat", 0, c1 + c3 + c5 + cp, srcs=("b1.out", "b3.out", "b5.out", "bp.out")),
    ]


def dqn(actions: int = 18) -> List[Op]:
    """The deep Q-network the paper lists among its vision benchmarks (Section 5): the published
    architecture on a stack of four 84 x 84 frames -- 8x8 / stride 4 conv to 32 channels, 4x4 /
    stride 2 conv to 64, 3x3 / stride 1 conv to 64, each with bias and relu and no padding, then
    dense 3136 -> 512 with relu and dense 512 -> one value per action.  The first dense layer reads
    the last conv's [64, 7, 7] output flattened in (channel, row, column) order."""
    return [conv("c1", "x", "c1", 4, 32, 8, 4, 0, bn=False, bias=True),
            conv("c2", "c1", "c2", 32, 64, 4, 2, 0, bn=False, bias=True),
            conv("c3", "c2", "c3", 64, 64, 3, 1, 0, bn=False, bias=True),
            Op("dense", "fc1", "c3", "h", cin=64 * 7 * 7, cout=512, bias=True, relu=True),
            Op("dense", "fc2", "h", "q", cin=512, cout=actions, bias=True)]


def out_hw(h: int, r: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - r) // stride + 1


def trace_shapes(ops: List[Op], h: int, w: int, c: int = 3):
    """Spatial size and channel count of every named tensor: {name: (C, H, W)}."""
    shp = {"x": (c, h, w)}
    for op in ops:
        ci, hi, wi = shp[op.src]
        if op.kind in ("conv", "dwconv", "maxpool"):
            shp[op.dst] = (op.cout, out_hw(hi, op.r, op.stride, op.pad), out_hw(wi, op.r, op.stride, op.pad))
        elif op.kind == "avgpool":
            shp[op.dst] = (ci, 1, 1)
        elif op.kind == "dense":
            shp[op.dst] = (op.cout, 1, 1)
        elif op.kind == "concat":
            shp[op.dst] = (sum(shp[s][0] for s in op.srcs), hi, wi)
        else:
            raise ValueError(op.kind)
    return shp


def macs_per_image(ops: List[Op], h: int, w: int, c: int = 3) -> int:
    """Multiply-accumulates of the contractions only (epilogues and pools not counted)."""
    shp = trace_shapes(ops, h, w, c)
    total = 0
    for op in ops:
        co, ho, wo = shp[op.dst]
        if op.kind == "conv":
            total += co * ho * wo * op.cin * op.r * op.r
        elif op.kind == "dwconv":
            total += co * ho * wo * op.r * op.r
        elif op.kind == "dense":
            total += op.cin * op.cout
    return total

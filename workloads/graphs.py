"""Unfused operator graphs of the vision networks (paper Section 4.1: the dataflow DAG the
fusion pass starts from).  One node per operator call, in the order a model definition
issues them; node i may only read nodes j < i.  Shapes and names only -- no arithmetic.

The fused layer tables of `nets.py` are what operator fusion should turn these graphs into;
the tests check exactly that.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

from .nets import INCEPTION_WIDTHS, MOBILENET_V1_BLOCKS, VGG16_CONV

CONTRACTIONS = ("conv2d", "dwconv2d", "dense")
ELEMENTWISE = ("bias_add", "scale_shift", "add", "relu")
OPAQUE = ("input", "maxpool", "avgpool", "concat")


@dataclass(frozen=True)
class Node:
    kind: str                     # one of CONTRACTIONS + ELEMENTWISE + OPAQUE
    name: str
    inputs: Tuple[int, ...]       # indices of producer nodes (constants are attributes, not nodes)
    attrs: Dict[str, int] = field(default_factory=dict)


class Graph:
    def __init__(self):
        self.nodes: List[Node] = []

    def add(self, kind: str, name: str, inputs=(), **attrs) -> int:
        assert all(0 <= i < len(self.nodes) for i in inputs)
        self.nodes.append(Node(kind, name, tuple(inputs), dict(attrs)))
        return len(self.nodes) - 1

    def patterns(self) -> List[int]:
        """0 opaque, 1 elementwise / broadcast, 2 contraction."""
        return [2 if n.kind in CONTRACTIONS else 1 if n.kind in ELEMENTWISE else 0 for n in self.nodes]

    def csr(self) -> Tuple[List[int], List[int]]:
        offs, flat = [0], []
        for n in self.nodes:
            flat.extend(n.inputs)
            offs.append(len(flat))
        return offs, flat


def _conv_bn_relu(g: Graph, name, src, cin, cout, r, stride, pad, relu=True, kind="conv2d") -> int:
    c = g.add(kind, name, (src,), cin=cin, cout=cout, r=r, stride=stride, pad=pad)
    b = g.add("scale_shift", name + ".bn", (c,))
    return g.add("relu", name + ".relu", (b,)) if relu else b


def basic_block(g: Graph, p: str, x: int, cin: int, cout: int, stride: int) -> int:
    """conv-bn-relu, conv-bn, (1x1 conv-bn shortcut), add, relu -- the diamond of a residual block."""
    t = _conv_bn_relu(g, f"{p}.conv1", x, cin, cout, 3, stride, 1)
    c2 = g.add("conv2d", f"{p}.conv2", (t,), cin=cout, cout=cout, r=3, stride=1, pad=1)
    b2 = g.add("scale_shift", f"{p}.conv2.bn", (c2,))
    if stride != 1 or cin != cout:
        shortcut = _conv_bn_relu(g, f"{p}.down", x, cin, cout, 1, stride, 0, relu=False)
    else:
        shortcut = x
    s = g.add("add", f"{p}.add", (b2, shortcut))
    return g.add("relu", f"{p}.out", (s,))


def resnet18(with_dense: bool = True) -> Graph:
    g = Graph()
    x = g.add("input", "x")
    t = _conv_bn_relu(g, "conv1", x, 3, 64, 7, 2, 3)
    cur = g.add("maxpool", "maxpool", (t,), r=3, stride=2, pad=1, cin=64, cout=64)
    cin = 64
    for stage, cout in enumerate((64, 128, 256, 512), start=1):
        for blk in range(2):
            stride = 2 if (stage > 1 and blk == 0) else 1
            cur = basic_block(g, f"l{stage}.b{blk}", cur, cin, cout, stride)
            cin = cout
    if with_dense:
        p = g.add("avgpool", "avgpool", (cur,), cin=512, cout=512)
        d = g.add("dense", "fc", (p,), cin=512, cout=1000)
        g.add("bias_add", "fc.bias", (d,))
    return g


def mobilenet_v1(with_dense: bool = True) -> Graph:
    g = Graph()
    x = g.add("input", "x")
    cur = _conv_bn_relu(g, "stem", x, 3, 32, 3, 2, 1)
    for i, (cin, cout, s) in enumerate(MOBILENET_V1_BLOCKS, start=1):
        cur = _conv_bn_relu(g, f"b{i}.dw", cur, cin, cin, 3, s, 1, kind="dwconv2d")
        cur = _conv_bn_relu(g, f"b{i}.pw", cur, cin, cout, 1, 1, 0)
    if with_dense:
        p = g.add("avgpool", "avgpool", (cur,), cin=1024, cout=1024)
        d = g.add("dense", "fc", (p,), cin=1024, cout=1000)
        g.add("bias_add", "fc.bias", (d,))
    return g


def single_block(cin: int = 64) -> Graph:
    """The ResNet basic block on its own (input already has cin channels)."""
    g = Graph()
    x = g.add("input", "x")
    basic_block(g, "blk", x, cin, cin, 1)
    return g


def vgg16_convs() -> Graph:
    g = Graph()
    cur, cin, blk, j = g.add("input", "x"), 3, 1, 1
    for v in VGG16_CONV:
        if v == "M":
            cur = g.add("maxpool", f"pool{blk}", (cur,), r=2, stride=2, pad=0, cin=cin, cout=cin)
            blk, j = blk + 1, 1
        else:
            c = g.add("conv2d", f"conv{blk}_{j}", (cur,), cin=cin, cout=v, r=3, stride=1, pad=1)
            b = g.add("bias_add", f"conv{blk}_{j}.bias", (c,))
            cur = g.add("relu", f"conv{blk}_{j}.relu", (b,))
            cin, j = v, j + 1
    return g


def dqn(actions: int = 18) -> Graph:
    """Operator graph of the deep Q-network (see workloads.nets.dqn): three conv + bias + relu, dense +
    bias + relu, dense + bias."""
    g = Graph()
    cur, cin = g.add("input", "x"), 4
    for name, cout, r, stride in (("c1", 32, 8, 4), ("c2", 64, 4, 2), ("c3", 64, 3, 1)):
        c = g.add("conv2d", name, (cur,), cin=cin, cout=cout, r=r, stride=stride, pad=0)
        b = g.add("bias_add", name + ".bias", (c,))
        cur, cin = g.add("relu", name + ".relu", (b,)), cout
    d = g.add("dense", "fc1", (cur,), cin=64 * 7 * 7, cout=512)
    b = g.add("bias_add", "fc1.bias", (d,))
    cur = g.add("relu", "fc1.relu", (b,))
    d = g.add("dense", "fc2", (cur,), cin=512, cout=actions)
    g.add("bias_add", "fc2.bias", (d,))
    return g


def inception_block(widths=INCEPTION_WIDTHS) -> Graph:
    """Four branches over one input, joined by a channel concatenation."""
    cin, c1, c3r, c3, c5r, c5, cp = widths
    g = Graph()
    x = g.add("input", "x")
    b1 = _conv_bn_relu(g, "b1", x, cin, c1, 1, 1, 0)
    t = _conv_bn_relu(g, "b3r", x, cin, c3r, 1, 1, 0)
    b3 = _conv_bn_relu(g, "b3", t, c3r, c3, 3, 1, 1)
    t = _conv_bn_relu(g, "b5r", x, cin, c5r, 1, 1, 0)
    b5 = _conv_bn_relu(g, "b5", t, c5r, c5, 5, 1, 2)
    p = g.add("maxpool", "pool", (x,), r=3, stride=1, pad=1, cin=cin, cout=cin)
    bp = _conv_bn_relu(g, "bp", p, cin, cp, 1, 1, 0)
    g.add("concat", "cat", (b1, b3, b5, bp), cout=c1 + c3 + c5 + cp)
    return g


def random_dag(rng, n: int, p_contraction: float = 0.25, p_opaque: float = 0.1) -> Graph:
    """A random operator DAG for property tests: unary / binary elementwise ops, contractions and
    opaque ops over earlier nodes, several outputs allowed."""
    g = Graph()
    g.add("input", "x")
    for i in range(1, n):
        u = rng.random()
        a = int(rng.integers(max(0, i - 6), i))
        if u < p_contraction:
            g.add("conv2d", f"n{i}", (a,), cin=8, cout=8, r=1, stride=1, pad=0)
        elif u < p_contraction + p_opaque:
            g.add("maxpool", f"n{i}", (a,), r=1, stride=1, pad=0, cin=8, cout=8)
        elif rng.random() < 0.35 and i > 1 and (b := int(rng.integers(max(0, i - 6), i))) != a:
            g.add("add", f"n{i}", (a, b))
        else:
            g.add(("relu", "scale_shift", "bias_add")[int(rng.integers(0, 3))], f"n{i}", (a,))
    return g

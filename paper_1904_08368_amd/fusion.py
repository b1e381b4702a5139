"""Operator fusion front half: dataflow graph -> fusion groups -> sequence of fused primitive
functions (paper Section 4.1).  The grouping itself is the library's relay_fuse_extract; this
module marshals the graph and turns every group into the record `FusedNet` launches.

A group that holds a contraction must have the shape the kernels fuse (paper Section 4.1,
"Lowering": the fused function is compiled as one operator): contraction, then optionally
bias add, scale/shift, add of one outside tensor, relu, each reading the one before, in that
order.  Anything else raises: there is no unfused fallback.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

from . import binding as B

KIND_OF = {"conv2d": "conv", "dwconv2d": "dwconv", "dense": "dense", "maxpool": "maxpool", "avgpool": "avgpool",
           "concat": "concat"}
EPILOGUE_ORDER = ("bias_add", "scale_shift", "add", "relu")


@dataclass(frozen=True)
class FusedOp:
    """One primitive function: the fields FusedNet reads."""
    kind: str
    name: str
    src: str
    dst: str
    cin: int = 0
    cout: int = 0
    r: int = 1
    stride: int = 1
    pad: int = 0
    bias: bool = False
    bn: bool = False
    relu: bool = False
    res: Optional[str] = None
    srcs: tuple = ()      # concat: the tensors joined along the channel axis (src = srcs[0])


def extract_groups(graph) -> List[List[int]]:
    """Fusion groups of `graph` (nodes with .kind, .inputs; graph.patterns(), graph.csr()), each a
    sorted list of node indices, in execution order (by the group's last node)."""
    offs, flat = graph.csr()
    _, group = B.relay_fuse_extract(graph.patterns(), offs, flat)
    members: Dict[int, List[int]] = {}
    for i, g in enumerate(group):
        members.setdefault(g, []).append(i)
    return sorted(members.values(), key=lambda ms: ms[-1])


def lower(graph, groups: Sequence[Sequence[int]]) -> List[FusedOp]:
    """One FusedOp per group (graph inputs produce none).  The tensor a group writes carries
    the name of the group's last node."""
    nodes = graph.nodes
    out_name: Dict[int, str] = {}          # node index -> name of the tensor holding its value
    ops: List[FusedOp] = []
    for ms in groups:
        first, last = nodes[ms[0]], nodes[ms[-1]]
        if first.kind == "input":
            assert len(ms) == 1
            out_name[ms[0]] = first.name
            continue
        inside = set(ms)
        if first.kind not in KIND_OF:
            raise ValueError(f"group {[nodes[m].name for m in ms]} does not start with a contraction or a pool")
        a = first.attrs
        fields = dict(kind=KIND_OF[first.kind], name=first.name, src=out_name[first.inputs[0]], dst=last.name,
                      cin=a.get("cin", 0), cout=a.get("cout", 0), r=a.get("r", 1), stride=a.get("stride", 1),
                      pad=a.get("pad", 0))
        stage, prev = -1, ms[0]
        for m in ms[1:]:
            n = nodes[m]
            if n.kind not in EPILOGUE_ORDER or EPILOGUE_ORDER.index(n.kind) <= stage or prev not in n.inputs:
                raise ValueError(f"no fused kernel for operator {n.name} in group {[nodes[k].name for k in ms]}")
            stage = EPILOGUE_ORDER.index(n.kind)
            if n.kind == "bias_add":
                fields["bias"] = True
            elif n.kind == "scale_shift":
                fields["bn"] = True
            elif n.kind == "relu":
                fields["relu"] = True
            else:
                others = [i for i in n.inputs if i != prev]
                if len(others) != 1 or others[0] in inside:
                    raise ValueError(f"add {n.name} must take exactly one tensor from outside its group")
                fields["res"] = out_name[others[0]]
            prev = m
        if fields["kind"] in ("maxpool", "avgpool", "concat") and len(ms) != 1:
            raise ValueError("pooling and concatenation are not fused")
        if fields["kind"] == "concat":
            fields["srcs"] = tuple(out_name[i] for i in first.inputs)
        ops.append(FusedOp(**fields))
        out_name[ms[-1]] = last.name
    return ops


def fuse(graph) -> List[FusedOp]:
    return lower(graph, extract_groups(graph))


def combine_parallel(ops: Sequence[FusedOp], windows: bool = False) -> List[List[int]]:
    """Parallel convolution combination (paper Section 4.4): indices of the fused convs that can
    run as one launch -- same input tensor, same window, stride and padding, same elementwise
    tail, no residual operand (its tail would read a second tensor).  One list per combined
    conv, at least two members each, in program order.

    windows=True also lets a 1x1 conv without padding join convs with an odd r x r window padded by
    r // 2 and the same stride (it is that window with zeros around the centre tap), and lets the
    members differ in whether they end in relu: the stride-2 3x3 conv of a residual stage and the
    1x1 shortcut conv beside it become one launch.  The widest-window members come first."""
    by_key: Dict[tuple, List[int]] = {}
    for i, op in enumerate(ops):
        if op.kind != "conv" or op.res is not None:
            continue
        centred = op.r % 2 == 1 and op.pad == op.r // 2
        if windows and centred:
            by_key.setdefault((op.src, op.cin, op.stride, op.bias, op.bn, "centred"), []).append(i)
        else:
            by_key.setdefault((op.src, op.cin, op.r, op.stride, op.pad, op.bias, op.bn, op.relu), []).append(i)
    groups = []
    for key, g in by_key.items():
        if key[-1] == "centred":
            rmax = max(ops[i].r for i in g)
            rest: Dict[tuple, List[int]] = {}
            for i in g:                                   # windows between 1 and the widest keep to themselves
                if ops[i].r not in (1, rmax):
                    rest.setdefault((ops[i].r, ops[i].relu), []).append(i)
            g = [i for i in g if ops[i].r == rmax] + [i for i in g if ops[i].r == 1 and rmax > 1]
            groups += [h for h in rest.values() if len(h) > 1]
            if rmax == 1 and len({ops[i].relu for i in g}) > 1:   # plain 1x1 members: same tail, as without windows
                by_relu: Dict[bool, List[int]] = {}
                for i in g:
                    by_relu.setdefault(ops[i].relu, []).append(i)
                groups += [h for h in by_relu.values() if len(h) > 1]
                continue
        if len(g) > 1:
            groups.append(g)
    return sorted(groups, key=lambda g: min(g))

"""Pins of the fusion-extraction oracle (paper Section 4.1): hand-worked graphs, the path
definition of post-domination by brute force, validity of the groups, the real networks."""
import os

import numpy as np
import pytest

from oracle import fusion as OF
from workloads import graphs, nets

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PAT = {k: 2 for k in graphs.CONTRACTIONS} | {k: 1 for k in graphs.ELEMENTWISE} | {k: 0 for k in graphs.OPAQUE}


def golden_cases():
    cases = []
    for line in open(os.path.join(ROOT, "tests", "golden", "handworked_fusion.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, kinds, ins, ipdom, group = [f.strip() for f in line.split("|")]
        inputs = [tuple(int(t) for t in f.split(",")) if f else () for f in ins.split(";")]
        cases.append((name, [PAT[k] for k in kinds.split()], inputs, [int(t) for t in ipdom.split()],
                      [int(t) for t in group.split()]))
    return cases


# ----------------------------------------------------------------------------- oracle pins
@pytest.mark.parametrize("case", golden_cases(), ids=lambda c: c[0])
def test_oracle_matches_handworked_cases(case):
    _, pat, inputs, ipdom, group = case
    got_ip, got_gr = OF.fuse(pat, inputs)
    assert got_ip == ipdom
    assert got_gr == group
    OF.check_classes(pat, inputs, got_gr)


def _paths_to_exit(i, cons):
    if not cons[i]:
        return [[i]]
    return [[i] + p for c in cons[i] for p in _paths_to_exit(c, cons)]


@pytest.mark.parametrize("seed", range(40))
def test_oracle_post_dominators_against_path_enumeration(seed):
    """The set definition used by the oracle agrees with the path definition: d post-dominates i
    iff d lies on every path from i to the exit; the immediate one is the first such d met on
    any of those paths."""
    rng = np.random.default_rng(1000 + seed)
    g = graphs.random_dag(rng, int(rng.integers(4, 14)))
    inputs = [n.inputs for n in g.nodes]
    cons = OF.consumers(len(inputs), inputs)
    pdom = OF.post_dominator_sets(inputs)
    ipdom = OF.immediate_post_dominators(inputs)
    for i in range(len(inputs)):
        paths = _paths_to_exit(i, cons)
        on_all = set(paths[0]).intersection(*map(set, paths[1:])) if len(paths) > 1 else set(paths[0])
        assert pdom[i] - {OF.EXIT} == on_all
        first = next((v for v in paths[0][1:] if v in on_all), OF.EXIT)
        assert ipdom[i] == first


@pytest.mark.parametrize("seed", range(60))
def test_oracle_groups_are_valid_and_not_needlessly_small(seed):
    rng = np.random.default_rng(2000 + seed)
    g = graphs.random_dag(rng, int(rng.integers(5, 30)))
    pat, inputs = g.patterns(), [n.inputs for n in g.nodes]
    ipdom, group = OF.fuse(pat, inputs)
    OF.check_classes(pat, inputs, group)
    cons = OF.consumers(len(inputs), inputs)
    for i in range(len(inputs)):
        # an operator with a single elementwise consumer that reads nothing but it is always fused
        # with that consumer: the simplest chain case cannot be refused by any rule
        if pat[i] != 0 and len(cons[i]) == 1 and pat[cons[i][0]] == 1 and len(set(inputs[cons[i][0]])) == 1:
            assert group[i] == group[cons[i][0]], (i, cons[i][0])
        if pat[i] == 0:
            assert sum(1 for x in group if x == group[i]) == 1


def test_oracle_on_the_networks_gives_one_group_per_layer():
    for g, table in ((graphs.resnet18(), nets.resnet18()), (graphs.mobilenet_v1(), nets.mobilenet_v1())):
        pat, inputs = g.patterns(), [n.inputs for n in g.nodes]
        _, group = OF.fuse(pat, inputs)
        OF.check_classes(pat, inputs, group)
        members = {}
        for i, gid in enumerate(group):
            members.setdefault(gid, []).append(i)
        layers = sorted((ms for ms in members.values() if g.nodes[ms[0]].kind != "input"), key=lambda ms: ms[-1])
        assert len(layers) == len(table)
        for ms, op in zip(layers, table):
            kinds = [g.nodes[m].kind for m in ms]
            want = [{"conv": "conv2d", "dwconv": "dwconv2d"}.get(op.kind, op.kind)]
            want += ["bias_add"] * op.bias + ["scale_shift"] * op.bn + ["add"] * (op.res is not None) + ["relu"] * op.relu
            assert kinds == want, (op.name, kinds)



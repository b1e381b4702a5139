"""CPU oracle -- TEST INFRASTRUCTURE ONLY: extraction of fusion groups from a dataflow DAG
(paper Section 4.1, "Extraction"), written from the definitions, slow on purpose.

The paper's steps: build the dataflow DAG between operators, build its post-dominator tree,
put subexpressions into equivalence classes by their immediate post-dominator, make one
primitive function per class.  It does not say which operators may share a class; the reading
taken here (and stated in the design notes) is the smallest rule that yields the fused
operators the paper describes (a contraction with the elementwise operators behind it,
diamonds of elementwise operators):

  R1  an operator joins the class of its immediate post-dominator d only if every operator on
      every path from it to d, d included, is elementwise/broadcast (pattern 1): nothing opaque
      and no second contraction is swallowed;
  R2  a class holds at most one contraction (pattern 2); opaque operators (pattern 0) stay alone;
  R3  operators are visited in dataflow (topological) order and a merge takes the operators on
      the paths along, so a class is always a connected, convex piece of the DAG; a merge that
      would break R2 is skipped.

Everything is computed from set definitions: post-dominators as intersections over
consumers, paths by explicit enumeration.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Set, Tuple

EXIT = -1  # the virtual exit node that every output flows into


def consumers(n: int, inputs: Sequence[Sequence[int]]) -> List[List[int]]:
    out: List[List[int]] = [[] for _ in range(n)]
    for i, ins in enumerate(inputs):
        for j in ins:
            if i not in out[j]:
                out[j].append(i)
    return out


def post_dominator_sets(inputs: Sequence[Sequence[int]]) -> List[Set[int]]:
    """pdom(i) = {i} united with the intersection of pdom(c) over the consumers c of i; an
    operator nobody consumes flows into EXIT.  (d post-dominates i iff every path from i to
    EXIT passes through d.)"""
    n = len(inputs)
    cons = consumers(n, inputs)
    pdom: List[Set[int]] = [set() for _ in range(n)]
    for i in reversed(range(n)):          # consumers have larger indices
        if not cons[i]:
            pdom[i] = {i, EXIT}
        else:
            common = set.intersection(*(pdom[c] for c in cons[i]))
            pdom[i] = {i} | common
    return pdom


def immediate_post_dominators(inputs: Sequence[Sequence[int]]) -> List[int]:
    """The strict post-dominator closest to i: the one that all other strict post-dominators
    of i post-dominate in turn."""
    pdom = post_dominator_sets(inputs)
    out = []
    for i in range(len(inputs)):
        strict = pdom[i] - {i}
        best = EXIT
        for d in strict:
            if d == EXIT:
                continue
            if all(e == d or e in pdom[d] for e in strict):
                best = d
        out.append(best)
    return out


def all_paths(src: int, dst: int, cons: List[List[int]]) -> List[List[int]]:
    """Every path src -> ... -> dst as a list of nodes, src excluded, dst included."""
    if src == dst:
        return [[]]
    paths = []
    for c in cons[src]:
        for tail in all_paths(c, dst, cons):
            paths.append([c] + tail)
    return paths


def fuse(patterns: Sequence[int], inputs: Sequence[Sequence[int]]) -> Tuple[List[int], List[int]]:
    """Returns (ipdom, group): group[i] = smallest node index of the class of i."""
    n = len(patterns)
    cons = consumers(n, inputs)
    ipdom = immediate_post_dominators(inputs)
    cls: List[Set[int]] = [{i} for i in range(n)]     # cls[i] is shared by all members

    def contractions(members: Set[int]) -> int:
        return sum(1 for m in members if patterns[m] == 2)

    for i in range(n):
        d = ipdom[i]
        if patterns[i] == 0 or d == EXIT:
            continue
        on_paths: Set[int] = set()
        for path in all_paths(i, d, cons):
            on_paths.update(path)
        if any(patterns[m] != 1 for m in on_paths):                 # R1
            continue
        merged: Set[int] = set(cls[i])
        for m in on_paths:
            merged |= cls[m]
        if contractions(merged) > 1:                                # R2
            continue
        for m in merged:                                            # R3
            cls[m] = merged
    return ipdom, [min(cls[i]) for i in range(n)]


def check_classes(patterns: Sequence[int], inputs: Sequence[Sequence[int]], group: Sequence[int]) -> None:
    """Invariants any valid grouping has: at most one contraction per class, opaque operators
    alone, exactly one operator of a class is read from outside it (its output), and the classes
    can be executed one after another (the class graph is acyclic)."""
    n = len(patterns)
    cons = consumers(n, inputs)
    members: Dict[int, List[int]] = {}
    for i, g in enumerate(group):
        members.setdefault(g, []).append(i)
    for g, ms in members.items():
        assert g == min(ms)
        assert sum(1 for m in ms if patterns[m] == 2) <= 1, ("two contractions", ms)
        if any(patterns[m] == 0 for m in ms):
            assert len(ms) == 1, ("opaque operator fused", ms)
        escaping = [m for m in ms if not cons[m] or any(group[c] != g for c in cons[m])]
        assert len(escaping) == 1, ("class with several outputs", ms, escaping)
        assert escaping[0] == max(ms)
    # acyclic class graph: order classes by their last operator; every input class must end earlier
    last = {g: max(ms) for g, ms in members.items()}
    for i, ins in enumerate(inputs):
        for j in ins:
            if group[j] != group[i]:
                assert last[group[j]] < last[group[i]], ("class order", j, i)

"""Fusion extraction (paper Section 4.1): parity of the library's pass with the oracle, lowering of
the real networks to the hand-written layer tables, argument checks.  All host code."""
import numpy as np
import pytest

from oracle import fusion as OF
from paper_1904_08368_amd import binding as B
from paper_1904_08368_amd import fusion as PF
from tests.test_fusion_oracle import golden_cases
from workloads import graphs, nets


def _csr(inputs):
    offs, flat = [0], []
    for ins in inputs:
        flat.extend(ins)
        offs.append(len(flat))
    return offs, flat


# ------------------------------------------------------------------- library pass vs oracle
@pytest.mark.parametrize("case", golden_cases(), ids=lambda c: c[0])
def test_library_matches_handworked_cases(case):
    _, pat, inputs, ipdom, group = case
    got_ip, got_gr = B.relay_fuse_extract(pat, *_csr(inputs))
    assert got_ip == ipdom and got_gr == group


@pytest.mark.parametrize("seed", range(300))
def test_library_matches_oracle_on_random_dags(seed):
    rng = np.random.default_rng(3000 + seed)
    g = graphs.random_dag(rng, int(rng.integers(2, 48)), p_contraction=float(rng.uniform(0.05, 0.4)),
                          p_opaque=float(rng.uniform(0.0, 0.2)))
    pat, inputs = g.patterns(), [n.inputs for n in g.nodes]
    want_ip, want_gr = OF.fuse(pat, inputs)
    got_ip, got_gr = B.relay_fuse_extract(pat, *g.csr())
    assert got_ip == want_ip
    assert got_gr == want_gr


@pytest.mark.parametrize("make", [graphs.resnet18, graphs.mobilenet_v1, graphs.single_block])
def test_library_matches_oracle_on_the_networks(make):
    g = make()
    pat, inputs = g.patterns(), [n.inputs for n in g.nodes]
    assert B.relay_fuse_extract(pat, *g.csr()) == OF.fuse(pat, inputs)


def test_single_operator_and_wide_fan_out():
    assert B.relay_fuse_extract([0], [0, 0], []) == ([-1], [0])
    # one conv read by 50 relus that are never joined: nothing post-dominates it but the exit
    n = 52
    pat = [0, 2] + [1] * 50
    inputs = [(), (0,)] + [(1,)] * 50
    ip, gr = B.relay_fuse_extract(pat, *_csr(inputs))
    assert ip == [1] + [-1] * 51 and gr == list(range(n))
    assert (ip, gr) == OF.fuse(pat, inputs)


# ------------------------------------------------------------------- lowering to the tables
def _same_layers(ops, table):
    assert len(ops) == len(table)
    rename = {"x": "x"}
    for a, b in zip(ops, table):
        for f in ("kind", "name", "cin", "cout", "r", "stride", "pad", "bias", "bn", "relu"):
            assert getattr(a, f) == getattr(b, f), (a.name, f)
        assert rename[a.src] == b.src, a.name
        assert (a.res is None) == (b.res is None) and (a.res is None or rename[a.res] == b.res), a.name
        rename[a.dst] = b.dst


def test_fusing_the_network_graphs_reproduces_the_layer_tables():
    _same_layers(PF.fuse(graphs.resnet18()), nets.resnet18())
    _same_layers(PF.fuse(graphs.resnet18(with_dense=False)), nets.resnet18(with_dense=False))
    _same_layers(PF.fuse(graphs.mobilenet_v1()), nets.mobilenet_v1())
    _same_layers(PF.fuse(graphs.single_block()), nets.basic_block())
    _same_layers(PF.fuse(graphs.vgg16_convs()), nets.vgg16_convs())
    _same_layers(PF.fuse(graphs.inception_block()), nets.inception_block())
    _same_layers(PF.fuse(graphs.dqn()), nets.dqn())


def test_lowering_refuses_groups_without_a_fused_kernel():
    g = graphs.Graph()
    x = g.add("input", "x")
    c = g.add("conv2d", "c", (x,), cin=8, cout=8, r=1, stride=1, pad=0)
    r = g.add("relu", "r", (c,))
    g.add("scale_shift", "late_bn", (r,))          # relu before scale/shift: not the fused order
    with pytest.raises(ValueError):
        PF.fuse(g)
    g = graphs.Graph()
    x = g.add("input", "x")
    g.add("relu", "lonely", (x,))                  # elementwise group with no contraction
    with pytest.raises(ValueError):
        PF.fuse(g)


# --------------------------------------------------------------------------- ABI validation
def test_fuse_extract_rejects_bad_graphs():
    import ctypes as C
    lib = B.lib()
    arr = lambda v: (C.c_int32 * len(v))(*v)
    out = (C.c_int32 * 4)()
    P = C.c_void_p
    OK, E_NULL, E_SHAPE, E_UNSUPPORTED = 0, 1, 2, 4     # relay_status values of include/relay_fused.h
    call = lambda n, pat, offs, ins, grp: lib.relay_fuse_extract(n, C.cast(pat, P) if pat else None, C.cast(offs, P),
                                                                 C.cast(ins, P), None, C.cast(grp, P) if grp else None)
    ok = (arr([0, 2, 1]), arr([0, 0, 1, 2]), arr([0, 1]))
    assert call(3, *ok, out) == OK
    assert call(3, None, ok[1], ok[2], out) == E_NULL
    assert call(3, *ok, None) == E_NULL
    assert call(0, *ok, out) == E_SHAPE
    assert call(3, arr([0, 5, 1]), ok[1], ok[2], out) == E_UNSUPPORTED
    assert call(3, ok[0], arr([0, 0, 2, 1]), ok[2], out) == E_SHAPE          # offsets decrease
    assert call(3, ok[0], ok[1], arr([0, 2]), out) == E_SHAPE                # reads a later operator
    assert call(3, ok[0], arr([1, 1, 2, 3]), ok[2], out) == E_SHAPE          # offsets do not start at 0
    assert b"earlier" in lib.relay_last_error() or b"in_offsets" in lib.relay_last_error()


def test_parallel_conv_grouping_equals_the_oracles():
    """The product's grouping for parallel convolution combination (paper Section 4.4), with and
    without members of different windows, against the oracle's own implementation of the rule."""
    from oracle import combine as OC
    from paper_1904_08368_amd import fusion
    from workloads import nets
    c = nets.conv
    tables = [nets.resnet18(), nets.mobilenet_v1(), nets.inception_block(), nets.vgg16_convs(),
              [c("a", "x", "a", 32, 8, 1, 2, 0, relu=False), c("b", "x", "b", 32, 16, 3, 2, 1), c("c", "x", "c", 32, 16, 3, 1, 1),
               c("d", "x", "d", 32, 16, 5, 2, 2), c("e", "x", "e", 32, 16, 3, 2, 0), c("f", "x", "f", 32, 16, 3, 2, 1, relu=False),
               c("g", "x", "g", 32, 24, 3, 2, 1, relu=False), c("h", "a", "h", 8, 8, 1, 1, 0), c("i", "a", "i", 8, 8, 1, 1, 0, relu=False),
               c("j", "a", "j", 8, 16, 1, 1, 0), c("k", "a", "k", 8, 8, 1, 1, 0, res="h")]]
    for ops in tables:
        for w in (False, True):
            assert fusion.combine_parallel(ops, windows=w) == OC.combine_groups(ops, windows=w), (ops[0].name, w)
    assert fusion.combine_parallel(tables[-1], windows=True) == [[3, 0], [5, 6], [7, 9]]

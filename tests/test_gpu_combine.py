"""GPU parity of the paper's Section 4.4 rewrites: axis scale folding (bit-exact against the
oracle's fp64 product rounded once) and parallel convolution combination (one launch whose
channel segments equal the members' own fused convs of the oracle), through the C ABI."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import combine as OC
from oracle.stack import run_float
from workloads import inputs, nets

pytestmark = pytest.mark.gpu
TOL_F16 = 1e-2


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


# ------------------------------------------------------------------------------ scale folding
@pytest.mark.parametrize("dt", ["f16", "f32"])
@pytest.mark.parametrize("axis", ["out", "in"])
def test_fold_scale_axis_is_bit_exact(G, dt, axis):
    from paper_1904_08368_amd import binding as B
    rng = np.random.default_rng(11)
    k, c, r = 37, 21, 3
    w = rng.standard_normal((k, c, r, r)).astype(np.float16 if dt == "f16" else np.float32)
    w[0, 0, 0, 0] = 1.0 + 2.0 ** -10            # products that land near fp16 rounding boundaries
    w[1, 1] = 6.1e-5                            # around the fp16 subnormal threshold
    s = (1.0 + 0.1 * rng.standard_normal(c if axis == "in" else k)).astype(np.float32)
    s[0] = np.float32(1.0 + 2.0 ** -11 + 2.0 ** -23)
    wd, sd = G.up(w), G.up(s)
    out = torch.empty_like(wd)
    B.relay_fold_scale_axis(B.RELAY_F16 if dt == "f16" else B.RELAY_F32, k, c, r * r,
                            B.FOLD_IN if axis == "in" else B.FOLD_OUT, wd, sd, out)
    torch.cuda.synchronize()
    want = OC.fold_scale_axis(w, s, axis, dt)
    got = out.cpu().numpy()
    assert got.dtype == want.dtype and np.array_equal(got.view(np.uint16 if dt == "f16" else np.uint32),
                                                      want.view(np.uint16 if dt == "f16" else np.uint32))
    # in place
    B.relay_fold_scale_axis(B.RELAY_F16 if dt == "f16" else B.RELAY_F32, k, c, r * r,
                            B.FOLD_IN if axis == "in" else B.FOLD_OUT, wd, sd, wd)
    torch.cuda.synchronize()
    assert np.array_equal(wd.cpu().numpy(), want)


def test_fold_bias_is_bit_exact(G):
    from paper_1904_08368_amd import binding as B
    rng = np.random.default_rng(12)
    k = 300
    b, sc, sf = (rng.standard_normal(k).astype(np.float32) for _ in range(3))
    out = torch.empty(k, dtype=torch.float32, device=G.DEV)
    for bias in (b, None):
        B.relay_fold_bias(k, G.up(bias), G.up(sc), G.up(sf), out)
        torch.cuda.synchronize()
        p = {"w": np.zeros((k, 1, 1, 1), np.float32), "scale": sc, "shift": sf}
        if bias is not None:
            p["bias"] = bias
        want = OC.fold_bn_into_conv(p, "f32")["bias"]
        assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32))


# ------------------------------------------------------------------------ parallel combination
def _members(cin, couts, r, seed, bias=False):
    ops = [nets.conv(f"m{j}", "x", f"m{j}", cin, k, r, 1, r // 2, bias=bias) for j, k in enumerate(couts)]
    return ops, [inputs.layer_params(op, 21, 10 * seed + j, "f16") for j, op in enumerate(ops)]


def _run_combined(G, x, ops, params, stride, pad, relu, x_wide=0, x_off=0, out_plan=None, tile=-1):
    """x [N,C,H,W] fp16 -> list of member outputs (NCHW numpy) plus the raw output tensors.
    x_wide > 0: the input is channels [x_off, x_off + C) of an NHWC tensor of x_wide channels.
    out_plan[i] = (buffer index, first channel, buffer channels) places segment i; default: own tensors."""
    from paper_1904_08368_amd import binding as B
    n, c, h, w = x.shape
    r = ops[0].r
    couts = [o.cout for o in ops]
    flags = B.flags_of(params[0].get("bias"), params[0].get("scale"), None, relu)
    d = B.conv_desc(n, c, h, w, sum(couts), r, r, stride, pad, B.RELAY_F16, B.RELAY_NHWC, flags)
    ho, wo = B.relay_conv2d_out_shape(d)
    xd = G.to_nhwc(x, c, B.RELAY_F16)
    if x_wide:
        wide = torch.full((n, h, w, x_wide), 99.0, dtype=torch.float16, device=G.DEV)
        wide[..., x_off:x_off + c] = xd
        xd = wide[..., x_off:x_off + c]
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=G.DEV)
    off = 0
    for o, p in zip(ops, params):
        dm = B.conv_desc(n, c, h, w, o.cout, r, r, stride, pad, B.RELAY_F16, B.RELAY_NHWC, flags)
        nb = B.relay_packed_weight_bytes(dm)
        B.relay_prepack_conv2d_weights(dm, G.up(p["w"]), c, wp[off:off + nb])
        off += nb
    cat = lambda key: None if params[0].get(key) is None else G.up(np.concatenate([p[key] for p in params]))
    bufs = {}
    ys = []
    for i, k in enumerate(couts):
        bi, c0, cw = out_plan[i] if out_plan else (i, 0, k)
        if bi not in bufs:
            bufs[bi] = torch.full((n, ho, wo, cw), -77.0, dtype=torch.float16, device=G.DEV)
        ys.append(bufs[bi][..., c0:c0 + k])
    B.relay_set_conv_tile(tile)
    try:
        B.relay_fused_conv2d_combined(d, xd, xd.stride(2), wp, cat("bias"), cat("scale"), cat("shift"), couts, ys,
                                      [y.stride(2) for y in ys])
    finally:
        B.relay_set_conv_tile(-1)
    torch.cuda.synchronize()
    return [G.from_nhwc(y, k) for y, k in zip(ys, couts)], bufs


def _check_members(x, ops, params, outs, stride, pad, relu):
    for o, p, got in zip(ops, params, outs):
        want = O.fused_conv2d(x, p["w"], stride=(stride, stride), pad=(pad, pad), bias=p.get("bias"),
                              scale=p.get("scale"), shift=p.get("shift"), relu_flag=relu, out_dtype="f16")
        assert got.shape == want.shape
        assert O.max_rel_err(got, want) <= TOL_F16, o.name


def test_inception_1x1_members_into_their_own_tensors(G):
    ops, params = _members(256, (128, 128, 32), 1, 0)
    x = inputs.activation(21, 0, (2, 256, 28, 28), "f16")
    outs, _ = _run_combined(G, x, ops, params, 1, 0, True)
    _check_members(x, ops, params, outs, 1, 0, True)
    assert all(o.min() >= 0 for o in outs)


@pytest.mark.parametrize("tile", [-1, 3, 4, 5, 9, 10, 16])
def test_ragged_segments_views_on_both_sides(G, tile):
    """Segment boundaries off the wave tiles (8, 24, 40 channels), a pixel count that is no multiple of
    any tile, the input a channel range of a wider tensor, two segments inside one wider output tensor
    whose other channels must stay untouched."""
    ops, params = _members(64, (8, 24, 40), 3, 1, bias=True)
    x = inputs.activation(21, 1, (3, 64, 9, 7), "f16")
    plan = [(0, 16, 64), (1, 0, 24), (0, 24, 64)]        # segment 0 -> buf0[16:24], 2 -> buf0[24:64]
    outs, bufs = _run_combined(G, x, ops, params, 1, 1, True, x_wide=96, x_off=32, out_plan=plan, tile=tile)
    _check_members(x, ops, params, outs, 1, 1, True)
    assert torch.all(bufs[0][..., :16] == -77.0)


def test_strided_conv_and_no_tail(G):
    ops, params = _members(32, (16, 48), 3, 2)
    for p in params:
        p.pop("scale"), p.pop("shift")
    x = inputs.activation(21, 2, (2, 32, 11, 13), "f16")
    outs, _ = _run_combined(G, x, ops, params, 2, 1, False)
    _check_members(x, ops, params, outs, 2, 1, False)
    assert min(o.min() for o in outs) < 0


def test_one_segment_equals_the_plain_entry_point(G):
    ops, params = _members(128, (96,), 3, 3)
    x = inputs.activation(21, 3, (2, 128, 14, 14), "f16")
    outs, _ = _run_combined(G, x, ops, params, 1, 1, True)
    p = params[0]
    plain = G.run_conv_f16(x, p["w"], 1, 1, scale=p["scale"], shift=p["shift"], relu=True)
    assert np.array_equal(outs[0], plain)


# ------------------------------------------------------------------------------ whole blocks
def _block(G, combine, fold_scale=False, batch=2, hw=28):
    from paper_1904_08368_amd import fusion
    from paper_1904_08368_amd.stack import FusedNet
    from workloads import graphs
    ops = fusion.fuse(graphs.inception_block())
    table = nets.inception_block()
    params = inputs.net_params(table, 22, "f16")
    x = inputs.image(22, batch, 256, hw, hw, "f16")
    net = FusedNet(ops, params, batch, hw, hw, "f16", in_channels=256, combine=combine, fold_scale=fold_scale)
    net.load_input(x)
    net.run()
    torch.cuda.synchronize()
    return net, ops, table, params, x


@pytest.mark.parametrize("combine", [False, True])
def test_inception_block_from_its_graph(G, combine):
    net, ops, table, params, x = _block(G, combine)
    ref = run_float(table, params, x, "f16")
    for a, b in zip(ops, table):
        assert O.max_rel_err(net.tensor(a.dst), ref[b.dst]) <= TOL_F16, a.name
    assert net.tensor("cat").shape == ref["cat"].shape == (2, 480, 28, 28)
    convs = [n for n in net.call_names if n not in ("nchw_to_nhwc", "pool")]
    assert len(convs) == (4 if combine else 6) and ("b1+b3r+b5r" in convs) == combine


def test_combined_and_separate_blocks_agree_bit_for_bit(G):
    a = _block(G, False)[0].tensor("cat")
    b = _block(G, True)[0].tensor("cat")
    assert np.array_equal(a, b)


def test_scale_folding_on_networks(G):
    """Folded networks against the oracle run on folded parameters (the same rewrite done in fp64)."""
    net, ops, table, params, x = _block(G, True, fold_scale=True)
    folded = [OC.fold_bn_into_conv(p, "f16") if p else p for p in params]
    ref = run_float(table, folded, x, "f16")
    assert O.max_rel_err(net.tensor("cat"), ref["cat"]) <= TOL_F16
    # and within fp16 rounding of the unfolded network
    assert O.max_rel_err(net.tensor("cat"), run_float(table, params, x, "f16")["cat"]) <= 2e-2
    # ResNet basic block: the residual conv takes the folded form through the plain entry point
    from paper_1904_08368_amd.stack import FusedNet
    table = nets.basic_block(64)
    params = inputs.net_params(table, 2, "f16")
    x = inputs.image(2, 1, 64, 56, 56, "f16")
    net = FusedNet(table, params, 1, 56, 56, "f16", in_channels=64, fold_scale=True)
    net.load_input(x)
    net.run()
    torch.cuda.synchronize()
    ref = run_float(table, [OC.fold_bn_into_conv(p, "f16") for p in params], x, "f16")
    assert O.max_rel_err(net.tensor("blk.out"), ref["blk.out"]) <= TOL_F16


def test_inception_block_batch32_sampled(G):
    """The configuration the benchmark times: batch 32, combined launch, concatenation by views.  The
    block input is the oracle's input too (first layer deep), so sampled outputs of every conv that
    reads it are recomputed one by one; the deeper convs are checked through the whole-block test."""
    net, ops, table, params, x = _block(G, True, batch=32)
    g = np.random.default_rng(2204)
    cat = net.tensor("cat")
    assert cat.shape == (32, 480, 28, 28) and not np.isnan(cat).any() and cat.min() >= 0
    for a, b, p in zip(ops, table, params):
        if b.kind != "conv" or b.src != "x":
            continue
        got = net.tensor(a.dst)
        pts = [(int(g.integers(32)), int(g.integers(b.cout)), int(g.integers(28)), int(g.integers(28))) for _ in range(120)]
        pts += [(0, 0, 0, 0), (31, b.cout - 1, 27, 27)]
        acc = O.conv2d_points(x, p["w"], pts, (1, 1), (0, 0))
        want = O.cast_f16(O.float_epilogue_points(acc, [t[1] for t in pts], scale=p["scale"], shift=p["shift"], relu_flag=True))
        gv = np.array([got[t] for t in pts]).astype(np.float64)
        rms = float(np.sqrt(np.mean(got.astype(np.float64) ** 2)))
        err = np.max(np.abs(gv - want.astype(np.float64)) / np.maximum(np.abs(want.astype(np.float64)), rms))
        assert err <= TOL_F16, b.name
    # the 1x1 member that goes straight into the concatenation sits in its channel range
    assert np.array_equal(cat[:, :128], net.tensor(ops[0].dst))


# ------------------------------------------------ members with different windows and tails
def _run_windows(G, x, full, centre, stride, tile=-1, reps=0, poison=True, centre_window=True):
    """full / centre: (op, params) of an r x r conv (relu) and of a 1x1 conv (no relu) reading x with
    the same stride -> their outputs from ONE launch (NCHW numpy)."""
    from paper_1904_08368_amd import binding as B
    n, c, h, w = x.shape
    (of, pf), (oc, pc) = full, centre
    r = of.r
    d = B.conv_desc(n, c, h, w, of.cout + oc.cout, r, r, stride, r // 2, B.RELAY_F16, B.RELAY_NHWC, B.HAS_BN | B.RELU)
    ho, wo = B.relay_conv2d_out_shape(d)
    xd = G.to_nhwc(x, c, B.RELAY_F16)
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=G.DEV)
    # the 1x1 filters at the centre tap; the taps around it are never read, so they can hold anything
    wc = inputs.rng_for(22, 4242).standard_normal((oc.cout, c, r, r)).astype(np.float16) if poison else \
        np.zeros((oc.cout, c, r, r), np.float16)
    wc[:, :, r // 2, r // 2] = pc["w"][:, :, 0, 0]
    B.relay_prepack_conv2d_weights(d, G.up(np.concatenate([pf["w"], wc])), c, wp)
    cat = lambda key: G.up(np.concatenate([pf[key], pc[key]]))
    ys = [torch.full((n, ho, wo, k), -77.0, dtype=torch.float16, device=G.DEV) for k in (of.cout, oc.cout)]
    sc, sf = cat("scale"), cat("shift")
    B.relay_set_conv_tile(tile)
    try:
        call = lambda: B.relay_fused_conv2d_combined_windows(d, xd, c, wp, None, sc, sf, [of.cout, oc.cout], ys,
                                                             [of.cout, oc.cout],
                                                             [B.WINDOW_FULL, B.WINDOW_CENTRE if centre_window else B.WINDOW_FULL], [1, 0])
        call()
        torch.cuda.synchronize()
        us = None
        if reps:
            g = torch.cuda.CUDAGraph()                 # replayed from a graph: the spacing is the GPU's, not Python's
            with torch.cuda.graph(g):
                for _ in range(reps):
                    call()
            g.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / reps
    finally:
        B.relay_set_conv_tile(-1)
    return [G.from_nhwc(y, k) for y, k in zip(ys, (of.cout, oc.cout))], us


@pytest.mark.parametrize("shape", [(2, 64, 56, 56, 128, 2), (3, 128, 28, 28, 256, 2), (2, 256, 14, 14, 512, 2),
                                   (1, 64, 17, 13, 128, 1)])
@pytest.mark.parametrize("tile", [-1, 0, 5])
def test_strided_conv_and_its_shortcut_conv_in_one_launch(G, shape, tile):
    """ResNet's 3x3 / stride 2 conv (bn, relu) and the 1x1 / stride 2 shortcut conv (bn) beside it:
    one launch, the shortcut as a centre-tap segment without relu; each against its own oracle conv."""
    n, c, h, w, k, st = shape
    of = nets.conv("a", "x", "a", c, k, 3, st, 1)
    oc = nets.conv("d", "x", "d", c, k, 1, st, 0, relu=False)
    pf, pc = inputs.layer_params(of, 22, k, "f16"), inputs.layer_params(oc, 22, k + 1, "f16")
    x = inputs.activation(22, c, (n, c, h, w), "f16")
    (ya, yd), _ = _run_windows(G, x, (of, pf), (oc, pc), st, tile=tile)
    wa = O.fused_conv2d(x, pf["w"], stride=(st, st), pad=(1, 1), scale=pf["scale"], shift=pf["shift"], relu_flag=True,
                        out_dtype="f16")
    wd = O.fused_conv2d(x, pc["w"], stride=(st, st), pad=(0, 0), scale=pc["scale"], shift=pc["shift"], relu_flag=False,
                        out_dtype="f16")
    assert ya.shape == wa.shape and yd.shape == wd.shape
    assert O.max_rel_err(ya, wa) <= TOL_F16 and ya.min() >= 0
    assert O.max_rel_err(yd, wd) <= TOL_F16 and yd.min() < 0          # the shortcut really has no relu


@pytest.mark.parametrize("fold_scale", [False, True])
def test_resnet18_with_stage_convs_and_shortcuts_merged(G, fold_scale):
    """ResNet-18 with the three (3x3 / stride 2, 1x1 / stride 2 shortcut) pairs as one launch each: three
    launches fewer, and the first pair's tensors the same bits as from the separate launches (the same
    sums in the same order: a centre-tap segment reduces over exactly the 1x1 conv's channels)."""
    from oracle.stack import run_float
    from paper_1904_08368_amd.stack import FusedNet
    ops = nets.resnet18()
    params = inputs.net_params(ops, 3, "f16")
    x = inputs.image(36, 2, 3, 224, 224, "f16")
    outs, launches = {}, {}
    for mode in (False, "windows"):
        net = FusedNet(ops, params, 2, 224, 224, "f16", combine=mode, fold_scale=fold_scale)
        net.load_input(x)
        net.run()
        torch.cuda.synchronize()
        launches[mode] = len(net.calls)
        outs[mode] = {name: net.tensor(name) for name in ("l2.b0.t", "l2.b0.d", "l2.b0.out", "l4.b1.out", "logits")
                      if name in net.bufs}
    assert launches[False] - launches["windows"] == 3
    assert outs[False].keys() == outs["windows"].keys() and "l4.b1.out" in outs[False]
    for name in ("l2.b0.t", "l2.b0.d", "l2.b0.out"):
        assert int((outs[False][name].view(np.uint16) != outs["windows"][name].view(np.uint16)).sum()) == 0, name
    # (at this batch the separate 256- and 512-channel convs split their reduction over workgroups, which
    # orders the partial sums differently: the deeper tensors agree to rounding, not to the bit)
    for name in ("l4.b1.out", "logits"):
        assert O.max_rel_err(outs["windows"][name], outs[False][name]) <= TOL_F16, name
    if not fold_scale:
        ref = run_float(ops, params, x, "f16")
        assert O.max_rel_err(outs["windows"]["logits"].reshape(2, 1000), ref["logits"]) <= 2e-2


@pytest.mark.parametrize("r", [1, 3])
def test_int8_combined_convs_bit_exact(r):
    """Quantized convs over the same input as one launch: every member equals its own oracle conv and its
    own separate launch bit for bit, with one common shift and with a scale per member; input and
    outputs are channel ranges of wider tensors."""
    from oracle import schemes as S
    from paper_1904_08368_amd import binding as B
    from tests import gpu_util as G
    g = np.random.default_rng(520 + r)
    n, c, hw, widths = 2, 64, 14, (64, 24, 40)
    k = sum(widths)
    pad = r // 2
    wide = g.integers(-127, 128, (n, c + 64, hw, hw)).astype(np.int8)            # the convs read channels 64 .. 127 of this
    x = wide[:, 64:]
    ws = [g.integers(-127, 128, (kk, c, r, r)).astype(np.int8) for kk in widths]
    bs = [g.integers(-4000, 4000, kk).astype(np.int32) for kk in widths]
    d = B.conv_desc(n, c, hw, hw, k, r, r, 1, pad, B.RELAY_I8, B.RELAY_NHWC, B.flags_of(True, None, None, True))
    xw = G.to_nhwc(wide, c + 64, B.RELAY_I8)
    xv = xw[..., 64:]
    wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=G.DEV)
    off = 0
    for wt, kk in zip(ws, widths):
        dm = B.conv_desc(n, c, hw, hw, kk, r, r, 1, pad, B.RELAY_I8, B.RELAY_NHWC, 0)
        nb = B.relay_packed_weight_bytes(dm)
        B.relay_prepack_conv2d_weights(dm, G.up(wt), c, wp[off:off + nb])
        off += nb
    bias = G.up(np.concatenate(bs))
    cat = torch.full((n, hw, hw, widths[0] + widths[1]), -128, dtype=torch.int8, device=G.DEV)   # members 0 and 1 share a joined tensor
    y2 = torch.full((n, hw, hw, widths[2]), -128, dtype=torch.int8, device=G.DEV)
    ys = [cat[..., :widths[0]], cat[..., widths[0]:], y2]
    lds = [cat.shape[-1], cat.shape[-1], widths[2]]
    s = 12 if r == 3 else 10
    # (i) one common power-of-two shift
    B.relay_qconv2d_combined(d, xv, xw.shape[-1], wp, bias, None, None, s, list(widths), ys, lds)
    torch.cuda.synchronize()
    outs = [G.from_nhwc(cat, cat.shape[-1])[:, :widths[0]], G.from_nhwc(cat, cat.shape[-1])[:, widths[0]:], G.from_nhwc(y2, widths[2])]
    for wt, b, got in zip(ws, bs, outs):
        ref = O.qconv2d_requant(x, wt, stride=(1, 1), pad=(pad, pad), bias=b, out_rshift=s, relu_flag=True)
        assert np.array_equal(got, ref)
        assert np.array_equal(got, G.run_qconv(np.ascontiguousarray(x), wt, 1, pad, bias=b, rshift=s, relu=True))
    # (ii) a scale of its own for every member
    scales = [2.0 ** -11.3, 2.0 ** -10.1, 2.0 ** -12.6] if r == 3 else [2.0 ** -9.3, 2.0 ** -8.1, 2.0 ** -10.6]
    ms = [S.quantize_multiplier(v) for v in scales]
    mult = np.concatenate([np.full(kk, m, dtype=np.int32) for kk, (m, _) in zip(widths, ms)])
    rsh = np.concatenate([np.full(kk, sh, dtype=np.int32) for kk, (_, sh) in zip(widths, ms)])
    cat.fill_(-128)
    y2.fill_(-128)
    B.relay_qconv2d_combined(d, xv, xw.shape[-1], wp, bias, G.up(mult), G.up(rsh), 0, list(widths), ys, lds)
    torch.cuda.synchronize()
    outs = [G.from_nhwc(cat, cat.shape[-1])[:, :widths[0]], G.from_nhwc(cat, cat.shape[-1])[:, widths[0]:], G.from_nhwc(y2, widths[2])]
    for wt, b, (m, sh), got in zip(ws, bs, ms, outs):
        ref = S.qconv2d_requant_scaled(x, wt, stride=(1, 1), pad=(pad, pad), bias=b, mult=m, rshift=sh, relu_flag=True)
        assert np.array_equal(got, ref)

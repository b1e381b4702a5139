"""Layer tables and seeded generators: shapes, MAC counts, determinism.  No GPU."""
import numpy as np

from workloads import inputs, nets


def test_resnet18_table():
    ops = nets.resnet18()
    convs = [o for o in ops if o.kind == "conv"]
    assert len(convs) == 20
    shp = nets.trace_shapes(ops, 224, 224)
    assert shp["c1"] == (64, 112, 112) and shp["s1.in"] == (64, 56, 56)
    assert shp["l4.b1.out"] == (512, 7, 7) and shp["logits"] == (1000, 1, 1)
    macs = nets.macs_per_image(nets.resnet18(with_dense=False), 224, 224)
    assert abs(macs / 1e6 - 1813.6) < 0.1                      # standard ResNet-18 conv MACs
    assert sum(1 for o in convs if o.res) == 8 and sum(1 for o in convs if not o.relu) == 3


def test_mobilenet_v1_table():
    ops = nets.mobilenet_v1()
    assert sum(1 for o in ops if o.kind == "dwconv") == 13
    shp = nets.trace_shapes(ops, 224, 224)
    assert shp["b13.out"] == (1024, 7, 7)
    macs = nets.macs_per_image(nets.mobilenet_v1(with_dense=False), 224, 224)
    assert abs(macs / 1e6 - 567.7) < 0.1
    dw = sum(shp[o.dst][0] * shp[o.dst][1] * shp[o.dst][2] * 9 for o in ops if o.kind == "dwconv")
    assert abs(dw / 1e6 - 17.4) < 0.1


def test_generators_are_seeded_and_typed():
    op = nets.resnet18()[0]
    a = inputs.layer_params(op, 3, 0, "f16")
    b = inputs.layer_params(op, 3, 0, "f16")
    assert a["w"].dtype == np.float16 and np.array_equal(a["w"], b["w"]) and a["scale"].dtype == np.float32
    assert abs(float(a["w"].astype(np.float64).std()) - (2 / 147) ** 0.5) < 0.01
    q = inputs.layer_params(op, 4, 0, "i8")
    assert q["w"].dtype == np.int8 and q["w"].min() >= -127 and "scale" not in q
    x = inputs.image(1, 1, 3, 32, 32, "f32")
    assert x.dtype == np.float32 and x.min() >= -1 and x.max() < 1
    assert inputs.default_out_rshift(576) == 12 and inputs.default_out_rshift(147) == 11


def test_int8_chain_recipe_keeps_activations_alive():
    """The closed-form shift rule must neither kill nor saturate a 20-conv int8 chain,
    otherwise end-to-end parity would compare constants."""
    from oracle.stack import run_quantized
    ops = nets.resnet18(with_dense=False)
    params = inputs.net_params(ops, 4, "i8")
    shifts = inputs.chain_shifts(ops)
    t = run_quantized(ops, params, shifts, inputs.image(4, 1, 3, 224, 224, "i8"))
    for op in ops:
        if op.kind != "conv":
            continue
        y = t[op.dst].astype(np.int64)
        assert (np.abs(y) == 127).mean() < 0.5, op.name
        assert (y != 0).mean() > 0.3, op.name
        assert y.min() >= -127


def test_dqn_table():
    """The published deep Q-network shapes: 84 -> 20 -> 9 -> 7, 3136 inputs to the first dense layer."""
    ops = nets.dqn()
    shp = nets.trace_shapes(ops, 84, 84, 4)
    assert [shp[o.dst] for o in ops] == [(32, 20, 20), (64, 9, 9), (64, 7, 7), (512, 1, 1), (18, 1, 1)]
    assert ops[3].cin == 64 * 7 * 7
    assert nets.macs_per_image(ops, 84, 84, 4) == 32 * 400 * 256 + 64 * 81 * 512 + 64 * 49 * 576 + 3136 * 512 + 512 * 18


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more ends with a message and a non-zero status
    before anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)

#!/usr/bin/env python3
"""Benchmark of the fused-operator hot path on one MI355X.

A step = one pass of the full ResNet-18 stack (layout conversion, 20 fused convs, both
pools, fused dense) over one batch of 32 synthetic 3x224x224 fp16 images, every kernel
coming from librelayfused.so.  Inputs and packed filters are resident in HBM before the
timed region; filter packing and batch-norm folding are compile-time work and untimed.

Prints ONE JSON line.  `value` = contraction FLOP (2*MAC of the convs and the dense) per
second over the whole step.  `roofline` covers the implicit-GEMM kernel variant that
takes the most time; `cpu_baseline` is the CPU oracle timed on this host on a bounded
sample.  `extra` holds per-layer figures and the int8 / MobileNet configurations.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"f16": 2500.0, "i8": 5000.0}     # dense MFMA peaks, TFLOP/s and TOP/s
HBM_PEAK_GBS = 8000.0


def _layer_table(net, ops, batch, reps, trials):
    """Per-launch duration of every call of the network: `reps` back-to-back launches (one
    graph replay) between two events on the launch stream, median of `trials`."""
    import torch
    from paper_1904_08368_amd import binding as B
    rows = []
    shp_in = {}
    for (fn, args), name in zip(net.calls, net.call_names):
        for _ in range(3):
            fn(*args)
        torch.cuda.synchronize()
        # the launches are replayed from a HIP graph so that their spacing is set by the GPU,
        # not by the Python call overhead (which exceeds the duration of the small layers)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(reps):
                fn(*args)
        g.replay()
        ts = []
        for _ in range(trials):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            e1.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3 / reps)      # us per launch
        del g
        row = {"name": name, "us": statistics.median(ts)}
        d = args[0]
        if fn in (B.relay_fused_conv2d_bias_bn_relu, B.relay_qconv2d_requant, B.relay_fused_dwconv_bias_relu):
            ho, wo = B.relay_conv2d_out_shape(d)
            es = 2 if d.dtype == B.RELAY_F16 else 1
            if fn is not B.relay_fused_dwconv_bias_relu:
                # logical reduction length: padded input channels of the stem carry zeros
                op = next(o for o in ops if o.name == name)
                macs = d.n * ho * wo * d.k * op.cin * d.r * d.s
                row["gflop"] = 2 * macs / 1e9
                row["kernel"] = B.relay_conv2d_kernel_name(d)
                byts = (d.n * d.h * d.w * op.cin + d.n * ho * wo * d.k * (2 if (d.flags & B.HAS_RESIDUAL) else 1)
                        + d.k * op.cin * d.r * d.s) * es
                row["mbytes"] = byts / 1e6
            else:   # depthwise: input + output + filters
                row["gflop"] = 2 * d.n * ho * wo * d.c * 9 / 1e9
                row["kernel"] = "dwconv3x3_f16_kernel"
                row["mbytes"] = (d.n * d.h * d.w * d.c + d.n * ho * wo * d.c + 9 * d.c) * es / 1e6
            row["tflops"] = row["gflop"] / row["us"] * 1e3           # GFLOP/us = 1000 TFLOP/s
            row["gbs"] = row["mbytes"] / row["us"] * 1e3              # MB/us = 1000 GB/s
            _bounds(row, d.dtype == B.RELAY_I8, fn is B.relay_fused_dwconv_bias_relu)
        elif fn is B.relay_fused_dwconv_pwconv:
            # a depthwise conv and its 1x1 conv in one launch: both convs' FLOP; input + output + both filter sets
            ho, wo = B.relay_conv2d_out_shape(d)
            k = args[6]
            row["gflop"] = 2 * d.n * ho * wo * d.c * (9 + k) / 1e9
            row["kernel"] = B.relay_dwconv_pwconv_kernel_name(d, k)
            row["mbytes"] = (d.n * d.h * d.w * d.c + d.n * ho * wo * k + 9 * d.c + k * d.c) * 2 / 1e6
            row["tflops"] = row["gflop"] / row["us"] * 1e3
            row["gbs"] = row["mbytes"] / row["us"] * 1e3
            _bounds(row, False, False)
            row["frac_hbm"] = row["gbs"] / HBM_PEAK_GBS
        elif fn is B.relay_fused_conv2d_first_layer:
            # the first layer read straight from the NCHW image: plain vector arithmetic, bound by its tensors
            ho, wo = B.relay_conv2d_out_shape(d)
            row["gflop"] = 2 * d.n * ho * wo * d.k * d.c * 9 / 1e9
            row["kernel"] = "conv_first_kernel"
            row["mbytes"] = (d.n * d.h * d.w * d.c + d.n * ho * wo * d.k + d.k * d.c * 9) * 2 / 1e6
            row["tflops"] = row["gflop"] / row["us"] * 1e3
            row["gbs"] = row["mbytes"] / row["us"] * 1e3
            _bounds(row, False, True)
        elif fn in (B.relay_fused_conv2d_bn_relu_maxpool, B.relay_qconv2d_requant_maxpool):
            # the conv with its max pool in the same launch: the conv's FLOP, input + pooled output + filters
            ho, wo = B.relay_conv2d_out_shape(d)
            es = 2 if d.dtype == B.RELAY_F16 else 1
            op = next(o for o in ops if o.name == name.split("+")[0])
            row["gflop"] = 2 * d.n * ho * wo * d.k * op.cin * d.r * d.s / 1e9
            row["kernel"] = B.relay_conv2d_maxpool_kernel_name(d)
            row["mbytes"] = (d.n * d.h * d.w * op.cin + d.n * (ho // 2) * (wo // 2) * d.k + d.k * op.cin * d.r * d.s) * es / 1e6
            row["tflops"] = row["gflop"] / row["us"] * 1e3
            row["gbs"] = row["mbytes"] / row["us"] * 1e3
            _bounds(row, d.dtype == B.RELAY_I8, False)
        rows.append(row)
    return rows


def _bounds(row, is_i8, is_dw):
    """Roofline position of one layer: arithmetic intensity (FLOP per algorithmic byte), the
    fraction of the matrix-core peak, and the fraction of min(matrix-core peak, intensity x HBM
    peak), the bound that applies to the layer (a depthwise layer: the HBM peak alone)."""
    peak = PEAK["i8" if is_i8 else "f16"]
    row["ai"] = row["gflop"] * 1e3 / row["mbytes"]
    if is_dw:
        row["frac_hbm"] = row["gbs"] / HBM_PEAK_GBS
        row["frac_bound"] = row["frac_hbm"]
        return
    bound = min(peak, row["ai"] * HBM_PEAK_GBS / 1e3)          # TFLOP/s
    row["bound"] = "mfma" if bound == peak else "hbm"
    row["frac_mfma"] = row["tflops"] / peak
    row["frac_bound"] = row["tflops"] / bound


def _measured_ceilings():
    """The chip's measured ceilings on this machine: the register-only matrix-instruction loop and a
    streaming copy (library probes), timed with events over back-to-back launches."""
    import torch
    from paper_1904_08368_amd import binding as B
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    iters, wgs = 256, 2048
    res = {}
    for name, fn, work in (("mfma_f16_tflops", lambda: B.relay_probe_mfma(B.RELAY_F16, iters, wgs, out), 2.0 * 32 * 32 * 16 * 4 * iters * 4 * wgs / 1e12),
                           ("mfma_i8_tops", lambda: B.relay_probe_mfma(B.RELAY_I8, iters, wgs, out), 2.0 * 32 * 32 * 32 * 4 * iters * 4 * wgs / 1e12),
                           ("copy_gbs", lambda: B.relay_probe_copy(src, dst, src.numel()), 2.0 * src.numel() / 1e9)):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        e1.synchronize()
        res[name] = round(work / (e0.elapsed_time(e1) / 10 * 1e-3), 1)
    return res


def _layer_boundary_costs():
    """What a boundary between two dependent layers costs on this machine: as a kernel boundary (back-to-back
    empty launches replayed from a HIP graph) and as a barrier across a resident grid inside one launch
    (the library's probe: device-scope release + atomic arrival + bounded poll + acquire, every thread
    storing one word per round), for the grid sizes a batch-1 layer chain would use."""
    import torch
    from paper_1904_08368_amd import binding as B
    cells = torch.zeros(4, dtype=torch.int32, device="cuda")

    def timed(fn, reps):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(reps):
                fn()
        g.replay()
        ts = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            e1.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3 / reps)
        return statistics.median(ts)

    res = {"kernel_boundary_us": round(timed(lambda: B.relay_probe_grid_barrier(256, 0, 1, cells), 20), 2), "grid_barrier_us": {}}
    rounds = 100
    for wgs in (16, 64, 128, 256):
        data = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
        us = timed(lambda: B.relay_probe_grid_barrier(wgs, rounds, 1 << 22, cells, data), 4)
        res["grid_barrier_us"][str(wgs)] = round((us - res["kernel_boundary_us"]) / rounds, 2)
    torch.cuda.synchronize()
    res["waits_ran_out"] = int(cells[1].item())
    return res


def _dominant(rows, peak):
    """The conv kernel variant with the most time per step among `rows`: (name, roofline dict)."""
    by_kernel = {}
    for r in rows:
        if r.get("kernel", "").startswith(CONV_KERNELS):
            k = by_kernel.setdefault(r["kernel"], {"us": 0.0, "gflop": 0.0, "launches": 0, "layers": []})
            k["us"] += r["us"]
            k["gflop"] += r["gflop"]
            k["launches"] += 1
            k["layers"].append(r["name"])
    name, dom = max(by_kernel.items(), key=lambda kv: kv[1]["us"])
    achieved = dom["gflop"] / dom["us"] * 1e3
    return name, {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s" if peak == PEAK["f16"] else "TOP/s",
                  "frac": round(achieved / peak, 4), "traffic": None, "kernel": name, "launches_per_step": dom["launches"],
                  "avg_launch_us": round(dom["us"] / dom["launches"], 2), "gflop_per_launch": round(dom["gflop"] / dom["launches"], 3),
                  "layers": dom["layers"]}


KERNEL_SOURCES = ("conv_igemm_dma.hip", "conv_halo.hip", "dma_common.hpp", "igemm_common.hpp", "lds_dma.hpp", "rounding.hpp",
                  "kernels.hpp", "fastdiv.hpp")


CONV_KERNELS = ("igemm", "conv3x3_halo", "conv3x3_stream")      # name prefixes of the MFMA conv kernels in the per-layer table


def _kernel_source_digest():
    """sha256 over the sources the implicit-GEMM kernel is compiled from."""
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_1904_08368_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def _hbm_traffic(kernel_name):
    """HBM bytes per launch of `kernel_name` from the stored rocprofv3 counter summary
    (FETCH_SIZE and WRITE_SIZE passes, each scaled by the reading of a copy of known size).
    None when there is no summary for this kernel or the kernel sources have changed since."""
    path = os.path.join(ROOT, "profiles", kernel_name.split("<")[0] + "_resnet18_fp16_b32_hbm_traffic.md")
    if not os.path.exists(path):
        return None
    kv = {}
    with open(path) as fh:
        for line in fh:
            if line.startswith("    ") and ":" in line:
                k, v = line.strip().split(":", 1)
                kv[k.strip()] = v.strip()
    if kv.get("kernel") != kernel_name or kv.get("source_sha256") != _kernel_source_digest():
        return None
    fetch = float(kv["fetch_size_kib_per_launch"]) * float(kv["fetch_scale"])
    write = float(kv["write_size_kib_per_launch"]) * float(kv["write_scale"])
    return round((fetch + write) * 1024.0)


def _time_steps(net, steps, warmup, use_graph):
    import torch
    step = net.replay if use_graph else net.run
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-extra", action="store_true", help="skip the int8 / MobileNet / batch-1 sections")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--layer-reps", type=int, default=20)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a 256 MiB device-to-device copy 10 times: a kernel of known HBM traffic that "
                         "scales FETCH_SIZE / WRITE_SIZE counter readings of the same profiler run")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this library runs on ONE GPU; the path shards over the batch axis with no "
              "collective, but nothing here launches more than one rank.", file=sys.stderr)
        return 2

    import torch
    from paper_1904_08368_amd import binding as B
    from paper_1904_08368_amd.stack import FusedNet
    from workloads import inputs, nets

    B.lib()                                   # fail loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    use_graph = not a.no_graph

    # ------------------------------------------------ headline: ResNet-18 fp16, batch 32
    # the layer sequence is what the library's fusion extraction makes of the operator graph
    from paper_1904_08368_amd import fusion
    from workloads import graphs
    graph = graphs.resnet18()
    fusion.extract_groups(graph)               # (first call: library and ctypes set-up)
    t0 = time.perf_counter()
    for _ in range(100):
        groups = fusion.extract_groups(graph)
    fuse_us = (time.perf_counter() - t0) / 100 * 1e6
    ops = fusion.lower(graph, groups)
    params = inputs.net_params(ops, 3, "f16")
    net = FusedNet(ops, params, a.batch, 224, 224, "f16")
    net.load_input(inputs.image(3, a.batch, 3, 224, 224, "f16"))
    if use_graph:
        net.capture()
    sec = _time_steps(net, a.steps, a.warmup, use_graph)
    flop = 2.0 * nets.macs_per_image(ops, 224, 224) * a.batch
    value = flop / sec / 1e12

    rows = _layer_table(net, ops, a.batch, a.layer_reps, 5)
    dom_name, roofline = _dominant(rows, PEAK["f16"])
    roofline["traffic"] = _hbm_traffic(dom_name)
    ceil = _measured_ceilings()
    roofline["measured_peak"] = ceil["mfma_f16_tflops"]          # register-only matrix-instruction loop on this machine
    roofline["frac_of_measured_peak"] = round(roofline["achieved"] / ceil["mfma_f16_tflops"], 4)
    conv_us = sum(r["us"] for r in rows if r.get("kernel", "").startswith(CONV_KERNELS))
    conv_gf = sum(r["gflop"] for r in rows if r.get("kernel", "").startswith(CONV_KERNELS))

    out = {
        "metric": "resnet18_fp16_fused_conv_stack_tflops", "value": round(value, 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "configs[2]: full ResNet-18 stack (20 fused convs + pools + dense 512->1000), "
                               f"fp16 / fp32 accumulate, batch {a.batch}, 3x224x224, NHWC",
                   "batch": a.batch, "hip_graph": use_graph},
        "ms_per_img": round(sec * 1e3 / a.batch, 5),
        "roofline": roofline,
    }
    extra = {"measured_ceilings": ceil,
             "fusion_extraction": {"operators": len(graph.nodes), "groups": len(groups),
                                   "host_us_per_call_incl_marshalling": round(fuse_us, 1)},
             "conv_kernels_only_tflops": round(conv_gf / conv_us * 1e3, 2),
             "sum_of_kernel_us": round(sum(r["us"] for r in rows), 1),
             "layers": [{k: (round(v, 3) if isinstance(v, float) else v) for k, v in r.items()} for r in rows]}

    if not a.no_extra:
        extra["layer_boundary_costs"] = _layer_boundary_costs()
        # ---- the same stack with operator fusion switched off (the paper's fusion ablation, Section 5.2):
        #      contraction, bias add, scale/shift, residual add and relu as separate launches and tensors
        un = FusedNet(ops, params, a.batch, 224, 224, "f16", fused=False)
        un.load_input(inputs.image(3, a.batch, 3, 224, 224, "f16"))
        if use_graph:
            un.capture()
        usec = _time_steps(un, max(10, a.steps // 2), a.warmup, use_graph)
        extra["fusion_ablation"] = {"unfused_ms_per_step": round(usec * 1e3, 4), "fused_ms_per_step": round(sec * 1e3, 4),
                                    "launches_unfused": len(un.calls), "launches_fused": len(net.calls),
                                    "speedup_from_fusion": round(usec / sec, 3)}
        del un
        # ---- batch 1 latency of the same stack
        n1 = FusedNet(ops, params, 1, 224, 224, "f16")
        n1.load_input(inputs.image(3, 1, 3, 224, 224, "f16"))
        if use_graph:
            n1.capture()
        extra["resnet18_fp16_batch1_ms_per_img"] = round(_time_steps(n1, a.steps, a.warmup, use_graph) * 1e3, 4)
        del n1
        # ---- config 4: int8 stack, batch 16
        qops = fusion.fuse(graphs.resnet18(with_dense=False))
        qp = inputs.net_params(qops, 4, "i8")
        qn = FusedNet(qops, qp, 16, 224, 224, "i8", shifts=inputs.chain_shifts(qops))
        qn.load_input(inputs.image(4, 16, 3, 224, 224, "i8"))
        if use_graph:
            qn.capture()
        qsec = _time_steps(qn, a.steps, a.warmup, use_graph)
        qrows = _layer_table(qn, qops, 16, a.layer_reps, 3)
        qus = sum(r["us"] for r in qrows if "gflop" in r)
        qgf = sum(r["gflop"] for r in qrows if "gflop" in r)
        _, qroof = _dominant(qrows, PEAK["i8"])
        qroof["measured_peak"] = ceil["mfma_i8_tops"]
        qroof["frac_of_measured_peak"] = round(qroof["achieved"] / ceil["mfma_i8_tops"], 4)
        extra["resnet18_int8_batch16"] = {
            "roofline": qroof,
            "tops": round(2.0 * nets.macs_per_image(qops, 224, 224) * 16 / qsec / 1e12, 3),
            "ms_per_img": round(qsec * 1e3 / 16, 5), "conv_kernels_only_tops": round(qgf / qus * 1e3, 2),
            "frac_of_int8_mfma_peak": round(qgf / qus * 1e3 / PEAK["i8"], 4),
            "layers": [{k: (round(v, 3) if isinstance(v, float) else v) for k, v in r.items()} for r in qrows]}
        del qn
        q1 = FusedNet(qops, qp, 1, 224, 224, "i8", shifts=inputs.chain_shifts(qops))     # (config 4 names batch 1 too)
        q1.load_input(inputs.image(4, 1, 3, 224, 224, "i8"))
        if use_graph:
            q1.capture()
        extra["resnet18_int8_batch16"]["batch1_ms_per_img"] = round(_time_steps(q1, a.steps, a.warmup, use_graph) * 1e3, 4)
        del q1
        # ---- config 5: MobileNet-v1, batch 32
        mops = fusion.fuse(graphs.mobilenet_v1())
        mp = inputs.net_params(mops, 5, "f16")
        mn = FusedNet(mops, mp, 32, 224, 224, "f16")
        mn.load_input(inputs.image(5, 32, 3, 224, 224, "f16"))
        if use_graph:
            mn.capture()
        msec = _time_steps(mn, a.steps, a.warmup, use_graph)
        mrows = _layer_table(mn, mops, 32, a.layer_reps, 3)
        dw = [r for r in mrows if r.get("kernel") == "dwconv3x3_f16_kernel"]
        pw = [r for r in mrows if r.get("kernel", "").startswith("igemm")]
        dw_gbs = sum(r["mbytes"] for r in dw) / sum(r["us"] for r in dw) * 1e3
        blocks = [r for r in mrows if r.get("kernel", "").startswith("dwpw_fused")]
        # the same network with every block as two launches (what the one-launch blocks are measured against)
        mn2 = FusedNet(mops, mp, 32, 224, 224, "f16", fuse_dwpw=False)
        mn2.load_input(inputs.image(5, 32, 3, 224, 224, "f16"))
        if use_graph:
            mn2.capture()
        msec2 = _time_steps(mn2, a.steps, a.warmup, use_graph)
        del mn2
        mn1 = FusedNet(mops, mp, 1, 224, 224, "f16")
        mn1.load_input(inputs.image(5, 1, 3, 224, 224, "f16"))
        if use_graph:
            mn1.capture()
        msec1 = _time_steps(mn1, a.steps, a.warmup, use_graph)
        del mn1
        extra["mobilenet_v1_fp16_batch32"] = {
            "ms_per_img": round(msec * 1e3 / 32, 5),
            "ms_per_img_every_block_two_launches": round(msec2 * 1e3 / 32, 5),
            "batch1_ms_per_img": round(msec1 * 1e3, 4),
            "one_launch_blocks": [{"name": r["name"], "us": round(r["us"], 2), "gbs": round(r["gbs"], 1),
                                   "frac_of_hbm_peak": round(r["frac_hbm"], 4),
                                   "frac_of_measured_copy": round(r["gbs"] / ceil["copy_gbs"], 4)} for r in blocks],
            "tflops": round(2.0 * nets.macs_per_image(mops, 224, 224) * 32 / msec / 1e12, 3),
            "depthwise_gbs": round(dw_gbs, 1), "depthwise_frac_of_hbm_peak": round(dw_gbs / HBM_PEAK_GBS, 4),
            "depthwise_frac_of_measured_copy": round(dw_gbs / ceil["copy_gbs"], 4),
            "pointwise_tflops": round(sum(r["gflop"] for r in pw) / sum(r["us"] for r in pw) * 1e3, 2),
            "layers": [{k: (round(v, 3) if isinstance(v, float) else v) for k, v in r.items()} for r in mrows]}
        del mn
        # ---- a second large vision model of the paper's evaluation: the VGG-16 conv stack, batch 32
        vops = fusion.fuse(graphs.vgg16_convs())
        vp = inputs.net_params(vops, 6, "f16")
        vn = FusedNet(vops, vp, 32, 224, 224, "f16")
        vn.load_input(inputs.image(6, 32, 3, 224, 224, "f16"))
        if use_graph:
            vn.capture()
        vsec = _time_steps(vn, max(5, a.steps // 10), 2, use_graph)
        extra["vgg16_conv_stack_fp16_batch32"] = {
            "ms_per_img": round(vsec * 1e3 / 32, 5),
            "tflops": round(2.0 * nets.macs_per_image(vops, 224, 224) * 32 / vsec / 1e12, 2),
            "frac_of_fp16_mfma_peak": round(2.0 * nets.macs_per_image(vops, 224, 224) * 32 / vsec / 1e12 / PEAK["f16"], 4)}
        del vn
        # ---- the deep Q-network of the paper's vision benchmarks (built from its operator graph), batch 1 and 32
        dops = fusion.fuse(graphs.dqn())
        dp = inputs.net_params(dops, 7, "f16")
        dres = {}
        for b in (1, 32):
            dn = FusedNet(dops, dp, b, 84, 84, "f16", in_channels=4)
            dn.load_input(inputs.image(7, b, 4, 84, 84, "f16"))
            if use_graph:
                dn.capture()
            dsec = _time_steps(dn, a.steps, a.warmup, use_graph)
            dres[f"batch{b}_us_per_step"] = round(dsec * 1e6, 2)
            dres[f"batch{b}_tflops"] = round(2.0 * nets.macs_per_image(dops, 84, 84, 4) * b / dsec / 1e12, 3)
            dres["launches"] = len(dn.calls)
            del dn
        extra["dqn_fp16"] = dres
        # ---- parallel convolution combination (paper Section 4.4) on an Inception-shaped block, batch 32:
        #      the three 1x1 convs that read the block input as one launch instead of three
        iops = fusion.fuse(graphs.inception_block())
        ip = inputs.net_params(iops, 22, "f16")
        res = {}
        for tag, kw in (("separate", {}), ("combined", {"combine": True}),
                        ("combined_scale_folded", {"combine": True, "fold_scale": True})):
            inet = FusedNet(iops, ip, 32, 28, 28, "f16", in_channels=256, **kw)
            inet.load_input(inputs.image(22, 32, 256, 28, 28, "f16"))
            if use_graph:
                inet.capture()
            res[tag + "_ms"] = round(_time_steps(inet, a.steps, a.warmup, use_graph) * 1e3, 4)
            res[tag + "_launches"] = len(inet.calls)
            del inet
        res["speedup_from_combination"] = round(res["separate_ms"] / res["combined_ms"], 3)
        extra["parallel_conv_combination_inception_block_b32"] = res
        # ---- the same pass on the headline stack: each stride-2 3x3 conv and the 1x1 shortcut conv beside it
        #      as one launch (the shortcut as a centre-tap segment without relu); not the default, see the figures
        mnet = FusedNet(ops, params, a.batch, 224, 224, "f16", combine="windows")
        mnet.load_input(inputs.image(3, a.batch, 3, 224, 224, "f16"))
        if use_graph:
            mnet.capture()
        msec = _time_steps(mnet, a.steps, a.warmup, use_graph)
        extra["parallel_conv_combination_resnet18_shortcuts"] = {
            "separate_ms": round(sec * 1e3, 4), "separate_launches": len(net.calls),
            "merged_ms": round(msec * 1e3, 4), "merged_launches": len(mnet.calls)}
        del mnet

    if not a.no_cpu:
        # ---- the CPU oracle on this host: 4 of the 32 images, one pass of the same stack
        import oracle
        from oracle.stack import run_float
        nimg = a.batch
        xs = inputs.image(3, a.batch, 3, 224, 224, "f16")[:nimg]
        run_float(ops[:1], params[:1], xs[:1], "f16")            # load the library, page in
        passes = 3
        t0 = time.perf_counter()
        for _ in range(passes):
            run_float(ops, params, xs, "f16")
        dt = (time.perf_counter() - t0) / passes
        out["cpu_baseline"] = {"value": round(2.0 * nets.macs_per_image(ops, 224, 224) * nimg / dt / 1e12, 5),
                               "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"all {nimg} images of the batch, mean of {passes} passes of the full stack, fp64 loops",
                               "seconds": round(dt, 2)}
    if a.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        extra["copy_probe_bytes_each_way"] = 256 << 20
    out["extra"] = extra
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

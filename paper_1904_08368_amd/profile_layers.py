"""Run one representative layer of every kernel family a fixed number of times, for a profiler.

    rocprofv3 --kernel-trace --stats -d OUT -o kt --output-format csv -- python3 -m paper_1904_08368_amd.profile_layers
    rocprofv3 --kernel-trace --pmc <counters> -d OUT -o pmc --output-format csv -- python3 -m paper_1904_08368_amd.profile_layers

Every case launches its kernel WARM + REPS times through the C ABI on synthetic tensors of the
layer's real shape (ResNet-18 at batch 32 in fp16 and batch 16 in int8, MobileNet-v1 at batch 32),
then the two ceiling probes run.  One line per case goes to stdout (and, with --manifest FILE, to a
JSON file): the kernel's name as a trace prints it, the launch count, and the algorithmic work of
one launch, so that a trace can be cut into cases by kernel name and dispatch order.
"""
from __future__ import annotations

import argparse
import json
import sys

WARM, REPS = 3, 20


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--manifest", default=None)
    ap.add_argument("--only", default=None, help="comma-separated case names")
    a = ap.parse_args()
    import torch
    from . import binding as B
    B.lib()
    assert torch.cuda.is_available(), "needs a GPU"
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(190408368)
    rows = []

    def tensor(shape, i8):
        if i8:
            return torch.randint(-127, 128, shape, dtype=torch.int8, device=dev, generator=g)
        return torch.randn(shape, dtype=torch.float32, device=dev, generator=g).to(torch.float16)

    def run(name, kernel, fn, gflop, mbytes):
        if a.only and name not in a.only.split(","):
            return
        for _ in range(WARM + REPS):
            fn()
        torch.cuda.synchronize()
        rows.append({"case": name, "kernel": kernel, "launches": WARM + REPS, "gflop": gflop, "mbytes": mbytes})
        print(json.dumps(rows[-1]), flush=True)

    def conv_case(name, n, c, hw, k, r, stride, pad, i8, res, tile=-1):
        dtype = B.RELAY_I8 if i8 else B.RELAY_F16
        flags = B.flags_of(None, None if i8 else 1, 1 if res else None, True)
        d = B.conv_desc(n, c, hw, hw, k, r, r, stride, pad, dtype, B.RELAY_NHWC, flags)
        ho, wo = B.relay_conv2d_out_shape(d)
        x = tensor((n, hw, hw, c), i8)
        w = tensor((k, c, r, r), i8) if i8 else (tensor((k, c, r, r), False) * 0.05).to(torch.float16)
        wp = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=dev)
        B.relay_prepack_conv2d_weights(d, w, c, wp)
        y = torch.empty((n, ho, wo, k), dtype=x.dtype, device=dev)
        rr = tensor((n, ho, wo, k), i8) if res else None
        sc, sf = torch.ones(k, device=dev), torch.zeros(k, device=dev)
        B.relay_set_conv_tile(tile)
        try:
            kernel = B.relay_conv2d_kernel_name(d)

            def fn():
                B.relay_set_conv_tile(tile)
                try:
                    if i8:
                        B.relay_qconv2d_requant(d, x, wp, None, rr, 10 if res else 0, 10, y)
                    else:
                        B.relay_fused_conv2d_bias_bn_relu(d, x, wp, None, sc, sf, rr, y)
                finally:
                    B.relay_set_conv_tile(-1)
        finally:
            B.relay_set_conv_tile(-1)
        es = 1 if i8 else 2
        run(name, kernel, fn, 2.0 * n * ho * wo * k * c * r * r / 1e9,
            (n * hw * hw * c + n * ho * wo * k * (2 if res else 1) + k * c * r * r) * es / 1e6)

    # ---- the 3x3 stride-1 kernel (ResNet-18 stages 1-3), fp16 batch 32 and int8 batch 16
    conv_case("halo_f16_c64_56", 32, 64, 56, 64, 3, 1, 1, False, True)
    conv_case("halo_f16_c128_28", 32, 128, 28, 128, 3, 1, 1, False, False)
    conv_case("halo_f16_c256_14", 32, 256, 14, 256, 3, 1, 1, False, True)
    conv_case("halo_f16_c64_56_tile_128x64", 32, 64, 56, 64, 3, 1, 1, False, True, tile=100)   # (the default there is the 256 x 64 tile)
    conv_case("halo_f16_c256_56", 32, 256, 56, 256, 3, 1, 1, False, False)                      # (VGG-16's third stage: the 128 x 128 tile)
    conv_case("halo_i8_c64_56", 16, 64, 56, 64, 3, 1, 1, True, True)
    conv_case("halo_i8_c128_28", 16, 128, 28, 128, 3, 1, 1, True, False)
    # ---- the implicit-GEMM kernel: 64 x 64 tile with 256-byte chunks (stage 4), the stride-2 layers, 1x1 layers
    conv_case("igemm_f16_c512_7", 32, 512, 7, 512, 3, 1, 1, False, True, tile=15)   # (forced: the default there is the kernel of the next case)
    conv_case("halo_f16_c512_7", 32, 512, 7, 512, 3, 1, 1, False, True)
    conv_case("igemm_i8_c512_7", 16, 512, 7, 512, 3, 1, 1, True, True)
    conv_case("igemm_i8_c256_14", 16, 256, 14, 256, 3, 1, 1, True, False)
    conv_case("igemm_f16_s2_c64_56", 32, 64, 56, 128, 3, 2, 1, False, False)
    conv_case("pointwise_f16_c256_28", 32, 256, 28, 256, 1, 1, 0, False, False)
    conv_case("pointwise_f16_c512_14", 32, 512, 14, 512, 1, 1, 0, False, False)
    # ---- the persistent 3x3 kernel, forced (it is not chosen by default)
    conv_case("stream_f16_c64_56_v0", 32, 64, 56, 64, 3, 1, 1, False, True, tile=200)
    conv_case("stream_f16_c128_28_v0", 32, 128, 28, 128, 3, 1, 1, False, False, tile=200)

    # ---- the first layer with its max pool in one launch
    for i8, n in ((False, 32), (True, 16)):
        dtype = B.RELAY_I8 if i8 else B.RELAY_F16
        d = B.conv_desc(n, 3, 224, 224, 64, 7, 7, 2, 3, dtype, B.RELAY_NHWC4_PADDED, B.flags_of(None, None if i8 else 1, None, True))
        hp, wp_ = B.relay_nhwc4_padded_shape(d)
        x = tensor((n, hp, wp_, 4), i8)
        w = tensor((64, 3, 7, 7), i8) if i8 else (tensor((64, 3, 7, 7), False) * 0.1).to(torch.float16)
        wpk = torch.empty(B.relay_packed_weight_bytes(d), dtype=torch.uint8, device=dev)
        B.relay_prepack_conv2d_weights(d, w, 3, wpk)
        y = torch.empty((n, 56, 56, 64), dtype=x.dtype, device=dev)
        sc, sf = torch.ones(64, device=dev), torch.zeros(64, device=dev)
        fn = (lambda d=d, x=x, wpk=wpk, y=y: B.relay_qconv2d_requant_maxpool(d, x, wpk, None, 10, y)) if i8 else \
            (lambda d=d, x=x, wpk=wpk, y=y, sc=sc, sf=sf: B.relay_fused_conv2d_bn_relu_maxpool(d, x, wpk, None, sc, sf, y))
        es = 1 if i8 else 2
        run("stem_pool_" + ("i8" if i8 else "f16"), B.relay_conv2d_maxpool_kernel_name(d), fn,
            2.0 * n * 112 * 112 * 64 * 147 / 1e9, (n * 224 * 224 * 3 + n * 56 * 56 * 64 + 64 * 147) * es / 1e6)

    # ---- MobileNet-v1's first layer read from the NCHW image
    d = B.conv_desc(32, 3, 224, 224, 32, 3, 3, 2, 1, B.RELAY_F16, B.RELAY_NCHW, B.flags_of(None, 1, None, True))
    x = tensor((32, 3, 224, 224), False)
    wpk = torch.empty(B.relay_first_layer_packed_weight_bytes(d), dtype=torch.uint8, device=dev)
    B.relay_prepack_first_layer_weights(d, (tensor((32, 3, 3, 3), False) * 0.1).to(torch.float16), wpk)
    y = torch.empty((32, 112, 112, 32), dtype=torch.float16, device=dev)
    sc, sf = torch.ones(32, device=dev), torch.zeros(32, device=dev)
    run("first_f16_c3_224", "conv_first_kernel", lambda d=d, x=x, wpk=wpk, sc=sc, sf=sf, y=y: B.relay_fused_conv2d_first_layer(d, x, wpk, None, sc, sf, y),
        2.0 * 32 * 112 * 112 * 32 * 27 / 1e9, (32 * 224 * 224 * 3 + 32 * 112 * 112 * 32 + 32 * 27) * 2 / 1e6)

    # ---- depthwise 3x3 (MobileNet-v1, batch 32): the LDS-staged stride-1 kernel and the register-patch kernel
    for name, c, hw, stride, kernel in (("dw_s1_c128_56", 128, 56, 1, "dwconv3x3_s1_lds_kernel"), ("dw_s1_c64_112", 64, 112, 1, "dwconv3x3_s1_lds_kernel"),
                                        ("dw_s2_c128_56", 128, 56, 2, "dwconv3x3_f16_kernel"), ("dw_s1_c512_14", 512, 14, 1, "dwconv3x3_f16_kernel")):
        d = B.conv_desc(32, c, hw, hw, c, 3, 3, stride, 1, B.RELAY_F16, B.RELAY_NHWC, B.flags_of(None, 1, None, True))
        ho, wo = B.relay_conv2d_out_shape(d)
        x = tensor((32, hw, hw, c), False)
        w = tensor((c, 3, 3), False)
        wq = torch.empty((9, c), dtype=torch.float16, device=dev)
        B.relay_prepack_dwconv_weights(d, w, wq)
        y = torch.empty((32, ho, wo, c), dtype=torch.float16, device=dev)
        sc, sf = torch.ones(c, device=dev), torch.zeros(c, device=dev)
        run(name, kernel, lambda d=d, x=x, wq=wq, sc=sc, sf=sf, y=y: B.relay_fused_dwconv_bias_relu(d, x, wq, None, sc, sf, y),
            2.0 * 32 * ho * wo * c * 9 / 1e9, (32 * hw * hw * c + 32 * ho * wo * c + 9 * c) * 2 / 1e6)

    # ---- a depthwise conv and its 1x1 conv as one launch (MobileNet-v1 blocks 1-5 and 7, batch 32), and block 13, forced
    for name, c, hw, stride, k, tile in (("dwpw_b1_c32_112", 32, 112, 1, 64, -1), ("dwpw_b2_c64_112_s2", 64, 112, 2, 128, -1),
                                         ("dwpw_b3_c128_56", 128, 56, 1, 128, -1), ("dwpw_b4_c128_56_s2", 128, 56, 2, 256, -1),
                                         ("dwpw_b5_c256_28", 256, 28, 1, 256, -1), ("dwpw_b7_c512_14", 512, 14, 1, 512, -1),
                                         ("dwpw_b13_c1024_7_forced", 1024, 7, 1, 1024, 303)):
        d = B.conv_desc(32, c, hw, hw, c, 3, 3, stride, 1, B.RELAY_F16, B.RELAY_NHWC, B.flags_of(None, 1, None, True))
        ho, wo = B.relay_conv2d_out_shape(d)
        pflags = B.flags_of(None, 1, None, True)
        pd = B.conv_desc(32, c, ho, wo, k, 1, 1, 1, 0, B.RELAY_F16, B.RELAY_NHWC, pflags)
        x = tensor((32, hw, hw, c), False)
        wq = torch.empty((9, c), dtype=torch.float16, device=dev)
        B.relay_prepack_dwconv_weights(d, tensor((c, 3, 3), False), wq)
        wpk = torch.empty(B.relay_packed_weight_bytes(pd), dtype=torch.uint8, device=dev)
        B.relay_prepack_conv2d_weights(pd, (tensor((k, c, 1, 1), False) * 0.1).to(torch.float16), c, wpk)
        y = torch.empty((32, ho, wo, k), dtype=torch.float16, device=dev)
        sc, sf, psc, psf = torch.ones(c, device=dev), torch.zeros(c, device=dev), torch.ones(k, device=dev), torch.zeros(k, device=dev)
        B.relay_set_conv_tile(tile)
        try:
            kernel = B.relay_dwconv_pwconv_kernel_name(d, k)
        finally:
            B.relay_set_conv_tile(-1)

        def fn(d=d, x=x, wq=wq, sc=sc, sf=sf, k=k, pflags=pflags, wpk=wpk, psc=psc, psf=psf, y=y, tile=tile):
            B.relay_set_conv_tile(tile)
            try:
                B.relay_fused_dwconv_pwconv(d, x, wq, None, sc, sf, k, pflags, wpk, None, psc, psf, y)
            finally:
                B.relay_set_conv_tile(-1)
        run(name, kernel, fn, 2.0 * 32 * ho * wo * c * (9 + k) / 1e9, (32 * hw * hw * c + 32 * ho * wo * k + 9 * c + k * c) * 2 / 1e6)

    # ---- measured ceilings
    out = torch.zeros(1, dtype=torch.int32, device=dev)
    iters, wgs = 256, 256 * 8      # ~0.1 ms per launch: long enough to fill the chip, short enough for 32-bit counters
    run("ceiling_mfma_f16", "mfma_loop_kernel<false>", lambda: B.relay_probe_mfma(B.RELAY_F16, iters, wgs, out),
        2.0 * 32 * 32 * 16 * 4 * iters * 4 * wgs / 1e9, 0.0)
    run("ceiling_mfma_i8", "mfma_loop_kernel<true>", lambda: B.relay_probe_mfma(B.RELAY_I8, iters, wgs, out),
        2.0 * 32 * 32 * 32 * 4 * iters * 4 * wgs / 1e9, 0.0)
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    run("ceiling_copy_256MiB", "stream_copy_kernel", lambda: B.relay_probe_copy(src, dst, src.numel()), 0.0, 2 * src.numel() / 1e6)
    if a.manifest:
        with open(a.manifest, "w") as fh:
            json.dump(rows, fh, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())

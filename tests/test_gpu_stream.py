"""GPU parity of the persistent 3x3 / stride 1 kernel (workgroups that walk a list of tiles): every
variant, fp16 within tolerance and int8 bit for bit against the oracle, with and without a
residual operand, with grids small enough that a workgroup walks several tiles, and one layer at
its full benchmark size."""
import numpy as np
import pytest
import torch

import oracle as O

pytestmark = pytest.mark.gpu
STREAM = 200          # relay_set_conv_tile(STREAM + variant)
VARIANTS = (0, 1, 2)


@pytest.fixture(scope="module")
def G():
    from paper_1904_08368_amd import binding as B
    B.lib()
    assert torch.cuda.is_available()
    from tests import gpu_util
    return gpu_util


def _with_grid(B, wgs, fn):
    B.relay_set_conv_workgroups(wgs)
    try:
        return fn()
    finally:
        B.relay_set_conv_workgroups(0)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("wgs", [0, 3, 8])       # 3, 8: a workgroup walks up to four tiles
def test_stream_kernel_fp16(G, variant, wgs):
    from paper_1904_08368_amd import binding as B
    g = np.random.default_rng(300 + variant)
    for n, c, h, w, k, res in ((2, 64, 13, 17, 64, True), (3, 128, 9, 11, 72, False), (2, 64, 20, 20, 192, True),
                               (1, 32, 30, 7, 64, True), (2, 256, 7, 7, 64, False)):
        x = g.standard_normal((n, c, h, w)).astype(np.float16)
        wt = (g.standard_normal((k, c, 3, 3)) * np.sqrt(2.0 / (9 * c))).astype(np.float16)
        sc = (1 + 0.1 * g.standard_normal(k)).astype(np.float32)
        sf = (0.1 * g.standard_normal(k)).astype(np.float32)
        r = g.standard_normal((n, k, h, w)).astype(np.float16) if res else None
        ref = O.fused_conv2d(x, wt, stride=(1, 1), pad=(1, 1), scale=sc, shift=sf, residual=r, relu_flag=True)
        d = B.conv_desc(n, c, h, w, k, 3, 3, 1, 1, B.RELAY_F16, B.RELAY_NHWC, B.flags_of(None, sc, r, True))
        B.relay_set_conv_tile(STREAM + variant)
        try:
            assert "conv3x3_stream_kernel" in B.relay_conv2d_kernel_name(d)
        finally:
            B.relay_set_conv_tile(-1)
        got = _with_grid(B, wgs, lambda: G.run_conv_f16(x, wt, 1, 1, scale=sc, shift=sf, residual=r, relu=True,
                                                         tile=STREAM + variant))
        assert not np.isnan(got).any() and got.min() >= 0
        assert O.max_rel_err(got, ref) <= 1e-2, (n, c, h, w, k)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("wgs", [0, 3])
def test_stream_kernel_int8_bit_exact_and_repeatable(G, variant, wgs):
    from paper_1904_08368_amd import binding as B
    g = np.random.default_rng(320 + variant)
    for n, c, h, w, k, res in ((2, 64, 13, 17, 64, True), (3, 128, 9, 11, 72, False), (2, 256, 10, 10, 128, True)):
        x = g.integers(-127, 128, (n, c, h, w)).astype(np.int8)
        wt = g.integers(-127, 128, (k, c, 3, 3)).astype(np.int8)
        r = g.integers(-127, 128, (n, k, h, w)).astype(np.int8) if res else None
        b = g.integers(-5000, 5000, k).astype(np.int32)
        for s, relu in ((12, False), (31, True), (0, False)):
            ref = O.qconv2d_requant(x, wt, stride=(1, 1), pad=(1, 1), bias=b, residual=r, residual_lshift=min(s, 12) if res else 0,
                                    out_rshift=s, relu_flag=relu)
            for _ in range(2):
                got = _with_grid(B, wgs, lambda: G.run_qconv(x, wt, 1, 1, bias=b, residual=r, lshift=min(s, 12) if res else 0,
                                                             rshift=s, relu=relu, tile=STREAM + variant))
                assert np.array_equal(got, ref), (n, c, s)


def test_stream_kernel_full_size_layer_every_element(G):
    """64 -> 64 channels at 56 x 56 with a residual operand, batch 40: 509 tiles of 256 positions on
    256 workgroups (two tiles each, a ragged last one), every output element against the oracle."""
    from paper_1904_08368_amd import binding as B
    g = np.random.default_rng(340)
    n, c, hw, k = 40, 64, 56, 64
    x = g.standard_normal((n, c, hw, hw)).astype(np.float16)
    wt = (g.standard_normal((k, c, 3, 3)) * np.sqrt(2.0 / (9 * c))).astype(np.float16)
    sc = (1 + 0.1 * g.standard_normal(k)).astype(np.float32)
    sf = (0.1 * g.standard_normal(k)).astype(np.float32)
    r = g.standard_normal((n, k, hw, hw)).astype(np.float16)
    ref = O.fused_conv2d(x, wt, stride=(1, 1), pad=(1, 1), scale=sc, shift=sf, residual=r, relu_flag=True)
    for variant in (0, 2):
        got = G.run_conv_f16(x, wt, 1, 1, scale=sc, shift=sf, residual=r, relu=True, tile=STREAM + variant)
        assert O.max_rel_err(got, ref) <= 1e-2, variant


def test_stream_kernel_is_not_chosen_by_default(G):
    from paper_1904_08368_amd import binding as B
    for dtype, n in ((B.RELAY_F16, 32), (B.RELAY_I8, 16)):
        for c, hw in ((64, 56), (128, 28), (256, 14), (512, 7)):
            d = B.conv_desc(n, c, hw, hw, c, 3, 3, 1, 1, dtype, B.RELAY_NHWC, B.RELU)
            assert "stream" not in B.relay_conv2d_kernel_name(d)


def test_grid_barrier_probe_completes_and_its_bounded_wait_gives_up(G):
    """The probe behind the layer-boundary figures of the benchmark: with a generous poll limit every
    barrier completes, the counters come back to zero and every thread has counted every round; with a
    limit of one poll (forced from the host) the kernel still ends -- a wait that runs out raises the flag
    and the workgroups leave -- whatever the flag then says."""
    from paper_1904_08368_amd import binding as B
    cells = torch.zeros(4, dtype=torch.int32, device=G.DEV)
    data = torch.zeros(128 * 256, dtype=torch.float32, device=G.DEV)
    for _ in range(2):                                   # twice: the second launch starts from what the first left
        B.relay_probe_grid_barrier(128, 50, 1 << 22, cells, data)
        torch.cuda.synchronize()
        assert cells.tolist() == [0, 0, 0, 0]
    assert bool((data == 100).all())
    B.relay_probe_grid_barrier(256, 20, 1, cells, None)
    torch.cuda.synchronize()                             # returns: no wait is unbounded
    assert cells[1].item() in (0, 1)
    cells.zero_()
    B.relay_probe_grid_barrier(64, 5, 1 << 22, cells, None)
    torch.cuda.synchronize()
    assert cells.tolist() == [0, 0, 0, 0]

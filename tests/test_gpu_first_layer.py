"""GPU parity of the first-layer conv2d (NCHW image in, NHWC out, one launch) against the CPU oracle, and
against the two-launch route (padded NHWC4 copy + implicit-GEMM conv) it replaces."""
import numpy as np
import pytest
import torch

import oracle as O
from workloads import inputs

pytestmark = pytest.mark.gpu
TOL_F16 = 1e-2


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


def _case(seed, n, h, w, k):
    g = np.random.default_rng(inputs.BASE_SEED + 91000 + seed)
    x = g.standard_normal((n, 3, h, w)).astype(np.float16)
    wt = (g.standard_normal((k, 3, 3, 3)) * np.sqrt(2.0 / 27)).astype(np.float16)
    b = (0.1 * g.standard_normal(k)).astype(np.float32)
    sc = (1 + 0.1 * g.standard_normal(k)).astype(np.float32)
    sf = (0.1 * g.standard_normal(k)).astype(np.float32)
    return x, wt, b, sc, sf


# several blocks and a ragged last one, one-row and one-thread-per-row images, the widest and narrowest channel counts
SHAPES = [(2, 32, 32, 32), (1, 2, 8, 16), (3, 18, 40, 64), (1, 224, 224, 32), (5, 6, 8, 128), (2, 64, 72, 48)]


@pytest.mark.parametrize("shape", SHAPES)
def test_first_layer_matches_oracle(G, shape):
    n, h, w, k = shape
    x, wt, b, sc, sf = _case(h + k, n, h, w, k)
    want = O.fused_conv2d(x, wt, stride=(2, 2), pad=(1, 1), bias=b, scale=sc, shift=sf, relu_flag=True, out_dtype="f16")
    got = G.run_first_layer_f16(x, wt, bias=b, scale=sc, shift=sf, relu=True)
    assert got.shape == want.shape and not np.isnan(got).any()
    assert O.max_rel_err(got, want) <= TOL_F16
    assert got.min() >= 0
    # no tail at all: the bare contraction, negative values kept
    want0 = O.fused_conv2d(x, wt, stride=(2, 2), pad=(1, 1), out_dtype="f16")
    got0 = G.run_first_layer_f16(x, wt)
    assert O.max_rel_err(got0, want0) <= TOL_F16 and got0.min() < 0


def test_first_layer_taps_and_padding_are_where_they_belong(G):
    """One-hot filters: output channel j copies input (c, r, s) number j, so every tap, the zero padding on
    all four sides and the pixel-to-thread mapping are checked exactly (products with 1 and sums with 0)."""
    g = np.random.default_rng(inputs.BASE_SEED + 91500)
    x = g.standard_normal((2, 3, 12, 24)).astype(np.float16)
    wt = np.zeros((32, 3, 3, 3), dtype=np.float16)
    for j in range(27):
        wt[j, j // 9, (j % 9) // 3, j % 3] = 1
    got = G.run_first_layer_f16(x, wt)
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
    for j in range(27):
        c, r, s = j // 9, (j % 9) // 3, j % 3
        assert np.array_equal(got[:, j], xp[:, c, r:r + 12:2, s:s + 24:2]), (c, r, s)
    assert not got[:, 27:].any()


def test_first_layer_agrees_with_the_two_launch_route(G):
    x, wt, b, sc, sf = _case(7, 2, 56, 64, 32)
    one = G.run_first_layer_f16(x, wt, bias=b, scale=sc, shift=sf, relu=True)
    two = G.run_conv_f16(x, wt, 2, 1, bias=b, scale=sc, shift=sf, relu=True)
    assert O.max_rel_err(one, two) <= 2e-3      # same products, fp32 sums in another order

"""GPU parity of the 1x1-convolution GEMM kernel (HGC_PATH_POINTWISE) against the FP64 oracle, through the
C ABI's ordinary entry points with the path forced; same tolerance as every convolution:
|gpu - oracle| <= 4e-3 * sum|w*x| + 1e-3, integer-valued inputs exact.
"""
import numpy as np
import pytest

import paper_1901_00858_amd as hgc
from workloads import ConvLayer, make_integer_tensors, make_tensors, mobilenet_v1, resnet50

from gpu_helpers import assert_full, assert_points, run_layer, sample_points, say

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _forced():
    hgc.load()
    hgc.set_forced_path(hgc.PATH_POINTWISE)
    yield
    hgc.set_forced_path(hgc.PATH_AUTO)


#          N   C    H   W   M
SHAPES = [
    (2, 32, 8, 8, 32),          # one stage, one tile, 8-pixel chunks
    (3, 64, 14, 14, 96),        # 196 pixels an image: 4-pixel chunks, tiles straddle images, ragged rows of w
    (1, 128, 56, 56, 64),       # many pixel tiles of one image
    (5, 96, 7, 8, 40),          # 56 pixels an image, tile = several images, M below one tile
    (4, 160, 6, 6, 200),        # 36 pixels an image (4-pixel chunks), two row tiles, the second ragged
    (2, 256, 10, 12, 130),      # 8 stages
    (7, 32, 2, 2, 32),          # 4 pixels an image
    (1, 64, 1, 4, 33),          # a single chunk in all
    (9, 64, 14, 14, 256),       # 1764 pixels: 14 pixel tiles of 128, the last ragged, two row tiles
    (84, 64, 28, 28, 128),      # 65856 pixels: enough tiles for the wide (256-pixel) tile
    (42, 32, 56, 56, 64),       # the wide tile with 64 rows a workgroup (M <= 64), a single stage
    (32, 64, 28, 28, 300),      # 256 rows a workgroup, the second row tile ragged
    (8, 64, 56, 56, 64),        # 64 rows x 128 pixels a workgroup (the small shapes above take 64 x 64 tiles)
]


def _layer(t, bias=1, relu=1):
    N, C, H, W, M = t
    return ConvLayer("pw", N, C, H, W, M, 1, 1, 0, 1, bias, relu)


@pytest.mark.parametrize("t", SHAPES, ids=["x".join(map(str, s)) for s in SHAPES])
def test_shapes_full_tensor(oracle, t):
    for bias, relu, ws, packed in [(1, 1, False, False), (0, 0, True, False), (1, 0, True, True)]:
        L = _layer(t, bias, relu)
        plan = hgc.conv2d_plan(L, ws, packed).as_dict()
        assert plan["path"] == hgc.PATH_POINTWISE, plan
        say(f"[pw] {L} ws={ws} packed={packed} plan={plan}")
        x, w, b = make_tensors(L, seed=200 + bias)
        y = run_layer(L, x, w, b, use_ws=ws, packed=packed)
        assert_full(oracle, L, x, w, b, y)


@pytest.mark.parametrize("t", SHAPES[:7], ids=["x".join(map(str, s)) for s in SHAPES[:7]])
def test_integer_inputs_are_exact(oracle, t):
    L = _layer(t, 1, 0)
    x, w, b = make_integer_tensors(L, seed=9) if L.Kg * 8 + 8 <= 2048 else make_integer_tensors(L, seed=9, xmax=1, wmax=1)
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, b)
    for ws, packed in ((False, False), (True, True)):
        y = run_layer(L, x, w, b, use_ws=ws, packed=packed)
        assert np.array_equal(y.astype(np.float64), pre), f"{L} ws={ws} packed={packed}"


def test_layers_the_kernel_does_not_take_fall_back(oracle):
    """Forcing the path on layers outside its conditions leaves the ordinary choice in place."""
    for t, why in [((1, 200, 7, 7, 96, 1, 1, 0, 1), "49 pixels an image"), ((1, 36, 10, 10, 48, 1, 1, 0, 1), "C % 32"),
                   ((2, 32, 16, 16, 32, 1, 2, 0, 1), "stride 2"), ((2, 64, 14, 14, 96, 3, 1, 1, 1), "3x3"),
                   ((2, 64, 12, 12, 64, 1, 1, 0, 2), "groups")]:
        N, C, H, W, M, k, s, p, G = t
        L = ConvLayer("nopw", N, C, H, W, M, k, s, p, G, 1, 1)
        plan = hgc.conv2d_plan(L, True, False).as_dict()
        assert plan["path"] != hgc.PATH_POINTWISE, (why, plan)
        x, w, b = make_tensors(L, seed=3)
        assert_full(oracle, L, x, w, b, run_layer(L, x, w, b, use_ws=True))


def test_benchmark_layers_at_their_batch_sizes(oracle):
    """The 1x1 layers of the MobileNet- and ResNet-shaped stacks the kernel takes by itself (no forcing), at the
    batches the benchmark times, on sampled outputs."""
    hgc.set_forced_path(hgc.PATH_AUTO)
    taken = 0
    for cfg, layers in (("mobilenet_v1", mobilenet_v1(64)), ("resnet50", resnet50(32))):
        for L in layers:
            if L.k != 1:
                continue
            plan = hgc.conv2d_plan(L, True, True).as_dict()
            if plan["path"] != hgc.PATH_POINTWISE:
                continue
            taken += 1
            say(f"[pw-bench] {cfg} {L.name} plan={plan}")
            x, w, b = make_tensors(L, seed=11)
            y = run_layer(L, x, w, b, use_ws=True, packed=True)
            assert_points(oracle, L, x, w, b, y, sample_points(L, np.random.default_rng(5), 3000))
    assert taken >= 8

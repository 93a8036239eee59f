"""Pins for the max-pooling oracle (oracle/max_pool_oracle.c).

Caffe's MAX pooling (the paper keeps Caffe's layers, Sections 2 and 5): output size rounded up,
windows clipped to the image, padding never part of the maximum.  Pinned by a hand-worked
fixture, by a library routine (torch's max_pool2d with ceil_mode, float32 on FP16 values is exact),
by an independently written second form (padding with -inf, then strided windows), by closed forms
(monotone ramps: the window's last element; a 1x1 window is the identity; a window that covers
the image is the global maximum) and by the output sizes of the pooling layers of AlexNet-, VGG-
and ResNet-shaped nets.  A floor instead of a ceiling, zero padding taking part in the maximum,
swapped axes or a stride applied to the wrong axis each fail at least one of them.
"""
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _rand(shape, seed):
    return np.random.default_rng(seed).normal(0, 1, size=shape).astype(np.float16)


def test_hand_worked_fixture(oracle):
    fx = json.load(open(os.path.join(HERE, "golden", "hand_worked_max_pool.json")))
    x = np.array(fx["x"], dtype=np.float16)
    assert np.array_equal(oracle.max_pool_forward((1, 1, 5, 5, 2, 2, 0), x), np.array(fx["k2_s2_p0"], dtype=np.float16))
    assert np.array_equal(oracle.max_pool_forward((1, 1, 5, 5, 3, 2, 1), x), np.array(fx["k3_s2_p1"], dtype=np.float16))


@pytest.mark.parametrize("k,s,p", [(2, 2, 0), (3, 2, 0), (3, 2, 1), (3, 1, 1), (2, 2, 1), (3, 3, 0), (5, 2, 2), (2, 1, 0), (4, 3, 1)])
@pytest.mark.parametrize("shape", [(1, 1, 5, 5), (2, 3, 7, 9), (1, 2, 12, 6), (2, 2, 13, 13)])
def test_against_torch_ceil_mode(oracle, shape, k, s, p):
    import torch
    x = _rand(shape, 1)
    y = oracle.max_pool_forward(shape + (k, s, p), x)
    t = torch.nn.functional.max_pool2d(torch.from_numpy(x).float(), k, s, p, ceil_mode=True).numpy()
    assert y.shape == t.shape
    assert np.array_equal(y.astype(np.float32), t)


@pytest.mark.parametrize("k,s,p", [(2, 2, 0), (3, 2, 1), (3, 2, 0), (5, 3, 2)])
def test_against_minus_infinity_padding(oracle, k, s, p):
    """Second form: pad with -inf on all sides (far side generously), then take plain strided windows."""
    shape = (2, 2, 9, 11)
    x = _rand(shape, 2)
    ho, wo = oracle.max_pool_shape(shape + (k, s, p))
    big = np.full((2, 2, 9 + 2 * p + k + s, 11 + 2 * p + k + s), -np.inf)
    big[:, :, p:p + 9, p:p + 11] = x.astype(np.float64)
    ref = np.empty((2, 2, ho, wo))
    for oh in range(ho):
        for ow in range(wo):
            ref[:, :, oh, ow] = big[:, :, oh * s:oh * s + k, ow * s:ow * s + k].max(axis=(2, 3))
    assert np.all(np.isfinite(ref))                      # every window holds at least one real value
    assert np.array_equal(oracle.max_pool_forward(shape + (k, s, p), x).astype(np.float64), ref)


def test_closed_forms(oracle):
    H, W = 9, 10
    ramp = (np.arange(H)[:, None] * 16 + np.arange(W)[None, :]).astype(np.float16).reshape(1, 1, H, W)
    y = oracle.max_pool_forward((1, 1, H, W, 3, 2, 0), ramp)
    ho, wo = y.shape[2:]
    for oh in range(ho):                                  # increasing along both axes: the window's last element
        for ow in range(wo):
            assert y[0, 0, oh, ow] == 16 * min(2 * oh + 2, H - 1) + min(2 * ow + 2, W - 1)
    x = _rand((2, 3, 6, 7), 3)
    assert np.array_equal(oracle.max_pool_forward((2, 3, 6, 7, 1, 1, 0), x), x)
    g = oracle.max_pool_forward((2, 3, 6, 6, 6, 1, 0), x[:, :, :, :6])
    assert g.shape == (2, 3, 1, 1) and np.array_equal(g[:, :, 0, 0], x[:, :, :, :6].max(axis=(2, 3)))
    neg = -np.abs(_rand((1, 1, 5, 5), 4)) - np.float16(1.0)
    assert np.all(oracle.max_pool_forward((1, 1, 5, 5, 3, 2, 1), neg) < 0)       # padding is not a zero candidate


def test_output_sizes_of_known_networks(oracle):
    assert oracle.max_pool_shape((1, 96, 55, 55, 3, 2, 0)) == (27, 27)      # AlexNet pool1
    assert oracle.max_pool_shape((1, 256, 13, 13, 3, 2, 0)) == (6, 6)       # AlexNet pool5
    assert oracle.max_pool_shape((1, 64, 224, 224, 2, 2, 0)) == (112, 112)  # VGG-16 pool1
    assert oracle.max_pool_shape((1, 512, 14, 14, 2, 2, 0)) == (7, 7)       # VGG-16 pool5
    assert oracle.max_pool_shape((1, 64, 112, 112, 3, 2, 0)) == (56, 56)    # ResNet (Caffe) pool1: rounding up
    assert oracle.max_pool_shape((1, 64, 112, 112, 3, 2, 1)) == (57, 57)    # with pad 1 Caffe rounds up to 57
    assert oracle.max_pool_shape((1, 1, 4, 4, 2, 2, 1)) == (3, 3)
    assert oracle.max_pool_shape((1, 1, 3, 3, 2, 2, 1)) == (2, 2)           # a third window would start at 2*2 - 1 = 3, beyond the image: dropped
    for bad in [(1, 1, 4, 4, 2, 2, 2), (1, 1, 4, 4, 0, 1, 0), (1, 1, 1, 1, 3, 1, 0), (0, 1, 4, 4, 2, 2, 0)]:
        with pytest.raises(ValueError):
            oracle.max_pool_shape(bad)


def test_axes_and_planes_are_kept_apart(oracle):
    x = _rand((2, 3, 8, 6), 5)
    y = oracle.max_pool_forward((2, 3, 8, 6, 2, 2, 0), x)
    assert y.shape == (2, 3, 4, 3)
    yt = oracle.max_pool_forward((2, 3, 6, 8, 2, 2, 0), np.ascontiguousarray(x.transpose(0, 1, 3, 2)))
    assert np.array_equal(yt, y.transpose(0, 1, 3, 2))
    z = x.copy()
    z[1, 2] += np.float16(100.0)
    yz = oracle.max_pool_forward((2, 3, 8, 6, 2, 2, 0), z)
    assert np.array_equal(yz[0], y[0]) and np.array_equal(yz[1, :2], y[1, :2]) and np.all(yz[1, 2] > y[1, 2])

"""Pins for the inner-product oracle (oracle/inner_product_oracle.c).

The layer is pre[n][m] = b[m] + sum_k w[m][k] x[n][k] (BVLC Caffe's inner product, kept by
the paper: Sections 2 and 5; Section 3.1 names it as an accumulation-heavy layer).  Pinned by a
hand-worked fixture, by a library routine (numpy's float64 matrix product), by the special cases
that reduce it to the separately pinned convolution oracle (a convolution whose kernel covers the
whole image; a 1x1 convolution on a 1x1 image), by closed forms and by the invariants of the
definition.  A transposed operand, a dropped or doubled bias, a wrong stride between rows or a
bias inside the magnitude each fail at least one of them.
"""
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _rand(shape, seed):
    rng = np.random.default_rng(seed)
    return rng.uniform(-2, 2, size=shape).astype(np.float16)


def test_hand_worked_fixture(oracle):
    fx = json.load(open(os.path.join(HERE, "golden", "hand_worked_inner_product.json")))
    x = np.array(fx["x"], dtype=np.float16)
    w = np.array(fx["w"], dtype=np.float16)
    b = np.array(fx["b"], dtype=np.float16)
    pre, mag = oracle.inner_product_forward((2, 3, 4, 1, 0), x, w, b)
    assert np.array_equal(pre, np.array(fx["pre"], dtype=np.float64))
    assert np.array_equal(mag, np.array(fx["mag"], dtype=np.float64))
    pre0, mag0 = oracle.inner_product_forward((2, 3, 4, 0, 0), x, w, None)
    assert np.array_equal(pre0, np.array(fx["pre_without_bias"], dtype=np.float64))
    assert np.array_equal(mag0, mag)


@pytest.mark.parametrize("N,K,M", [(1, 1, 1), (1, 37, 5), (3, 64, 7), (5, 129, 33), (2, 1000, 3)])
def test_against_numpy_matrix_product(oracle, N, K, M):
    x, w, b = _rand((N, K), 1), _rand((M, K), 2), _rand((M,), 3)
    pre, mag = oracle.inner_product_forward((N, K, M, 1, 0), x, w, b)
    x64, w64, b64 = x.astype(np.float64), w.astype(np.float64), b.astype(np.float64)
    ref = x64 @ w64.T + b64[None, :]
    refmag = np.abs(x64) @ np.abs(w64).T
    # FP64 sums of exact products in two different orders: a few ulps of the magnitude
    assert np.all(np.abs(pre - ref) <= 1e-13 * (refmag + 1))
    assert np.all(np.abs(mag - refmag) <= 1e-13 * (refmag + 1))


@pytest.mark.parametrize("C,H,W,M", [(3, 4, 4, 5), (2, 6, 6, 4), (8, 1, 1, 6), (4, 3, 3, 3)])
def test_equals_a_convolution_whose_kernel_covers_the_image(oracle, C, H, W, M):
    """x[n] flattened in C, H, W order is exactly the patch a k = H = W convolution reads."""
    N = 2
    x = _rand((N, C, H, W), 4)
    w = _rand((M, C, H, W), 5)
    b = _rand((M,), 6)
    pre_c, mag_c = oracle.conv2d_forward((N, C, H, W, M, H, 1, 0, 1, 1, 0), x, w, b)
    pre_i, mag_i = oracle.inner_product_forward((N, C * H * W, M, 1, 0), x.reshape(N, -1), w.reshape(M, -1), b)
    assert pre_c.shape == (N, M, 1, 1)
    assert np.array_equal(pre_c.reshape(N, M), pre_i)          # same products, same order of summation
    assert np.array_equal(mag_c.reshape(N, M), mag_i)


def test_closed_forms(oracle):
    N, K, M = 3, 50, 4
    ones_x, ones_w = np.ones((N, K), np.float16), np.ones((M, K), np.float16)
    b = np.arange(M).astype(np.float16)
    pre, mag = oracle.inner_product_forward((N, K, M, 1, 0), ones_x, ones_w, b)
    assert np.array_equal(pre, K + np.tile(np.arange(M, dtype=np.float64), (N, 1)))
    assert np.array_equal(mag, np.full((N, M), float(K)))
    # one-hot x picks a column of w: catches a transposed weight matrix
    w = _rand((M, K), 7)
    x = np.zeros((N, K), np.float16)
    cols = [0, 17, K - 1]
    for n, c in enumerate(cols):
        x[n, c] = 1
    pre, _ = oracle.inner_product_forward((N, K, M, 0, 0), x, w, None)
    for n, c in enumerate(cols):
        assert np.array_equal(pre[n], w[:, c].astype(np.float64))


def test_linearity_and_bias(oracle):
    N, K, M = 2, 33, 5
    x1, x2, w, b = _rand((N, K), 8), _rand((N, K), 9), _rand((M, K), 10), _rand((M,), 11)
    # keep x1 + x2 exactly representable: small integers over 8
    x1 = (np.round(x1.astype(np.float64) * 8) / 8).astype(np.float16)
    x2 = (np.round(x2.astype(np.float64) * 8) / 8).astype(np.float16)
    p1, _ = oracle.inner_product_forward((N, K, M, 0, 0), x1, w, None)
    p2, _ = oracle.inner_product_forward((N, K, M, 0, 0), x2, w, None)
    p12, _ = oracle.inner_product_forward((N, K, M, 0, 0), (x1 + x2).astype(np.float16), w, None)
    assert np.allclose(p12, p1 + p2, rtol=0, atol=1e-12)
    pb, mb = oracle.inner_product_forward((N, K, M, 1, 0), x1, w, b)
    p0, m0 = oracle.inner_product_forward((N, K, M, 0, 0), x1, w, None)
    assert np.allclose(pb - p0, b.astype(np.float64)[None, :], rtol=0, atol=1e-12)   # added exactly once
    assert np.array_equal(mb, m0)                                                      # bias is not a tap


def test_integer_inputs_give_exact_integers(oracle):
    rng = np.random.default_rng(12)
    N, K, M = 4, 300, 6
    x = rng.integers(-4, 5, size=(N, K)).astype(np.float16)
    w = rng.integers(-2, 3, size=(M, K)).astype(np.float16)
    b = rng.integers(-8, 9, size=(M,)).astype(np.float16)
    pre, _ = oracle.inner_product_forward((N, K, M, 1, 0), x, w, b)
    ref = x.astype(np.int64) @ w.astype(np.int64).T + b.astype(np.int64)[None, :]
    assert np.array_equal(pre, ref.astype(np.float64))


def test_bad_descriptors_are_rejected(oracle):
    x, w = np.zeros((1, 4), np.float16), np.zeros((2, 4), np.float16)
    for d in [(0, 4, 2, 0, 0), (1, 0, 2, 0, 0), (1, 4, 0, 0, 0), (1, 4, 2, 2, 0), (1, 4, 2, 0, 3), (1, 4, 2)]:
        with pytest.raises(ValueError):
            oracle.inner_product_forward(d, x, w, None)
    with pytest.raises(ValueError):
        oracle.inner_product_forward((1, 4, 2, 1, 0), x, w, None)       # bias without b
    with pytest.raises(ValueError):
        oracle.inner_product_forward((1, 5, 2, 0, 0), x, w, None)       # sizes do not match

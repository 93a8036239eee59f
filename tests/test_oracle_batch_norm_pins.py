"""Pins for the batch-norm oracle (oracle/batch_norm_oracle.c).

The layer is BVLC Caffe's batch norm, kept by the paper (Sections 2 and 5): per channel, the mean
and the biased variance over (n, h, w), then y = gamma (x - mean) / sqrt(var + eps) + beta.
Section 3.1 describes how the FP16 engine reaches these two accumulations without leaving FP16's
range (mean of group means; a power-of-two scale around the squares); both change rounding only,
so the oracle is the definition itself.  Pinned by a hand-worked fixture, by a library routine
(numpy's float64 mean and var), by closed forms (an arithmetic progression, two-valued data), by
the invariants of the definition (zero mean and var/(var+eps) second moment of the output,
invariance under x -> a x + b, independence of channels) and by stored-statistics cases.  A
channel/image transposition, the unbiased variance, eps outside the root, a dropped beta or a
gamma applied after beta each fail at least one of them.  The last tests replay the paper's two
devices in emulated FP16 arithmetic, to show that the reading taken of them does what the paper
says they do.
"""
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _rand(shape, seed, loc=0.0, scale=1.0):
    rng = np.random.default_rng(seed)
    return rng.normal(loc, scale, size=shape).astype(np.float16)


def test_hand_worked_fixture(oracle):
    fx = json.load(open(os.path.join(HERE, "golden", "hand_worked_batch_norm.json")))
    N, C, H, W = fx["shape"]
    x = np.array(fx["x"], dtype=np.float16)
    pre, mag, mean, var = oracle.batch_norm_forward((N, C, H, W, 0, 0, 0), x, eps=fx["eps"])
    assert np.array_equal(mean, np.array(fx["mean"], dtype=np.float64))
    assert np.array_equal(var, np.array(fx["var"], dtype=np.float64))
    assert np.array_equal(pre, np.array(fx["pre"], dtype=np.float64))
    assert np.array_equal(mag, np.array(fx["mag"], dtype=np.float64))
    pre, mag, _, _ = oracle.batch_norm_forward((N, C, H, W, 0, 1, 0), x, eps=fx["eps"],
                                               gamma=fx["gamma"], beta=fx["beta"])
    assert np.array_equal(pre, np.array(fx["pre_scale"], dtype=np.float64))
    assert np.array_equal(mag, np.array(fx["mag_scale"], dtype=np.float64))
    pre, _, mean, var = oracle.batch_norm_forward((N, C, H, W, 1, 0, 0), x, eps=fx["eps"], mean=fx["mean_in"],
                                                  var=fx["var_in"], stat_scale=fx["stat_scale"])
    assert np.array_equal(mean, np.array([1.0, 4.0])) and np.array_equal(var, np.array([9.0, 2.0]))
    assert np.array_equal(pre, np.array(fx["pre_global"], dtype=np.float64))


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (1, 3, 5, 7), (4, 2, 3, 3), (3, 5, 1, 9), (2, 7, 6, 4)])
def test_against_numpy_mean_and_var(oracle, shape):
    N, C, H, W = shape
    x = _rand(shape, 11, loc=1.5, scale=2.0)
    g = np.linspace(0.5, 2.0, C).astype(np.float32)
    b = np.linspace(-1.0, 1.0, C).astype(np.float32)
    eps = 1e-3
    pre, mag, mean, var = oracle.batch_norm_forward((N, C, H, W, 0, 1, 0), x, eps=eps, gamma=g, beta=b)
    xd = x.astype(np.float64)
    m = xd.mean(axis=(0, 2, 3))
    v = xd.var(axis=(0, 2, 3))                      # numpy's default is the biased variance
    assert np.allclose(mean, m, rtol=0, atol=1e-13)
    assert np.allclose(var, v, rtol=1e-13, atol=1e-13)
    sd = np.sqrt(v + eps)
    ref = g.astype(np.float64)[None, :, None, None] * (xd - m[None, :, None, None]) / sd[None, :, None, None] \
        + b.astype(np.float64)[None, :, None, None]
    assert np.allclose(pre, ref, rtol=1e-12, atol=1e-12)
    refmag = np.abs(g.astype(np.float64))[None, :, None, None] * (np.abs(xd) + np.abs(m)[None, :, None, None]) \
        / sd[None, :, None, None] + np.abs(b.astype(np.float64))[None, :, None, None]
    assert np.allclose(mag, refmag, rtol=1e-12, atol=1e-12)


def test_arithmetic_progression_closed_form(oracle):
    """0, 1, ..., L-1 spread over images and pixels: mean (L-1)/2, variance (L^2-1)/12."""
    N, H, W = 4, 4, 8
    L = N * H * W
    x = np.zeros((N, 2, H, W), dtype=np.float16)
    x[:, 0] = np.arange(L, dtype=np.float64).reshape(N, H, W)
    x[:, 1] = 3.0                                     # a constant neighbour channel
    _, _, mean, var = oracle.batch_norm_forward((N, 2, H, W, 0, 0, 0), x, eps=1e-5)
    assert mean[0] == (L - 1) / 2 and var[0] == (L * L - 1) / 12
    assert mean[1] == 3.0 and var[1] == 0.0


def test_two_valued_data_and_where_eps_sits(oracle):
    """Half the values +a, half -a: mean 0, var a^2, y = +-a / sqrt(a^2 + eps)."""
    a, eps = 3.0, 16.0
    x = np.empty((2, 1, 2, 2), dtype=np.float16)
    x[0], x[1] = a, -a
    pre, _, mean, var = oracle.batch_norm_forward((2, 1, 2, 2, 0, 0, 0), x, eps=eps)
    assert mean[0] == 0.0 and var[0] == 9.0
    assert np.array_equal(pre[0], np.full((1, 2, 2), 3.0 / 5.0)) and np.array_equal(pre[1], np.full((1, 2, 2), -3.0 / 5.0))


def test_constant_channel_gives_beta(oracle):
    x = np.full((3, 2, 2, 2), 7.5, dtype=np.float16)
    pre, _, _, var = oracle.batch_norm_forward((3, 2, 2, 2, 0, 1, 0), x, eps=1e-5, gamma=[2.0, 3.0], beta=[0.25, -4.0])
    assert np.all(var == 0.0)
    assert np.all(pre[:, 0] == 0.25) and np.all(pre[:, 1] == -4.0)


def test_output_moments(oracle):
    """Per channel the output (gamma 1, beta 0) sums to zero and its mean square is var/(var+eps)."""
    shape = (5, 4, 6, 5)
    x = _rand(shape, 3, loc=-2.0, scale=0.7)
    eps = 0.01
    pre, _, _, var = oracle.batch_norm_forward(shape + (0, 0, 0), x, eps=eps)
    assert np.allclose(pre.mean(axis=(0, 2, 3)), 0.0, atol=1e-13)
    assert np.allclose((pre ** 2).mean(axis=(0, 2, 3)), var / (var + eps), rtol=1e-12)


def test_affine_invariance_with_integer_data(oracle):
    """x -> 2x + 3 (exact in FP16 on small integers) with eps -> 4 eps leaves the output unchanged."""
    rng = np.random.default_rng(5)
    x = rng.integers(-20, 20, size=(3, 3, 4, 4)).astype(np.float16)
    p0, _, m0, v0 = oracle.batch_norm_forward((3, 3, 4, 4, 0, 0, 0), x, eps=0.5)
    p1, _, m1, v1 = oracle.batch_norm_forward((3, 3, 4, 4, 0, 0, 0), (2 * x + 3).astype(np.float16), eps=2.0)
    assert np.allclose(m1, 2 * m0 + 3, atol=1e-12) and np.allclose(v1, 4 * v0, rtol=1e-12)
    assert np.allclose(p0, p1, atol=1e-12)


def test_channels_are_independent_and_images_are_pooled(oracle):
    N, C, H, W = 3, 4, 2, 5                          # N != C, so a swapped index shows
    x = _rand((N, C, H, W), 9)
    x[:, 2] += np.float16(10.0)
    base = oracle.batch_norm_forward((N, C, H, W, 0, 0, 0), x)
    y = x.copy()
    y[1, 2, 0, 0] += np.float16(4.0)                 # one value of channel 2 in image 1
    new = oracle.batch_norm_forward((N, C, H, W, 0, 0, 0), y)
    for c in (0, 1, 3):
        assert np.array_equal(base[0][:, c], new[0][:, c])
    assert np.all(base[0][:, 2] != new[0][:, 2])      # every image of channel 2 moves: statistics pool over n
    assert abs(base[2][2] - 10.0) < 1.0 and abs(base[2][0]) < 1.0


def test_stored_statistics_ignore_the_batch(oracle):
    N, C, H, W = 2, 3, 3, 3
    x = _rand((N, C, H, W), 21, loc=4.0)
    m = np.array([1.0, -2.0, 0.5], dtype=np.float32)
    v = np.array([4.0, 0.25, 1.0], dtype=np.float32)
    g = np.array([1.0, -1.0, 0.5], dtype=np.float32)
    b = np.array([0.0, 2.0, -3.0], dtype=np.float32)
    eps = 1e-5
    pre, _, mean, var = oracle.batch_norm_forward((N, C, H, W, 1, 1, 0), x, eps=eps, mean=m * 4, var=v * 4,
                                                  stat_scale=0.25, gamma=g, beta=b)
    assert np.array_equal(mean, m.astype(np.float64)) and np.array_equal(var, v.astype(np.float64))
    xd = x.astype(np.float64)
    for c in range(C):
        ref = float(g[c]) * (xd[:, c] - float(m[c])) / np.sqrt(float(v[c]) + eps) + float(b[c])
        assert np.allclose(pre[:, c], ref, rtol=1e-13, atol=1e-13)
    # with the batch's own statistics stored, the two modes agree
    _, _, bm, bv = oracle.batch_norm_forward((N, C, H, W, 0, 0, 0), x, eps=eps)
    bm32, bv32 = bm.astype(np.float32), bv.astype(np.float32)
    p_batch, _, _, _ = oracle.batch_norm_forward((N, C, H, W, 0, 0, 0), x, eps=eps)
    p_glob, _, _, _ = oracle.batch_norm_forward((N, C, H, W, 1, 0, 0), x, eps=eps, mean=bm32, var=bv32)
    assert np.allclose(p_batch, p_glob, rtol=1e-5, atol=1e-5)


def test_rejects_bad_requests(oracle):
    x = np.zeros((1, 1, 1, 1), dtype=np.float16)
    with pytest.raises(ValueError):
        oracle.batch_norm_forward((1, 1, 1, 1, 0, 0, 0), x, eps=0.0)
    with pytest.raises(ValueError):
        oracle.batch_norm_forward((1, 1, 1, 1, 2, 0, 0), x)
    with pytest.raises(ValueError):
        oracle.batch_norm_forward((1, 1, 1, 1, 1, 0, 0), x)            # stored statistics missing
    with pytest.raises(ValueError):
        oracle.batch_norm_forward((1, 1, 1, 1, 0, 1, 0), x, gamma=[1.0])
    with pytest.raises(ValueError):
        oracle.batch_norm_forward((1, 2, 1, 1, 0, 0, 0), x)


# ---- folding stored statistics into the convolution in front (Section 3.3's pattern) -----------

def test_fold_by_hand(oracle):
    """a = gamma / sqrt(scale * var + eps): channel 0: 2 / sqrt(0.5 * 18 + 7) = 0.5; channel 1: -1 / sqrt(0.5 * 4 + 7) = -1/3."""
    w = np.array([[[[2.0, -4.0]]], [[[3.0, 6.0]]]], dtype=np.float16)          # [M=2][1][1][2]
    b = np.array([1.0, -2.0], dtype=np.float16)
    wo, bo = oracle.batch_norm_fold(w, b, mean=[4.0, 2.0], var=[18.0, 4.0], eps=7.0, stat_scale=0.5,
                                    gamma=[2.0, -1.0], beta=[0.25, 1.0])
    assert np.array_equal(wo[0], np.array([[[1.0, -2.0]]]))                     # 0.5 * w
    assert np.allclose(wo[1], np.array([[[-1.0, -2.0]]]), rtol=1e-15)           # -w / 3
    assert bo[0] == 0.5 * (1.0 - 2.0) + 0.25                                    # a (b - scale * mean) + beta
    assert abs(bo[1] - (-(-2.0 - 1.0) / 3.0 + 1.0)) < 1e-15
    w1, b1 = oracle.batch_norm_fold(w, None, mean=[0.0, 0.0], var=[1.0, 1.0], eps=3.0)   # no bias, no scale layer
    assert np.array_equal(w1, w.astype(np.float64) / 2.0) and np.array_equal(b1, np.zeros(2))


def test_fold_reproduces_batch_norm_after_convolution(oracle):
    """conv(x, w', b') = batchnorm(conv(x, w, b)): the convolution oracle and the batch-norm oracle on one side,
    the folded parameters in a brute-force FP64 convolution on the other."""
    N, C, H, W, M, k = 2, 3, 5, 6, 4, 3
    x = _rand((N, C, H, W), 31)
    w = _rand((M, C, k, k), 32, scale=0.3)
    b = _rand((M,), 33)
    mean = np.array([0.5, -1.0, 0.0, 2.0], dtype=np.float32)
    var = np.array([2.0, 0.5, 1.0, 4.0], dtype=np.float32)
    gamma = np.array([1.0, -2.0, 0.5, 1.5], dtype=np.float32)
    beta = np.array([0.0, 1.0, -1.0, 0.25], dtype=np.float32)
    pre, _ = oracle.conv2d_forward((N, C, H, W, M, k, 1, 1, 1, 1, 0), x, w, b)
    sd = np.sqrt(var.astype(np.float64) + 1e-3)
    want = gamma.astype(np.float64)[None, :, None, None] * (pre - mean.astype(np.float64)[None, :, None, None]) \
        / sd[None, :, None, None] + beta.astype(np.float64)[None, :, None, None]
    wo, bo = oracle.batch_norm_fold(w, b, mean, var, eps=1e-3, gamma=gamma, beta=beta)
    xp = np.zeros((N, C, H + 2, W + 2))
    xp[:, :, 1:-1, 1:-1] = x.astype(np.float64)
    got = np.empty_like(want)
    for oh in range(H):
        for ow in range(W):
            got[:, :, oh, ow] = np.einsum("ncrq,mcrq->nm", xp[:, :, oh:oh + k, ow:ow + k], wo) + bo[None, :]
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


# ---- the paper's two devices, replayed in emulated FP16 (Section 3.1) ------------------------

def _fp16_running_sum(v):
    acc = np.float16(0.0)
    for t in v:
        acc = np.float16(acc + np.float16(t))
    return acc


def _fp16_grouped_mean(v, group):
    """Mean of the groups' means, every sum, product and intermediate held in FP16."""
    means = []
    for i in range(0, len(v), group):
        part = v[i:i + group]
        means.append(np.float16(_fp16_running_sum(part) * np.float16(1.0 / len(part))))
    return np.float16(_fp16_running_sum(means) * np.float16(1.0 / len(means)))


def test_fp16_plain_mean_fails_and_grouped_mean_holds():
    """Image-like data (0..255): a running FP16 sum overflows, or 1/L underflows; grouping avoids both."""
    rng = np.random.default_rng(1)
    v = rng.integers(0, 256, size=4096).astype(np.float16)
    with np.errstate(over="ignore"):
        plain = _fp16_running_sum(v)
    assert not np.isfinite(plain)                                     # 4096 * 127 exceeds 65504
    L = 1 << 25
    assert np.float16(1.0 / L) == 0.0                                  # the inverse length is lost to zero
    grouped = _fp16_grouped_mean(v, 64)
    exact = v.astype(np.float64).mean()
    assert np.isfinite(grouped) and abs(float(grouped) - exact) <= 0.01 * exact


def test_fp16_squares_need_the_scale():
    """255^2 is the largest finite FP16 already; scaled by 1/32 the squares sum safely and scale back by 32^2."""
    rng = np.random.default_rng(2)
    v = rng.integers(0, 256, size=64).astype(np.float16)
    mean = np.float16(v.astype(np.float64).mean())
    with np.errstate(over="ignore"):
        plain = _fp16_running_sum([np.float16(np.float16(t - mean) * np.float16(t - mean)) for t in v])
    assert not np.isfinite(plain)
    s = np.float16(1.0 / 32)
    scaled = [np.float16(np.float16(np.float16(t - mean) * s) * np.float16(np.float16(t - mean) * s)) for t in v]
    var = float(np.float16(_fp16_running_sum(scaled) * np.float16(1.0 / len(v)))) * 32.0 * 32.0
    exact = v.astype(np.float64).var()
    assert abs(var - exact) <= 0.02 * exact
    small = (rng.uniform(-1, 1, size=64) * 2.0 ** -10).astype(np.float16)
    sq = [np.float16(t * t) for t in small]                             # around 2^-20 and below: FP16 subnormals
    up = [np.float16(np.float16(t * np.float16(32)) * np.float16(t * np.float16(32))) for t in small]
    exact_sq = (small.astype(np.float64) ** 2).sum()
    err_plain = abs(float(_fp16_running_sum(sq)) - exact_sq)
    err_scaled = abs(float(_fp16_running_sum(up)) / 1024.0 - exact_sq)
    assert err_scaled < err_plain

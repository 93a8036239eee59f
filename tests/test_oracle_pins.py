"""Pins for the CPU oracle: what the layer definition and plain mathematics fix.

The paper prints no worked example for this layer, so the oracle is pinned by
(1) a hand-worked fixture, (2) an independently structured second form
(materialised im2col matrix times weight matrix), (3) a library routine from an
unrelated code base (torch conv2d in float64 on the CPU), (4) closed forms and
(5) the invariants of the definition.  Each pin is chosen so that a plausible
slip (flipped kernel, wrong pad sign, ceil instead of floor, wrong group slice,
dropped bias) fails at least one of them.
"""
import json
import os

import numpy as np
import pytest

from workloads import ConvLayer, make_tensors, make_integer_tensors

HERE = os.path.dirname(os.path.abspath(__file__))

TINY = [
    # N  C  H  W  M  k  s  p  G
    (2, 4, 5, 6, 6, 3, 2, 1, 2),
    (1, 3, 7, 5, 4, 3, 1, 1, 1),
    (2, 6, 9, 8, 6, 5, 2, 2, 3),
    (1, 2, 4, 4, 2, 1, 1, 0, 1),
    (1, 4, 8, 8, 4, 3, 1, 1, 4),     # depthwise
    (1, 2, 11, 11, 3, 7, 2, 3, 1),   # floor drops a padded row: (11+6-7)/2 = 5 -> 6 outputs
    (1, 2, 10, 10, 3, 7, 2, 3, 1),   # (10+6-7)/2 = 4.5 -> floor
    (3, 8, 6, 7, 8, 2, 3, 0, 2),     # even kernel, stride > kernel
    (1, 1, 3, 3, 1, 3, 1, 0, 1),     # single output pixel
    (1, 2, 2, 2, 2, 4, 1, 1, 1),     # kernel larger than the image, saved by padding
]


def layer_of(t, bias=1, relu=0, name="tiny"):
    N, C, H, W, M, k, s, p, G = t
    return ConvLayer(name, N, C, H, W, M, k, s, p, G, bias, relu)


def im2col_form(L, x, w, b):
    """Second form: build the (Kg x P) patch matrix per group, multiply by the
    (Mg x Kg) weight matrix.  Different loop structure from the oracle."""
    xd = x.astype(np.float64)
    wd = w.astype(np.float64)
    xp = np.zeros((L.N, L.C, L.H + 2 * L.p, L.W + 2 * L.p))
    xp[:, :, L.p:L.p + L.H, L.p:L.p + L.W] = xd
    out = np.zeros(L.y_shape)
    for n in range(L.N):
        for g in range(L.G):
            cols = np.zeros((L.Kg, L.Ho * L.Wo))
            row = 0
            for c in range(L.Cg):
                for r in range(L.k):
                    for q in range(L.k):
                        patch = xp[n, g * L.Cg + c,
                                   r:r + (L.Ho - 1) * L.s + 1:L.s,
                                   q:q + (L.Wo - 1) * L.s + 1:L.s]
                        cols[row] = patch.reshape(-1)
                        row += 1
            wm = wd[g * L.Mg:(g + 1) * L.Mg].reshape(L.Mg, L.Kg)
            out[n, g * L.Mg:(g + 1) * L.Mg] = (wm @ cols).reshape(L.Mg, L.Ho, L.Wo)
    if b is not None:
        out += b.astype(np.float64)[None, :, None, None]
    return out


def test_half_decode_all_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(v)) for v in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    # values the format fixes: smallest subnormal, largest finite (paper, Section 3.1 range)
    assert oracle.half_to_double(0x0001) == 2.0 ** -24
    assert oracle.half_to_double(0x7BFF) == 65504.0


def test_hand_worked_fixture(oracle):
    with open(os.path.join(HERE, "golden", "hand_worked_3x3.json")) as f:
        gold = json.load(f)
    x0 = np.array(gold["x"], dtype=np.float16).reshape(1, 1, 3, 3)
    w = np.array(gold["w"], dtype=np.float16).reshape(1, 1, 2, 2)
    for case in gold["cases"]:
        x = -x0 if case.get("negate_x") else x0
        b = np.array([case["bias"]], dtype=np.float16)
        desc = (1, 1, 3, 3, 1, 2, case["stride"], case["pad"], 1, 1, 0)
        pre, mag = oracle.conv2d_forward(desc, x, w, b)
        assert np.array_equal(pre[0, 0], np.array(case["pre"], dtype=np.float64))
        assert np.array_equal(mag[0, 0], np.array(case["mag"], dtype=np.float64))


@pytest.mark.parametrize("t", TINY)
def test_matches_im2col_second_form(oracle, t):
    L = layer_of(t)
    x, w, b = make_tensors(L, seed=11)
    pre, mag = oracle.conv2d_forward(L.desc(), x, w, b)
    assert pre.shape == L.y_shape
    want = im2col_form(L, x, w, b)
    assert np.max(np.abs(pre - want)) < 1e-12
    # magnitude: same sum over |w|,|x| without the bias
    wantmag = im2col_form(L, np.abs(x), np.abs(w), None)
    assert np.max(np.abs(mag - wantmag)) < 1e-12


@pytest.mark.parametrize("t", TINY)
def test_matches_torch_float64_witness(oracle, t):
    torch = pytest.importorskip("torch")
    L = layer_of(t)
    x, w, b = make_tensors(L, seed=5)
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, b)
    want = torch.nn.functional.conv2d(
        torch.from_numpy(x.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
        torch.from_numpy(b.astype(np.float64)), stride=L.s, padding=L.p, dilation=1, groups=L.G)
    assert tuple(want.shape) == L.y_shape
    assert np.max(np.abs(pre - want.numpy())) < 1e-10


def test_pointwise_is_a_matmul(oracle):
    L = ConvLayer("pw", 2, 5, 4, 3, 7, 1, 1, 0, 1, 0, 0)
    x, w, _ = make_tensors(L, seed=3)
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, None)
    W2 = w.astype(np.float64).reshape(7, 5)
    for n in range(2):
        X2 = x[n].astype(np.float64).reshape(5, 12)
        assert np.max(np.abs(pre[n].reshape(7, 12) - W2 @ X2)) < 1e-13


@pytest.mark.parametrize("k", [1, 3, 5])
def test_centre_delta_reproduces_input(oracle, k):
    C = 3
    L = ConvLayer("delta", 2, C, 6, 7, C, k, 1, (k - 1) // 2, C, 0, 0)
    x, _, _ = make_tensors(L, seed=1)
    w = np.zeros(L.w_shape, dtype=np.float16)
    w[:, 0, k // 2, k // 2] = 1.0
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, None)
    assert np.array_equal(pre, x.astype(np.float64))


def test_corner_delta_fixes_orientation(oracle):
    """A one at tap (0,0) reads x[oh*s-p, ow*s-p]: cross-correlation, no kernel flip."""
    for s, p in [(1, 1), (2, 1), (1, 0), (2, 2)]:
        L = ConvLayer("corner", 1, 1, 7, 8, 1, 3, s, p, 1, 0, 0)
        x, _, _ = make_tensors(L, seed=2)
        w = np.zeros(L.w_shape, dtype=np.float16)
        w[0, 0, 0, 0] = 1.0
        pre, _ = oracle.conv2d_forward(L.desc(), x, w, None)
        xd = x.astype(np.float64)[0, 0]
        for oh in range(L.Ho):
            for ow in range(L.Wo):
                ih, iw = oh * s - p, ow * s - p
                want = xd[ih, iw] if 0 <= ih < L.H and 0 <= iw < L.W else 0.0
                assert pre[0, 0, oh, ow] == want
    # and a one at tap (0,2) of a 3x3 reads the pixel to the right, one row up
    L = ConvLayer("corner2", 1, 1, 5, 5, 1, 3, 1, 1, 1, 0, 0)
    x, _, _ = make_tensors(L, seed=4)
    w = np.zeros(L.w_shape, dtype=np.float16)
    w[0, 0, 0, 2] = 1.0
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, None)
    assert pre[0, 0, 2, 2] == float(x[0, 0, 1, 3])


def test_linearity_in_x_and_w(oracle):
    L = layer_of(TINY[0], bias=0)
    x1, w1, _ = make_tensors(L, seed=21)
    x2, w2, _ = make_tensors(L, seed=22)
    # sums of FP16 values are formed so that they stay FP16-representable
    x1 = (np.round(x1.astype(np.float64) * 64) / 64).astype(np.float16)
    x2 = (np.round(x2.astype(np.float64) * 64) / 64).astype(np.float16)
    xs = (x1.astype(np.float64) + 2 * x2.astype(np.float64)).astype(np.float16)
    assert np.array_equal(xs.astype(np.float64), x1.astype(np.float64) + 2 * x2.astype(np.float64))
    d = L.desc()
    a, _ = oracle.conv2d_forward(d, x1, w1, None)
    b, _ = oracle.conv2d_forward(d, x2, w1, None)
    c, _ = oracle.conv2d_forward(d, xs, w1, None)
    assert np.max(np.abs(c - (a + 2 * b))) < 1e-12
    w1 = (np.round(w1.astype(np.float64) * 256) / 256).astype(np.float16)
    w2 = (np.round(w2.astype(np.float64) * 256) / 256).astype(np.float16)
    ws = (w1.astype(np.float64) - w2.astype(np.float64)).astype(np.float16)
    assert np.array_equal(ws.astype(np.float64), w1.astype(np.float64) - w2.astype(np.float64))
    a, _ = oracle.conv2d_forward(d, x1, w1, None)
    b, _ = oracle.conv2d_forward(d, x1, w2, None)
    c, _ = oracle.conv2d_forward(d, x1, ws, None)
    assert np.max(np.abs(c - (a - b))) < 1e-12


@pytest.mark.parametrize("H,W,k,s,p", [(6, 7, 3, 1, 1), (7, 7, 3, 2, 1), (8, 6, 5, 2, 2),
                                       (10, 10, 7, 2, 3), (9, 9, 11, 4, 5), (5, 5, 2, 2, 0)])
def test_all_ones_counts_in_bounds_taps(oracle, H, W, k, s, p):
    """x = w = 1, no bias: y = Cg * (#taps inside the image); the count factorises per axis."""
    Cg = 3
    L = ConvLayer("ones", 1, Cg, H, W, 2, k, s, p, 1, 0, 0)
    x = np.ones(L.x_shape, dtype=np.float16)
    w = np.ones(L.w_shape, dtype=np.float16)
    pre, mag = oracle.conv2d_forward(L.desc(), x, w, None)

    def inside(o, size):
        lo = max(0, p - o * s)                 # first tap with o*s - p + r >= 0
        hi = min(k, size + p - o * s)          # one past the last tap below `size`
        return max(0, hi - lo)

    Ho = (H + 2 * p - k) // s + 1
    Wo = (W + 2 * p - k) // s + 1
    assert pre.shape == (1, 2, Ho, Wo)
    for oh in range(Ho):
        for ow in range(Wo):
            want = Cg * inside(oh, H) * inside(ow, W)
            assert pre[0, 0, oh, ow] == want and pre[0, 1, oh, ow] == want
    assert np.array_equal(pre, mag)


def test_output_size_floor_cases(oracle):
    assert oracle.out_shape((1, 3, 224, 224, 64, 7, 2, 3, 1, 1, 1)) == (1, 64, 112, 112)
    assert oracle.out_shape((1, 3, 224, 224, 32, 3, 2, 1, 1, 1, 1)) == (1, 32, 112, 112)
    assert oracle.out_shape((1, 3, 227, 227, 96, 11, 4, 0, 1, 1, 1)) == (1, 96, 55, 55)
    # the array the C code fills has the same shape: last padded row is never read
    L = ConvLayer("floor", 1, 1, 6, 6, 1, 3, 2, 1, 1, 0, 0)     # (6+2-3)/2 = 2.5 -> 3 outputs
    x = np.zeros(L.x_shape, dtype=np.float16)
    x[0, 0, 5, 5] = 1.0                                          # bottom-right pixel
    w = np.ones(L.w_shape, dtype=np.float16)
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, None)
    assert pre.shape == (1, 1, 3, 3)
    # output (2,2) covers rows/cols 3..5, so it sees the pixel; nothing else does
    want = np.zeros((3, 3)); want[2, 2] = 1.0
    assert np.array_equal(pre[0, 0], want)


def test_groups_are_independent_convolutions(oracle):
    L = ConvLayer("grp", 2, 6, 5, 5, 9, 3, 1, 1, 3, 1, 0)
    x, w, b = make_tensors(L, seed=8)
    pre, mag = oracle.conv2d_forward(L.desc(), x, w, b)
    for g in range(3):
        Ls = ConvLayer("slice", 2, 2, 5, 5, 3, 3, 1, 1, 1, 1, 0)
        ps, ms = oracle.conv2d_forward(Ls.desc(), x[:, 2 * g:2 * g + 2], w[3 * g:3 * g + 3], b[3 * g:3 * g + 3])
        assert np.array_equal(pre[:, 3 * g:3 * g + 3], ps)
        assert np.array_equal(mag[:, 3 * g:3 * g + 3], ms)
    # a change in group 0's input channels must not reach group 1's outputs
    x2 = x.copy(); x2[:, 0:2] += np.float16(1.0)
    pre2, _ = oracle.conv2d_forward(L.desc(), x2, w, b)
    assert np.array_equal(pre2[:, 3:], pre[:, 3:]) and not np.array_equal(pre2[:, :3], pre[:, :3])


def test_depthwise_is_per_channel(oracle):
    C = 5
    L = ConvLayer("dw", 1, C, 6, 6, C, 3, 2, 1, C, 1, 0)
    x, w, b = make_tensors(L, seed=9)
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, b)
    for c in range(C):
        L1 = ConvLayer("one", 1, 1, 6, 6, 1, 3, 2, 1, 1, 1, 0)
        p1, _ = oracle.conv2d_forward(L1.desc(), x[:, c:c + 1], w[c:c + 1], b[c:c + 1])
        assert np.array_equal(pre[:, c:c + 1], p1)


def test_bias_enters_pre_not_mag_and_relu_reference(oracle):
    L = layer_of(TINY[1], bias=1)
    x, w, b = make_tensors(L, seed=13)
    pre, mag = oracle.conv2d_forward(L.desc(), x, w, b)
    L0 = layer_of(TINY[1], bias=0)
    pre0, mag0 = oracle.conv2d_forward(L0.desc(), x, w, None)
    assert np.array_equal(mag, mag0)
    assert np.max(np.abs(pre - pre0 - b.astype(np.float64)[None, :, None, None])) < 1e-13
    ref, bound = oracle.reference(pre, mag, relu=1)
    assert np.array_equal(ref, np.where(pre > 0, pre, 0.0))
    assert np.array_equal(bound, 4e-3 * mag + 1e-3)
    assert (pre < 0).any() and (pre > 0).any()


def test_points_equal_full_tensor(oracle):
    L = layer_of(TINY[2])
    x, w, b = make_tensors(L, seed=17)
    pre, mag = oracle.conv2d_forward(L.desc(), x, w, b)
    rng = np.random.default_rng(0)
    idx = np.stack([rng.integers(0, d, 200) for d in L.y_shape], axis=1)
    pp, pm = oracle.conv2d_points(L.desc(), x, w, b, idx)
    assert np.array_equal(pp, pre[tuple(idx.T)])
    assert np.array_equal(pm, mag[tuple(idx.T)])
    with pytest.raises(ValueError):
        oracle.conv2d_points(L.desc(), x, w, b, [[0, 0, L.Ho, 0]])


def test_integer_inputs_give_exact_integers(oracle):
    L = ConvLayer("int", 2, 8, 9, 9, 8, 3, 1, 1, 2, 1, 0)
    x, w, b = make_integer_tensors(L, seed=4)
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, b)
    assert np.array_equal(pre, np.round(pre))
    assert np.max(np.abs(pre)) <= L.Kg * 8 + 8
    want = im2col_form(L, x, w, b)
    assert np.array_equal(pre, want)


def test_bad_descriptors_are_rejected(oracle):
    x = np.zeros((1, 2, 4, 4), dtype=np.float16)
    w = np.zeros((2, 2, 3, 3), dtype=np.float16)
    for desc in [(1, 2, 4, 4, 2, 3, 0, 1, 1, 0, 0),      # stride 0
                 (1, 3, 4, 4, 2, 3, 1, 1, 2, 0, 0),      # C % group
                 (1, 2, 4, 4, 3, 3, 1, 1, 2, 0, 0),      # M % group
                 (1, 2, 4, 4, 2, 7, 1, 1, 1, 0, 0)]:     # kernel larger than padded image
        with pytest.raises(ValueError):
            oracle.conv2d_forward(desc, x, w, None)


def test_config1_is_fast_and_sane(oracle):
    import time
    from workloads import config1
    L = config1()[0]
    x, w, b = make_tensors(L, seed=0)
    assert abs(float(np.std(w.astype(np.float64))) - np.sqrt(2 / 27)) < 0.03
    assert float(np.max(np.abs(x.astype(np.float64)))) <= 1.0
    assert float(np.max(np.abs(b.astype(np.float64)))) <= 0.1001
    t = time.perf_counter()
    pre, mag = oracle.conv2d_forward(L.desc(), x, w, b)
    assert time.perf_counter() - t < 1.0
    assert pre.shape == (1, 16, 32, 32)
    want = im2col_form(L, x, w, b)
    assert np.max(np.abs(pre - want)) < 1e-12

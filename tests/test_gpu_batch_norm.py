"""GPU parity of hgc_batch_norm_forward against the FP64 oracle, through the C ABI.

Bar: |y - ref| <= 1e-3 |ref| + 2e-5 mag + 1e-7 with mag = |gamma| (|x| + |mean|) / sqrt(var + eps) + |beta|:
the first term is the one FP16 rounding at the store with a factor two to spare, the second the
FP32 statistics and the FP32 multiply-add (about 300 * 2^-24 of the terms that cancel).  Batch
statistics: |mean - ref| <= 2e-6 * mean|x| + 1e-7, |var - ref| <= 2e-5 * var + 1e-9.
"""
import numpy as np
import pytest

import paper_1901_00858_amd as hgc
from workloads import uniform01, normal01

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def activations(N, C, H, W, seed, kind="conv"):
    """Seeded inputs.  conv: what a convolution hands to batch norm, channel c ~ N(m_c, s_c) with
    m_c in [-2, 2] and s_c in [0.25, 2.25]; image: integers 0..255 (the paper's overflow example);
    offset: mean 100, deviation 1 (the terms of the output cancel to one part in a hundred)."""
    n = N * C * H * W
    if kind == "image":
        x = np.floor(256.0 * uniform01(seed, 0, n)).reshape(N, C, H, W)
    else:
        z = normal01(seed, 0, n).reshape(N, C, H, W)
        if kind == "offset":
            m = np.full(C, 100.0)
            s = np.ones(C)
        else:
            m = 4.0 * uniform01(seed, 1, C) - 2.0
            s = 0.25 + 2.0 * uniform01(seed, 2, C)
        x = m[None, :, None, None] + s[None, :, None, None] * z
    return x.astype(np.float16)


def affine(C, seed):
    g = (0.5 + uniform01(seed, 3, C)).astype(np.float32) * np.where(np.arange(C) % 3 == 2, -1.0, 1.0).astype(np.float32)
    b = (uniform01(seed, 4, C) - 0.5).astype(np.float32)
    return g, b


def run(desc, x, eps=1e-5, mean=None, var=None, stat_scale=1.0, gamma=None, beta=None, offset=0, in_place=False,
        want_stats=True):
    """One call through the raw entry point; offset shifts the x and y bases by that many halves."""
    import torch
    N, C, H, W = desc[:4]
    n = x.size
    xbuf = torch.empty(n + offset, dtype=torch.float16, device="cuda")
    xd = xbuf[offset:]
    xd.copy_(torch.from_numpy(np.ascontiguousarray(x).reshape(-1)))
    if in_place:
        yd = xd
    else:
        ybuf = torch.empty(n + offset, dtype=torch.float16, device="cuda")
        ybuf.view(torch.int16).fill_(0x7E00)                  # NaN pattern: unwritten outputs show up
        yd = ybuf[offset:]

    def f32(a):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    d = hgc.BatchNormDesc.make(desc, eps, stat_scale)
    if d.use_global_stats:
        md, vd = f32(mean), f32(var)
    elif want_stats:
        md = torch.full((C,), float("nan"), dtype=torch.float32, device="cuda")
        vd = torch.full((C,), float("nan"), dtype=torch.float32, device="cuda")
    else:
        md = vd = None
    gd, bd = f32(gamma), f32(beta)
    need = hgc.batch_norm_workspace_size(d)
    ws = torch.empty(need + 2, dtype=torch.uint8, device="cuda")
    ptr = lambda t: 0 if t is None else t.data_ptr()
    st = hgc.batch_norm_forward_raw(d, xd.data_ptr(), ptr(md), ptr(vd), ptr(gd), ptr(bd), yd.data_ptr(),
                                    ws.data_ptr() + 2, need, torch.cuda.current_stream().cuda_stream)   # odd workspace base
    assert st == 0, hgc.status_string(st)
    torch.cuda.synchronize()
    y = yd.cpu().numpy().reshape(N, C, H, W)
    if d.use_global_stats or not want_stats:
        return y, None, None
    return y, md.cpu().numpy(), vd.cpu().numpy()


def check(oracle, desc, x, y, tag, eps=1e-5, gmean=None, gvar=None, **kw):
    pre, mag, mean, var = oracle.batch_norm_forward(desc, x, eps=eps, **kw)
    ok, ratio, where = oracle.check_batch_norm(y, pre, mag, desc[6])
    assert ok, f"{tag} {desc}: |err|/bound = {ratio:.3g} at {where}: got {y[where]}, pre {pre[where]}, mag {mag[where]}"
    if gmean is not None:
        absx = np.abs(x.astype(np.float64)).mean(axis=(0, 2, 3))
        assert np.all(np.abs(gmean - mean) <= 2e-6 * absx + 1e-7), f"{tag} {desc}: mean {gmean} vs {mean}"
        assert np.all(np.abs(gvar - var) <= 2e-5 * var + 1e-9), f"{tag} {desc}: var {gvar} vs {var}"
    return ratio


SHAPES = [
    # N, C, H, W.  Plane lengths: 1; odd (element loads); % 2, % 4, % 8 (each vector width); one, two and
    # seven groups per plane with a ragged last group; a long odd plane split into two groups
    (1, 1, 1, 1), (1, 3, 5, 7), (3, 5, 7, 7), (2, 3, 3, 6), (2, 4, 14, 14), (3, 5, 6, 6), (4, 8, 28, 28),
    (2, 2, 64, 64), (1, 2, 50, 50), (3, 16, 56, 56), (2, 3, 112, 112), (1, 1, 45, 47), (5, 70, 9, 8),
    # short planes (a plane per 16 lanes): every load width with 1 to 16 loads per lane, plane counts that
    # do not fill the last wave, 1x1 maps; then lengths just past that path (one wave per plane again)
    (3, 5, 15, 15), (2, 6, 10, 13), (2, 3, 11, 11), (2, 9, 12, 12), (2, 4, 16, 16), (3, 7, 4, 4), (33, 3, 1, 1),
    (1, 37, 2, 1), (2, 67, 8, 4), (1, 131, 14, 14), (2, 3, 16, 17), (1, 5, 17, 17), (2, 2, 24, 24),
]


@pytest.mark.parametrize("shape", SHAPES, ids=["x".join(map(str, s)) for s in SHAPES])
def test_shapes(oracle, shape):
    N, C, H, W = shape
    x = activations(N, C, H, W, seed=sum(shape))
    g, b = affine(C, seed=7)
    for sb, relu in ((0, 0), (1, 0), (1, 1)):
        desc = (N, C, H, W, 0, sb, relu)
        say(f"[bn] {desc}")
        kw = dict(gamma=g, beta=b) if sb else {}
        y, m, v = run(desc, x, **kw)
        check(oracle, desc, x, y, "bn", gmean=m, gvar=v, **kw)


def test_image_like_and_offset_data(oracle):
    """0..255 data, whose squares overflow FP16 (Section 3.1 of the paper), and data far from zero."""
    for kind, shape in (("image", (2, 3, 32, 32)), ("image", (1, 3, 224, 224)), ("offset", (4, 6, 28, 28))):
        N, C, H, W = shape
        x = activations(N, C, H, W, seed=3, kind=kind)
        desc = (N, C, H, W, 0, 0, 0)
        say(f"[bn-{kind}] {desc}")
        y, m, v = run(desc, x)
        check(oracle, desc, x, y, kind, gmean=m, gvar=v)
        assert np.all(np.isfinite(y))


def test_stored_statistics(oracle):
    for shape in [(2, 6, 14, 14), (1, 5, 7, 9), (3, 4, 16, 16)]:
        N, C, H, W = shape
        x = activations(N, C, H, W, seed=11)
        g, b = affine(C, seed=8)
        mean = (4.0 * uniform01(5, 5, C) - 2.0).astype(np.float32) * 8
        var = (0.1 + 3.0 * uniform01(5, 6, C)).astype(np.float32) * 8
        for sb, relu in ((0, 0), (1, 1)):
            desc = (N, C, H, W, 1, sb, relu)
            say(f"[bn-stored] {desc}")
            kw = dict(mean=mean, var=var, stat_scale=0.125)
            if sb:
                kw.update(gamma=g, beta=b)
            y, _, _ = run(desc, x, eps=1e-3, **kw)
            check(oracle, desc, x, y, "stored", eps=1e-3, **kw)


def test_exact_case():
    """Half the values 3, half -3, eps 7: mean 0, var 9, root 4, y = +-0.75 with no rounding anywhere."""
    x = np.empty((2, 3, 4, 4), dtype=np.float16)
    x[0], x[1] = 3.0, -3.0
    y, m, v = run((2, 3, 4, 4, 0, 0, 0), x, eps=7.0)
    assert np.all(m == 0.0) and np.all(v == 9.0)
    assert np.all(y[0] == 0.75) and np.all(y[1] == -0.75)
    yr, _, _ = run((2, 3, 4, 4, 0, 0, 1), x, eps=7.0)
    assert np.all(yr[0] == 0.75) and np.all(yr[1] == 0.0)


def test_constant_channel_and_single_value(oracle):
    x = np.full((2, 2, 3, 3), 5.5, dtype=np.float16)
    y, m, v = run((2, 2, 3, 3, 0, 1, 0), x, gamma=[2.0, -1.0], beta=[0.25, 3.0])
    assert np.all(m == 5.5) and np.all(v == 0.0)
    assert np.all(y[:, 0] == 0.25) and np.all(y[:, 1] == 3.0)
    y1, _, v1 = run((1, 1, 1, 1, 0, 0, 0), np.array([[[[-7.0]]]], dtype=np.float16))
    assert v1[0] == 0.0 and y1[0, 0, 0, 0] == 0.0


def test_in_place_and_without_statistics_outputs(oracle):
    N, C, H, W = 3, 6, 14, 14
    x = activations(N, C, H, W, seed=4)
    desc = (N, C, H, W, 0, 0, 1)
    y0, _, _ = run(desc, x)
    y1, _, _ = run(desc, x, in_place=True, want_stats=False)
    assert np.array_equal(y0, y1)
    check(oracle, desc, x, y1, "in-place")


def test_unaligned_bases(oracle):
    """Bases off by 1, 2, 4 halves: narrower loads (another order of summation within a group), same bar."""
    N, C, H, W = 2, 5, 16, 16
    x = activations(N, C, H, W, seed=6)
    desc = (N, C, H, W, 0, 0, 0)
    for off in (1, 2, 4, 7):
        say(f"[bn-unaligned] offset {off}")
        y, m, v = run(desc, x, offset=off)
        check(oracle, desc, x, y, f"offset {off}", gmean=m, gvar=v)


def test_repeatable():
    N, C, H, W = 4, 32, 28, 28
    x = activations(N, C, H, W, seed=9)
    a = run((N, C, H, W, 0, 0, 0), x)
    b = run((N, C, H, W, 0, 0, 0), x)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])


def test_benchmark_size_against_the_full_oracle(oracle):
    """The first batch norm of a ResNet-50-shaped stack at the batch the benchmark times: 32 x 64 x 112 x 112."""
    N, C, H, W = 32, 64, 112, 112
    x = activations(N, C, H, W, seed=50)
    g, b = affine(C, seed=51)
    desc = (N, C, H, W, 0, 1, 1)
    say(f"[bn-full] {desc}")
    y, m, v = run(desc, x, gamma=g, beta=b)
    check(oracle, desc, x, y, "full", gmean=m, gvar=v, gamma=g, beta=b)


def test_binding_wrapper(oracle):
    import torch
    N, C, H, W = 2, 8, 14, 14
    x = activations(N, C, H, W, seed=12)
    xd = torch.from_numpy(x).cuda()
    mean = torch.empty(C, dtype=torch.float32, device="cuda")
    var = torch.empty(C, dtype=torch.float32, device="cuda")
    y = hgc.batch_norm_forward((N, C, H, W, 0, 0, 0), xd, mean=mean, var=var)
    torch.cuda.synchronize()
    check(oracle, (N, C, H, W, 0, 0, 0), x, y.cpu().numpy(), "wrapper", gmean=mean.cpu().numpy(), gvar=var.cpu().numpy())
    with pytest.raises(ValueError):
        hgc.batch_norm_forward((N, C, H, W, 1, 0, 0), xd)


def test_fold_into_the_convolution(oracle):
    """hgc_batch_norm_fold: the folded parameters are the oracle's, rounded once; and the folded convolution on
    the GPU computes batch norm after the convolution as the two oracles define it.  Bound of the second
    check: the unfolded pair would be allowed |a| (4e-3 mag + 1e-3) from the convolution plus the batch norm's
    own rounding; folding rounds every weight once more (2^-11 of |a| mag, inside the first term) and the
    bias once (2^-11 |b'|)."""
    import torch
    from workloads import ConvLayer, make_tensors
    for L in [ConvLayer("fold.a", 2, 16, 14, 14, 32, 3, 1, 1), ConvLayer("fold.b", 1, 8, 9, 9, 12, 1, 1, 0, 1, 0, 0),
              ConvLayer("fold.c", 2, 12, 10, 10, 24, 3, 2, 1, 4)]:
        x, w, b = make_tensors(L, seed=77)
        M = L.M
        mean = (2.0 * uniform01(9, 1, M) - 1.0).astype(np.float32) * 4
        var = (0.2 + 2.0 * uniform01(9, 2, M)).astype(np.float32) * 4
        gamma, beta = affine(M, seed=9)
        eps, scale = 1e-3, 0.25
        for with_scale in (True, False):
            g, bt = (gamma, beta) if with_scale else (None, None)
            say(f"[bn-fold] {L.name} scale layer {with_scale}")
            dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
            wo, bo = hgc.batch_norm_fold(L, dev(w), dev(b) if L.bias else None, dev(mean), dev(var), eps=eps,
                                         stat_scale=scale, gamma=dev(g), beta=dev(bt))
            torch.cuda.synchronize()
            w64, b64 = oracle.batch_norm_fold(w, b if L.bias else None, mean, var, eps=eps, stat_scale=scale, gamma=g, beta=bt)
            assert np.array_equal(wo.cpu().numpy(), w64.astype(np.float16))
            assert np.array_equal(bo.cpu().numpy(), b64.astype(np.float16))
            folded = ConvLayer(L.name, L.N, L.C, L.H, L.W, L.M, L.k, L.s, L.p, L.G, 1, 1)
            ws = torch.empty(max(1, hgc.conv2d_workspace_size(folded)), dtype=torch.uint8, device="cuda")
            y = hgc.conv2d_forward_ws(folded, dev(x), wo, bo, None, ws)
            torch.cuda.synchronize()
            pre, mag = oracle.conv2d_forward(L.desc(), x, w, b if L.bias else None)
            a = (g.astype(np.float64) if with_scale else 1.0) / np.sqrt(scale * var.astype(np.float64) + eps)
            ref = a[None, :, None, None] * (pre - scale * mean.astype(np.float64)[None, :, None, None]) \
                + (bt.astype(np.float64)[None, :, None, None] if with_scale else 0.0)
            ref = np.maximum(ref, 0.0)
            bound = np.abs(a)[None, :, None, None] * (4e-3 * mag + 1e-3) + 2.0 ** -11 * np.abs(b64)[None, :, None, None] \
                + 1e-3 * np.abs(ref) + 1e-3
            err = np.abs(y.cpu().numpy().astype(np.float64) - ref)
            worst = np.unravel_index(np.argmax(err / bound), err.shape)
            assert np.all(err <= bound), f"{L.name}: |err| {err[worst]} > {bound[worst]} at {worst}"

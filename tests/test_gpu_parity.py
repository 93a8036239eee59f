"""GPU parity: the HIP path, called through the C ABI, against the FP64 oracle.

Tolerance (stated for this build): |gpu - oracle| <= 4e-3 * sum|w*x| + 1e-3, the sum
taken over the taps before the bias and ReLU; integer-valued inputs must match exactly.
"""
import numpy as np
import pytest

import paper_1901_00858_amd as hgc
from workloads import CONFIGS, ConvLayer, layer_seed, make_integer_tensors, make_tensors

from gpu_helpers import assert_full, assert_points, run_layer, sample_points, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    hgc.load()
    hgc.set_forced_path(hgc.PATH_AUTO)
    yield
    hgc.set_forced_path(hgc.PATH_AUTO)


#          N  C   H   W   M  k  s  p  G
SHAPES = [
    (1, 3, 32, 32, 16, 3, 1, 1, 1),      # config 1
    (2, 16, 20, 24, 32, 3, 1, 1, 1),     # aligned channels, even W
    (2, 16, 21, 23, 32, 3, 1, 1, 1),     # odd W: 2-byte input loads
    (1, 24, 17, 18, 40, 3, 1, 1, 1),     # Cg % 16 != 0, ragged channel tile
    (1, 20, 17, 18, 72, 3, 1, 1, 1),     # Cg % 8 != 0: scalar weight loads
    (3, 32, 15, 15, 64, 3, 2, 1, 1),     # stride 2, odd W
    (2, 32, 28, 28, 64, 3, 2, 1, 1),     # stride 2, even W, floor drops a padded row
    (1, 64, 9, 40, 160, 3, 1, 0, 1),     # pad 0, wide, M ragged against 128 (two tiles)
    (2, 64, 14, 14, 96, 3, 1, 1, 2),     # groups
    (1, 48, 13, 13, 48, 3, 1, 1, 3),     # groups, odd W
    (2, 64, 12, 12, 64, 1, 1, 0, 1),     # pointwise
    (1, 200, 7, 7, 96, 1, 1, 0, 1),      # pointwise, odd W, Cg % 64 != 0
    (1, 36, 10, 10, 48, 1, 1, 0, 1),     # pointwise, Cg % 8 != 0
    (2, 32, 16, 16, 32, 1, 2, 0, 1),     # pointwise, stride 2
    (1, 96, 27, 27, 64, 5, 1, 2, 2),     # 5x5 grouped (AlexNet conv2 style), odd W
    (1, 16, 20, 20, 32, 5, 2, 2, 1),     # 5x5 stride 2
    (1, 3, 40, 40, 32, 7, 2, 3, 1),      # stem style
    (1, 3, 37, 37, 24, 7, 2, 3, 1),      # stem style, odd W, ragged M
    (1, 3, 43, 43, 24, 11, 4, 0, 1),     # AlexNet conv1 style -> direct path
    (1, 8, 12, 12, 16, 2, 2, 0, 1),      # even kernel -> direct path
    (2, 24, 19, 19, 24, 3, 1, 1, 24),    # depthwise
    (1, 16, 30, 30, 16, 3, 2, 1, 16),    # depthwise stride 2
    (1, 8, 16, 16, 8, 5, 1, 2, 8),       # depthwise 5x5
    (2, 16, 24, 32, 16, 3, 1, 1, 16),    # depthwise, 8-pixel vectors, rows end on wave boundaries
    (1, 8, 9, 56, 8, 3, 1, 1, 8),        # depthwise, 8-pixel vectors, halo fetched across waves
    (1, 8, 12, 28, 8, 3, 1, 1, 8),       # depthwise, 4-pixel vectors
    (1, 8, 14, 14, 8, 3, 1, 1, 8),       # depthwise, 2-pixel vectors
    (2, 8, 9, 6, 8, 3, 1, 1, 8),         # depthwise, 2-pixel vectors, three groups a row, odd height
    (3, 16, 5, 10, 16, 3, 1, 1, 16),     # depthwise, 2-pixel vectors, rows shorter than a wave
    (1, 8, 7, 2, 8, 3, 1, 1, 8),         # depthwise, rows of two pixels
    (2, 8, 30, 4, 8, 3, 1, 1, 8),        # depthwise, rows of four pixels: a first and a last group only
    (1, 8, 10, 112, 8, 3, 2, 1, 8),      # depthwise stride 2, 8-pixel input vectors
    (2, 8, 28, 28, 8, 3, 2, 1, 8),       # depthwise stride 2, 4-pixel input vectors
    (1, 8, 9, 9, 16, 3, 1, 1, 8),        # channel multiplier 2 (Mg = 2) -> direct
    (1, 16, 33, 70, 32, 3, 1, 1, 1),     # several window tiles in both directions
    (1, 16, 3, 3, 32, 3, 1, 0, 1),       # single output pixel
]


def _layer(t, bias=1, relu=1):
    N, C, H, W, M, k, s, p, G = t
    return ConvLayer("case", N, C, H, W, M, k, s, p, G, bias, relu)


@pytest.mark.parametrize("t", SHAPES)
def test_shapes_full_tensor(oracle, t):
    for bias, relu, ws, packed in [(1, 1, False, False), (0, 0, True, False), (1, 0, True, True)]:
        L = _layer(t, bias, relu)
        say(f"[case] {L} ws={ws} packed={packed} plan={hgc.conv2d_plan(L, ws, packed).as_dict()}")
        x, w, b = make_tensors(L, seed=100 + bias)
        y = run_layer(L, x, w, b, use_ws=ws, packed=packed)
        assert_full(oracle, L, x, w, b, y)


@pytest.mark.parametrize("t", SHAPES)
def test_integer_inputs_are_exact(oracle, t):
    L = _layer(t, 1, 0)
    if L.Kg * 8 + 8 > 2048:
        x, w, b = make_integer_tensors(L, seed=7, xmax=1, wmax=1)
        if L.Kg + 8 > 2048:
            pytest.skip("sums leave the exact range")
    else:
        x, w, b = make_integer_tensors(L, seed=7)
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, b)
    for ws, packed in ((False, False), (True, False), (True, True)):
        say(f"[int] {L} ws={ws} packed={packed}")
        y = run_layer(L, x, w, b, use_ws=ws, packed=packed)
        assert np.array_equal(y.astype(np.float64), pre), f"{L} ws={ws} packed={packed}"


def test_every_tile_variant_agrees_with_the_oracle(oracle):
    """Force each implicit-GEMM instantiation on a shape it accepts."""
    import ctypes
    probes = {1: (2, 64, 18, 20, 160, 1, 1, 0, 1), 3: (2, 32, 18, 20, 160, 3, 1, 1, 1),
              5: (1, 16, 18, 20, 96, 5, 1, 2, 1), 7: (1, 8, 18, 20, 48, 7, 1, 3, 1)}
    seen = 0
    try:
        for packed in (False, True):
            for v in range(128):
                for k, t in probes.items():
                    L = _layer(t)
                    hgc.set_forced_path(hgc.PATH_IGEMM, v)
                    p = hgc.conv2d_plan(L, packed, packed)
                    if p.path != hgc.PATH_IGEMM or p.variant != v:
                        continue
                    seen += 1
                    for ws in (False, True):
                        if packed and not ws:
                            continue
                        hgc.set_forced_path(hgc.PATH_IGEMM_SPLITK if ws else hgc.PATH_IGEMM, v)
                        say(f"[variant {v} packed={packed}] {L} ws={ws} plan={hgc.conv2d_plan(L, ws, packed).as_dict()}")
                        x, w, b = make_tensors(L, seed=v)
                        y = run_layer(L, x, w, b, use_ws=ws, packed=packed)
                        assert_full(oracle, L, x, w, b, y, tag=f"variant {v} packed={packed}")
    finally:
        hgc.set_forced_path(hgc.PATH_AUTO)
    assert seen >= 60


def test_two_steps_ahead_pipeline_at_every_step_count(oracle):
    """Instantiations that keep the loads two steps ahead: 1..6 channel blocks (odd and even
    counts, the one- and two-step prologues and tails), whole and split reductions."""
    ran = 0
    try:
        for packed in (False, True):
            for v in range(128):
                name = hgc.igemm_variant_name(v, packed)
                if not name:
                    break
                targs = name[name.index("<") + 1:].replace(" ", "").split(",")
                if targs[0] != "3" or targs[9] != "3":      # kernel extent 3, NSTAGE 3
                    continue
                cb = 8 * int(targs[5])
                for nblocks in (1, 2, 3, 4, 5, 6):
                    L = _layer((2, cb * nblocks - 8, 14, 24, 40, 3, 1, 1, 1))
                    for ws in (False, True):
                        if packed and not ws:
                            continue
                        hgc.set_forced_path(hgc.PATH_IGEMM_SPLITK if (ws and nblocks == 6) else hgc.PATH_IGEMM, v)
                        p = hgc.conv2d_plan(L, ws, packed)
                        if p.variant != v or p.path not in (hgc.PATH_IGEMM, hgc.PATH_IGEMM_SPLITK):
                            continue
                        say(f"[ahead2 variant {v} packed={packed}] {L} ws={ws} plan={p.as_dict()}")
                        x, w, b = make_tensors(L, seed=100 + v + nblocks)
                        y = run_layer(L, x, w, b, use_ws=ws, packed=packed)
                        assert_full(oracle, L, x, w, b, y, tag=f"ahead2 variant {v} packed={packed} blocks={nblocks}")
                        ran += 1
    finally:
        hgc.set_forced_path(hgc.PATH_AUTO)
    assert ran >= 40


def test_tuned_launch_shapes_keep_parity(oracle):
    """hgc_conv2d_tune remembers a measured shape: results stay within tolerance with it, the plan
    query reports it, a call with a smaller workspace falls back, and reset restores the model's plan."""
    import torch
    # the third takes the pointwise path (nothing to measure: run once as planned), the fourth is a 1x1 layer that cannot
    cases = [(1, 64, 28, 28, 96, 3, 1, 1, 1), (1, 256, 14, 14, 256, 3, 1, 1, 1), (2, 96, 14, 14, 160, 1, 1, 0, 1),
             (2, 96, 7, 7, 160, 1, 1, 0, 1)]
    try:
        for t in cases:
            L = _layer(t)
            x, w, b = make_tensors(L, seed=7)
            xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
            for packed in (False, True):
                hgc.conv2d_tune_reset()
                before = hgc.conv2d_plan(L, True, packed).as_dict()
                wbuf = hgc.conv2d_pack_weights(L, wd) if packed else wd
                need = hgc.conv2d_workspace_size(L)
                big = torch.empty(max(need, 16 << 20), dtype=torch.uint8, device="cuda")
                y = torch.empty(L.y_shape, dtype=torch.float16, device="cuda")
                say(f"[tune] {L} packed={packed} model plan {before}")
                chosen = hgc.conv2d_tune(L, xd, wbuf, bd, y, big, packed=packed).as_dict()
                torch.cuda.synchronize()
                assert_full(oracle, L, x, w, b, y.cpu().numpy(), tag=f"tune output packed={packed}")
                assert hgc.conv2d_plan(L, True, packed).as_dict() == chosen
                fwd = hgc.conv2d_forward_packed if packed else hgc.conv2d_forward_ws
                # the remembered shape, with the workspace it was measured with
                y.view(torch.int16).fill_(0x7E00)
                fwd(L, xd, wbuf, bd, y, big)
                torch.cuda.synchronize()
                assert_full(oracle, L, x, w, b, y.cpu().numpy(), tag=f"tuned {chosen} packed={packed}")
                # a workspace of only the advertised size: falls back where the shape needs more
                small = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
                y.view(torch.int16).fill_(0x7E00)
                fwd(L, xd, wbuf, bd, y, small)
                torch.cuda.synchronize()
                assert_full(oracle, L, x, w, b, y.cpu().numpy(), tag=f"tuned, small workspace packed={packed}")
                hgc.conv2d_tune_reset()
                assert hgc.conv2d_plan(L, True, packed).as_dict() == before
    finally:
        hgc.conv2d_tune_reset()


def test_direct_and_mfma_paths_agree(oracle):
    L = _layer((2, 32, 20, 22, 64, 3, 1, 1, 1))
    x, w, b = make_tensors(L, seed=1)
    try:
        hgc.set_forced_path(hgc.PATH_DIRECT)
        yd = run_layer(L, x, w, b)
        hgc.set_forced_path(hgc.PATH_IGEMM)
        ym = run_layer(L, x, w, b)
    finally:
        hgc.set_forced_path(hgc.PATH_AUTO)
    assert_full(oracle, L, x, w, b, yd, "direct")
    assert_full(oracle, L, x, w, b, ym, "igemm")
    # same call twice: bit-identical (no order-dependent accumulation)
    assert np.array_equal(run_layer(L, x, w, b, use_ws=True).view(np.uint16),
                          run_layer(L, x, w, b, use_ws=True).view(np.uint16))


def test_unaligned_base_pointers_fall_back(oracle):
    """Tensors that start 2 bytes into an allocation: vector loads are not allowed."""
    import torch
    L = _layer((1, 16, 12, 12, 32, 3, 1, 1, 1))
    x, w, b = make_tensors(L, seed=3)

    def shifted(a):
        buf = torch.zeros(a.size + 1, dtype=torch.float16, device="cuda")
        buf[1:] = torch.from_numpy(a.reshape(-1)).cuda()
        return buf, buf[1:].view(a.shape)

    xb, xs = shifted(x); wb, wsft = shifted(w); bb, bs = shifted(b)
    y = torch.empty(L.y_shape, dtype=torch.float16, device="cuda")
    d = hgc.ConvDesc.make(L)
    st = hgc.forward_raw(d, xs.data_ptr(), wsft.data_ptr(), bs.data_ptr(), y.data_ptr(),
                         torch.cuda.current_stream().cuda_stream)
    assert st == 0
    torch.cuda.synchronize()
    assert_full(oracle, L, x, w, b, y.cpu().numpy(), "unaligned")


@pytest.mark.parametrize("cfg", ["cfg1", "alexnet", "vgg16", "resnet50", "mobilenet_v1"])
def test_configs_batch1_full_tensor(oracle, cfg):
    worst = 0.0
    for i, L in enumerate(CONFIGS[cfg](1)):
        x, w, b = make_tensors(L, seed=layer_seed(cfg, i))
        pre, mag = oracle.conv2d_forward(L.desc(), x, w, b)
        for ws, packed in ((False, False), (True, False), (True, True)):
            say(f"[{cfg}] {L.name} ws={ws} packed={packed} plan={hgc.conv2d_plan(L, ws, packed).as_dict()}")
            y = run_layer(L, x, w, b, use_ws=ws, packed=packed)
            ok, ratio, where = oracle.check(y, pre, mag, L.relu)
            assert ok, f"{L} ws={ws} packed={packed}: |err|/bound={ratio:.3g} at {where}"
            worst = max(worst, ratio)
    say(f"[{cfg}] worst |err|/bound = {worst:.3f}")
    assert worst <= 1.0


@pytest.mark.parametrize("cfg,N", [("alexnet", 16), ("vgg16", 16), ("resnet50", 32), ("mobilenet_v1", 64)])
def test_configs_full_batch_sampled(oracle, cfg, N):
    """Full-size tensors in the launch configuration the benchmark uses; outputs the
    oracle evaluates one by one: corners, edges, first and last image, random points."""
    rng = np.random.default_rng(1234)
    for i, L in enumerate(CONFIGS[cfg](N)):
        x, w, b = make_tensors(L, seed=layer_seed(cfg, i))
        idx = sample_points(L, rng, 4000)
        for packed in (True, False):
            say(f"[{cfg} N={N}] {L.name} packed={packed} plan={hgc.conv2d_plan(L, True, packed).as_dict()}")
            y = run_layer(L, x, w, b, use_ws=True, packed=packed)
            assert_points(oracle, L, x, w, b, y, idx)
            assert np.isfinite(y.astype(np.float32)).all()


def test_packed_buffer_holds_the_weights_verbatim_and_zero_padding():
    """The pack kernel is pure data movement: check every byte it writes."""
    import torch
    L = _layer((1, 20, 9, 9, 12, 3, 1, 1, 2))            # Cg = 10, Mg = 6: ragged in both directions
    _, w, _ = make_tensors(L, seed=5)
    wd = torch.from_numpy(w).cuda()
    wp = hgc.conv2d_pack_weights(L, wd).cpu().numpy()
    raw = wp[:w.size * 2].view(np.float16).reshape(w.shape)
    assert np.array_equal(raw.view(np.uint16), w.view(np.uint16))
    T, Mg, Cg, G = 9, 6, 10, 2
    MB8, NP8 = 1, 2
    off = (w.size * 2 + 255) // 256 * 256
    assert not wp[w.size * 2:off].any()
    units = wp[off:off + G * MB8 * NP8 * T * 8 * 16].view(np.float16).reshape(G, MB8, NP8, T, 8, 8)
    want = np.zeros_like(units)
    wg = w.reshape(G, Mg, Cg, T)
    for g in range(G):
        for m in range(Mg):
            for c in range(Cg):
                want[g, m // 8, c // 8, :, m % 8, c % 8] = wg[g, m, c, :]
    assert np.array_equal(units.view(np.uint16), want.view(np.uint16))
    assert not wp[off + units.size * 2:].any() and wp.size == hgc.conv2d_packed_weights_size(L)


def test_first_layer_section_of_the_packed_buffer():
    """C <= 4: the extra section holds units [k rows][tap pairs][64-padded rows] of two taps x 4 channels."""
    import torch
    L = _layer((1, 3, 12, 12, 40, 7, 2, 3, 1))
    _, w, _ = make_tensors(L, seed=6)
    wp = hgc.conv2d_pack_weights(L, torch.from_numpy(w).cuda()).cpu().numpy()
    M, C, k = 40, 3, 7
    raw_end = (w.size * 2 + 255) // 256 * 256
    igemm_units = 1 * ((M + 7) // 8) * 1 * k * k * 8
    zero_off = raw_end + (igemm_units * 16 + 255) // 256 * 256
    c4_off = zero_off + 1024
    assert not wp[zero_off:c4_off].any()
    qpn, mpad = (k + 1) // 2, 64
    sec = wp[c4_off:c4_off + k * qpn * mpad * 16].view(np.float16).reshape(k, qpn, mpad, 2, 4)
    want = np.zeros_like(sec)
    for r in range(k):
        for q in range(k):
            want[r, q // 2, :M, q % 2, :C] = w[:, :, r, q]
    assert np.array_equal(sec.view(np.uint16), want.view(np.uint16))
    assert not wp[c4_off + sec.size * 2:].any() and wp.size == hgc.conv2d_packed_weights_size(L)


FIRST = [
    # N  C  H   W   M  k  s  p
    (1, 3, 224, 224, 64, 3, 1, 1),      # VGG conv1
    (2, 3, 224, 224, 64, 7, 2, 3),      # ResNet stem
    (2, 3, 224, 224, 32, 3, 2, 1),      # MobileNet conv1
    (1, 1, 28, 28, 20, 5, 1, 0),        # config-1-like: one channel, 5x5, M not a multiple of 32
    (3, 4, 17, 19, 48, 3, 1, 1),        # odd width: one-pixel loads; M = 48 (ragged second block)
    (2, 2, 9, 40, 70, 5, 2, 2),         # three M tiles of 32.., ragged everything
    (1, 3, 7, 7, 16, 7, 1, 3),          # kernel as large as the image
    (2, 3, 33, 66, 64, 3, 2, 0),        # no padding, stride 2
    (1, 3, 227, 227, 96, 11, 4, 0),     # AlexNet conv1: 11x11 stride 4 (patches of thousands of items)
    (2, 3, 64, 50, 40, 11, 4, 2),       # 11x11 with padding, ragged tiles, M = 40
    (1, 1, 31, 31, 16, 11, 1, 5),       # 11x11 stride 1, one channel, odd width
]


@pytest.mark.parametrize("t", FIRST, ids=[f"f{i}" for i in range(len(FIRST))])
def test_first_layer_kernel(oracle, t):
    N, C, H, W, M, k, s, p = t
    for bias, relu in ((1, 1), (0, 0)):
        L = ConvLayer("first", N, C, H, W, M, k, s, p, 1, bias, relu)
        x, w, b = make_tensors(L, seed=40 + k)
        # weights from the packed buffer's section, and gathered from the caller's layout
        for ws, packed in ((True, True), (True, False), (False, False)):
            plan = hgc.conv2d_plan(L, ws, packed).as_dict()
            assert plan["path"] == hgc.PATH_FIRST_LAYER, plan
            say(f"[first layer] {L} ws={ws} packed={packed} plan={plan}")
            y = run_layer(L, x, w, b, use_ws=ws, packed=packed)
            assert_full(oracle, L, x, w, b, y, tag=f"first layer packed={packed}")


def test_first_layer_kernel_integer_exact_and_unaligned_input(oracle):
    import torch
    L = ConvLayer("first", 2, 3, 20, 22, 40, 3, 1, 1, 1, 1, 0)
    x, w, b = make_integer_tensors(L, seed=3)
    pre, _ = oracle.conv2d_forward(L.desc(), x, w, b)
    y = run_layer(L, x, w, b, use_ws=True, packed=True)
    assert np.array_equal(y.astype(np.float64), pre)
    # x at a 2-byte aligned address: the one-pixel-load form
    x, w, b = make_tensors(L, seed=4)
    xbuf = torch.empty(x.size + 1, dtype=torch.float16, device="cuda")
    xbuf[1:].copy_(torch.from_numpy(x.reshape(-1)))
    xd = xbuf[1:].view(L.N, L.C, L.H, L.W)
    wp = hgc.conv2d_pack_weights(L, torch.from_numpy(w).cuda())
    yd = torch.empty(L.y_shape, dtype=torch.float16, device="cuda")
    yd.view(torch.int16).fill_(0x7E00)
    st = hgc.forward_packed_raw(hgc.ConvDesc.make(L), xd.data_ptr(), wp.data_ptr(), torch.from_numpy(b).cuda().data_ptr(),
                                yd.data_ptr(), 0, 0, torch.cuda.current_stream().cuda_stream)
    assert st == 0
    torch.cuda.synchronize()
    assert_full(oracle, L, x, w, b, yd.cpu().numpy(), tag="first layer, unaligned x")


def test_first_layer_kernel_caller_layout_with_unaligned_weights(oracle):
    """Weights in the caller's layout at a 2-byte aligned address: the kernel gathers them with 2-byte loads."""
    import torch
    for t in ((1, 3, 40, 44, 64, 3, 1, 1), (1, 3, 51, 51, 48, 11, 4, 0)):
        N, C, H, W, M, k, s_, p_ = t
        L = ConvLayer("first", N, C, H, W, M, k, s_, p_, 1, 1, 1)
        assert hgc.conv2d_plan(L, False, False).as_dict()["path"] == hgc.PATH_FIRST_LAYER
        x, w, b = make_tensors(L, seed=9)
        wbuf = torch.empty(w.size + 1, dtype=torch.float16, device="cuda")
        wbuf[1:].copy_(torch.from_numpy(w.reshape(-1)))
        xd, bd = torch.from_numpy(x).cuda(), torch.from_numpy(b).cuda()
        yd = torch.empty(L.y_shape, dtype=torch.float16, device="cuda")
        yd.view(torch.int16).fill_(0x7E00)
        st = hgc.forward_raw(hgc.ConvDesc.make(L), xd.data_ptr(), wbuf[1:].data_ptr(), bd.data_ptr(), yd.data_ptr(),
                             torch.cuda.current_stream().cuda_stream)
        assert st == 0
        torch.cuda.synchronize()
        assert_full(oracle, L, x, w, b, yd.cpu().numpy(), tag="first layer, unaligned w")


MULTI = [
    # N  C   H   W   M  k  s  p  G: small maps, image counts that do not fill the last tile
    (5, 64, 7, 7, 96, 3, 1, 1, 1),
    (7, 96, 7, 7, 64, 1, 1, 0, 1),
    (3, 32, 5, 9, 40, 3, 2, 1, 1),
    (6, 16, 14, 14, 32, 3, 1, 1, 2),
    (9, 24, 4, 4, 48, 1, 1, 0, 1),
    (4, 72, 7, 7, 160, 3, 1, 1, 1),
]


@pytest.mark.parametrize("t", MULTI, ids=[f"m{i}" for i in range(len(MULTI))])
def test_tiles_that_span_several_images(oracle, t):
    """Small feature maps share a workgroup tile: 2, 4 and 8 images per tile, whole and split
    reductions, both weight layouts; the planner's own choice as well."""
    L = _layer(t)
    x, w, b = make_tensors(L, seed=77)
    ran = 0
    try:
        for ti in (-1, 1, 2, 3):
            for split in (False, True):
                for packed in (False, True):
                    hgc.set_forced_path(hgc.PATH_IGEMM_SPLITK if split else (hgc.PATH_IGEMM if ti >= 0 else hgc.PATH_AUTO))
                    hgc.set_forced_tiling(-1, -1, ti)
                    plan = hgc.conv2d_plan(L, True, packed).as_dict()
                    if plan["path"] not in (hgc.PATH_IGEMM, hgc.PATH_IGEMM_SPLITK):
                        continue
                    if ti >= 0 and plan["tile_n"] != (1 << ti):
                        continue
                    say(f"[multi-image] {L} ti={ti} split={split} packed={packed} plan={plan}")
                    y = run_layer(L, x, w, b, use_ws=True, packed=packed)
                    assert_full(oracle, L, x, w, b, y, tag=f"tile_n={plan['tile_n']} split={plan['split_k']} packed={packed}")
                    ran += plan["tile_n"] > 1
    finally:
        hgc.set_forced_tiling(-1, -1, -1)
        hgc.set_forced_path(hgc.PATH_AUTO)
    assert ran >= 4

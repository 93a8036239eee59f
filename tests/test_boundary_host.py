"""Host-only tests of the C ABI: exported symbols, validation order, planning.

None of these touches a GPU: every error status is returned before any HIP call,
and the plan / workspace queries are plain host arithmetic.
"""
import ctypes
import os
import re

import pytest

import paper_1901_00858_amd as hgc
from paper_1901_00858_amd import ConvDesc
from workloads import CONFIGS, ConvLayer

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000  # a non-NULL address that is never dereferenced on the paths tested here


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hgc.library_path()):
        from paper_1901_00858_amd.build import build_library
        build_library()
    return hgc.load()


def test_every_declared_symbol_is_exported(lib):
    with open(os.path.join(ROOT, "include", "hgc.h")) as f:
        text = f.read()
    names = set(re.findall(r"\b(hgc_[a-z0-9_]+)\s*\(", text))
    assert {"hgc_conv2d_forward", "hgc_conv2d_forward_ws", "hgc_conv2d_workspace_size",
            "hgc_conv2d_plan", "hgc_set_forced_path", "hgc_status_string", "hgc_version"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layouts_match_header(lib):
    assert ctypes.sizeof(ConvDesc) == 44
    assert ctypes.sizeof(hgc.Plan) == 64
    assert ctypes.sizeof(hgc.InnerProductDesc) == 20


GOOD = (1, 4, 8, 8, 4, 3, 1, 1, 1, 1, 1)


def _d(**kw):
    names = ("N", "C", "H", "W", "num_output", "kernel", "stride", "pad", "group", "bias", "relu")
    v = dict(zip(names, GOOD)); v.update(kw)
    return ConvDesc(*[v[n] for n in names])


def test_null_pointers_come_first(lib):
    d = _d()
    assert hgc.forward_raw(None, FAKE, FAKE, FAKE, FAKE) == -1
    assert hgc.forward_raw(d, 0, FAKE, FAKE, FAKE) == -1
    assert hgc.forward_raw(d, FAKE, 0, FAKE, FAKE) == -1
    assert hgc.forward_raw(d, FAKE, FAKE, FAKE, 0) == -1
    assert hgc.forward_raw(d, FAKE, FAKE, 0, FAKE) == -1          # bias=1 needs b
    # NULL wins over a bad descriptor
    assert hgc.forward_raw(_d(stride=0), 0, FAKE, FAKE, FAKE) == -1
    n = ctypes.c_size_t()
    assert lib.hgc_conv2d_workspace_size(None, ctypes.byref(n)) == -1
    assert lib.hgc_conv2d_workspace_size(ctypes.byref(d), None) == -1
    assert lib.hgc_conv2d_plan(ctypes.byref(d), 0, None) == -1


@pytest.mark.parametrize("kw", [
    dict(N=0), dict(C=0), dict(H=0), dict(W=-1), dict(num_output=0), dict(kernel=0), dict(stride=0),
    dict(pad=-1), dict(group=0), dict(group=3), dict(C=6, group=3, num_output=4),
    dict(bias=2), dict(relu=-1), dict(kernel=11), dict(H=2, W=9, kernel=5, pad=1),
])
def test_bad_descriptors(lib, kw):
    d = _d(**kw)
    assert hgc.forward_raw(d, FAKE, FAKE, FAKE, FAKE) == -2
    assert hgc.forward_ws_raw(d, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30) == -2
    n = ctypes.c_size_t()
    assert lib.hgc_conv2d_workspace_size(ctypes.byref(d), ctypes.byref(n)) == -2
    with pytest.raises(hgc.HgcError):
        hgc.conv2d_plan(d)


def test_too_large(lib):
    assert hgc.forward_raw(_d(N=70000, C=64, H=224, W=224), FAKE, FAKE, FAKE, FAKE) == -3
    assert hgc.forward_raw(_d(num_output=4 << 20, C=1024, group=1), FAKE, FAKE, FAKE, FAKE) == -3
    assert hgc.forward_raw(_d(N=4096, num_output=4096, H=64, W=64, C=4), FAKE, FAKE, FAKE, FAKE) == -3


def test_workspace_is_checked_before_any_launch(lib):
    L = ConvLayer("small_p", 1, 512, 14, 14, 512, 3, 1, 1)
    need = hgc.conv2d_workspace_size(L)
    plan = hgc.conv2d_plan(L, with_workspace=True)
    assert plan.path == hgc.PATH_IGEMM_SPLITK and plan.split_k > 1
    assert need >= plan.workspace_bytes == 4 * plan.split_k * 512 * 14 * 14
    d = ConvDesc.make(L)
    assert hgc.forward_ws_raw(d, FAKE, FAKE, FAKE, FAKE, 0, 0) == -4
    # FAKE is 16-byte aligned, so the call plans like hgc_conv2d_plan does
    assert hgc.forward_ws_raw(d, FAKE, FAKE, FAKE, FAKE, FAKE, plan.workspace_bytes - 1) == -4
    # the workspace-free entry never needs one
    assert hgc.conv2d_plan(L, with_workspace=False).workspace_bytes == 0


def test_packed_entry_points_validate_on_the_host(lib):
    L = ConvLayer("pk", 1, 20, 9, 9, 12, 3, 1, 1, 2)
    size = hgc.conv2d_packed_weights_size(L)
    raw = 2 * 12 * 10 * 9
    units = 2 * 1 * 2 * 9 * 8 * 16
    assert size == (raw + 255) // 256 * 256 + (units + 255) // 256 * 256 + 1024
    d = ConvDesc.make(L)
    assert lib.hgc_conv2d_pack_weights(ctypes.byref(d), None, ctypes.c_void_p(FAKE), None) == -1
    assert lib.hgc_conv2d_pack_weights(ctypes.byref(d), ctypes.c_void_p(FAKE), ctypes.c_void_p(FAKE + 16), None) == -6
    assert hgc.forward_packed_raw(d, FAKE, 0, FAKE, FAKE, 0, 0) == -1
    assert hgc.forward_packed_raw(d, FAKE, FAKE + 16, FAKE, FAKE, 0, 0) == -6
    assert hgc.forward_packed_raw(_d(stride=0), FAKE, FAKE, FAKE, FAKE, 0, 0) == -2
    p = hgc.conv2d_plan(L, True, packed=True)
    assert p.path in hgc.PATH_NAMES


def test_tuning_call_validates_on_the_host(lib):
    """hgc_conv2d_tune: same error order as the forward call, all before any GPU work."""
    d = _d()
    assert hgc.tune_raw(None, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 20, False) == -1
    assert hgc.tune_raw(d, 0, FAKE, FAKE, FAKE, FAKE, 1 << 20, False) == -1
    assert hgc.tune_raw(d, FAKE, FAKE, 0, FAKE, FAKE, 1 << 20, True) == -1       # bias=1 needs b
    assert hgc.tune_raw(_d(stride=0), FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 20, False) == -2
    assert hgc.tune_raw(d, FAKE, FAKE + 16, FAKE, FAKE, FAKE, 1 << 20, True) == -6   # packed buffer alignment
    hgc.conv2d_tune_reset()                                                       # harmless when empty


def test_launch_shapes_can_be_restored_on_the_host(lib):
    """hgc_conv2d_set_launch_shape: accepts exactly the shapes the planner can produce."""
    import math
    L = (1, 64, 28, 28, 96, 3, 1, 1, 1, 1, 1)
    try:
        hgc.conv2d_tune_reset()
        model = hgc.conv2d_plan(L, True, True).as_dict()
        assert model["path"] in (hgc.PATH_IGEMM, hgc.PATH_IGEMM_SPLITK)
        d = hgc.ConvDesc.make(L)
        assert lib.hgc_conv2d_set_launch_shape(None, 1, 0, 5, 0, 1) == -1
        assert lib.hgc_conv2d_set_launch_shape(ctypes.byref(d), 1, 9999, 5, 0, 1) == -2
        assert lib.hgc_conv2d_set_launch_shape(ctypes.byref(d), 1, model["variant"], 30, 0, 1) == -2
        assert lib.hgc_conv2d_set_launch_shape(ctypes.byref(d), 1, model["variant"], 5, 3, 1) == -2   # N = 1: no 8-image tiles
        # another window of the same instantiation
        other = 4 if model["tile_w"] != 16 else 3
        hgc.conv2d_set_launch_shape(L, True, model["variant"], other, 1)
        now = hgc.conv2d_plan(L, True, True).as_dict()
        assert (now["variant"], now["tile_w"], now["split_k"]) == (model["variant"], 1 << other, 1)
        assert hgc.conv2d_plan(L, True, False).as_dict() == hgc.conv2d_plan(L, True, False).as_dict()
        hgc.conv2d_tune_reset()
        assert hgc.conv2d_plan(L, True, True).as_dict() == model
    finally:
        hgc.conv2d_tune_reset()


def test_inner_product_validates_on_the_host(lib):
    """hgc_inner_product_forward: NULL, then BAD_DESC, then TOO_LARGE, all before any GPU work."""
    ip = hgc.InnerProductDesc
    good = ip(2, 64, 10, 1, 0)
    assert hgc.inner_product_forward_raw(None, FAKE, FAKE, FAKE, FAKE) == -1
    assert hgc.inner_product_forward_raw(good, 0, FAKE, FAKE, FAKE) == -1
    assert hgc.inner_product_forward_raw(good, FAKE, 0, FAKE, FAKE) == -1
    assert hgc.inner_product_forward_raw(good, FAKE, FAKE, FAKE, 0) == -1
    assert hgc.inner_product_forward_raw(good, FAKE, FAKE, 0, FAKE) == -1          # bias=1 needs b
    assert hgc.inner_product_forward_raw(ip(0, 64, 10, 0, 0), 0, FAKE, FAKE, FAKE) == -1   # NULL wins
    for bad in (ip(0, 64, 10, 0, 0), ip(2, 0, 10, 0, 0), ip(2, 64, 0, 0, 0), ip(2, 64, 10, 2, 0), ip(2, 64, 10, 0, -1)):
        assert hgc.inner_product_forward_raw(bad, FAKE, FAKE, FAKE, FAKE) == -2
    assert hgc.inner_product_forward_raw(ip(1, 1 << 16, 1 << 16, 0, 0), FAKE, FAKE, FAKE, FAKE) == -3
    assert hgc.inner_product_forward_raw(ip(1 << 16, 1 << 16, 1, 0, 0), FAKE, FAKE, FAKE, FAKE) == -3
    assert hgc.inner_product_forward_raw(ip(1 << 16, 1, 1 << 16, 0, 0), FAKE, FAKE, FAKE, FAKE) == -3


def test_batch_norm_validates_on_the_host(lib):
    """hgc_batch_norm_forward: NULL, BAD_DESC, TOO_LARGE, WORKSPACE, in that order, before any GPU work."""
    def bn(N, C, H, W, g=0, sb=0, relu=0, eps=1e-5, ss=1.0):
        return hgc.BatchNormDesc(N, C, H, W, g, sb, relu, eps, ss)
    assert ctypes.sizeof(hgc.BatchNormDesc) == 36
    good = bn(2, 16, 14, 14)
    st, need = hgc.batch_norm_workspace_size_raw(good)
    assert st == 0 and need >= 8 * 16 + 8 * 2 * 16                   # coefficients + one partial per plane
    st, need_g = hgc.batch_norm_workspace_size_raw(bn(2, 16, 14, 14, g=1))
    assert st == 0 and 8 * 16 <= need_g < need
    st, big = hgc.batch_norm_workspace_size_raw(bn(2, 16, 100, 100))   # 10000 values a plane: 5 groups each
    assert st == 0 and big >= 8 * 2 * 16 * 5
    assert hgc.batch_norm_workspace_size_raw(None)[0] == -1
    ws = (FAKE, 1 << 20)
    assert hgc.batch_norm_forward_raw(None, FAKE, 0, 0, 0, 0, FAKE, *ws) == -1
    assert hgc.batch_norm_forward_raw(good, 0, 0, 0, 0, 0, FAKE, *ws) == -1
    assert hgc.batch_norm_forward_raw(good, FAKE, 0, 0, 0, 0, 0, *ws) == -1
    assert hgc.batch_norm_forward_raw(bn(2, 16, 14, 14, g=1), FAKE, FAKE, 0, 0, 0, FAKE, *ws) == -1     # var missing
    assert hgc.batch_norm_forward_raw(bn(2, 16, 14, 14, sb=1), FAKE, 0, 0, FAKE, 0, FAKE, *ws) == -1    # beta missing
    assert hgc.batch_norm_forward_raw(bn(0, 16, 14, 14), 0, 0, 0, 0, 0, FAKE, *ws) == -1                # NULL wins
    for bad in (bn(0, 1, 1, 1), bn(1, 0, 1, 1), bn(1, 1, 0, 1), bn(1, 1, 1, -3), bn(1, 1, 1, 1, g=2), bn(1, 1, 1, 1, sb=-1),
                bn(1, 1, 1, 1, relu=2), bn(1, 1, 1, 1, eps=0.0), bn(1, 1, 1, 1, eps=-1.0), bn(1, 1, 1, 1, eps=float("nan")),
                bn(1, 1, 1, 1, eps=float("inf"))):
        assert hgc.batch_norm_forward_raw(bad, FAKE, 0, 0, 0, 0, FAKE, *ws) == -2
        assert hgc.batch_norm_workspace_size_raw(bad)[0] == -2
    assert hgc.batch_norm_forward_raw(bn(1, 1, 1, 1, g=1, ss=0.0), FAKE, FAKE, FAKE, 0, 0, FAKE, *ws) == -2
    assert hgc.batch_norm_forward_raw(bn(1, 1, 1, 1, g=0, ss=0.0), FAKE, 0, 0, 0, 0, FAKE, FAKE, 0) == -4   # ignored without stored statistics
    assert hgc.batch_norm_forward_raw(bn(1 << 10, 1 << 10, 1 << 6, 1 << 5), FAKE, 0, 0, 0, 0, FAKE, *ws) == -3
    assert hgc.batch_norm_forward_raw(good, FAKE, 0, 0, 0, 0, FAKE, 0, 1 << 20) == -4
    assert hgc.batch_norm_forward_raw(good, FAKE, 0, 0, 0, 0, FAKE, FAKE, need - 1) == -4


def test_batch_norm_fold_validates_on_the_host(lib):
    d = ConvDesc(1, 16, 8, 8, 32, 3, 1, 1, 1, 1, 1)
    f = lambda conv, *p, ss=1.0, eps=1e-5: hgc.batch_norm_fold_raw(conv, p[0], p[1], p[2], p[3], ss, eps, p[4], p[5], p[6], p[7])
    ok = (FAKE,) * 8
    assert f(None, *ok) == -1
    for missing in (0, 1, 2, 3, 6, 7):                        # w, b (bias = 1), mean, var, w_out, b_out
        p = list(ok); p[missing] = 0
        assert f(d, *p) == -1
    p = list(ok); p[4] = 0
    assert f(d, *p) == -1                                     # gamma without beta
    nobias = ConvDesc(1, 16, 8, 8, 32, 3, 1, 1, 1, 0, 1)
    p = list(ok); p[1] = 0
    assert f(ConvDesc(1, 16, 8, 8, 32, 3, 1, 1, 3, 0, 1), *p) == -2      # 16 channels in 3 groups
    assert f(ConvDesc(1, 0, 8, 8, 32, 3, 1, 1, 1, 0, 1), *p) == -2
    assert f(nobias, *p, eps=0.0) == -2
    assert f(nobias, *p, ss=-1.0) == -2
    assert f(ConvDesc(1, 1 << 14, 8, 8, 1 << 14, 3, 1, 1, 1, 0, 1), *p) == -3


def test_max_pool_validates_on_the_host(lib):
    """hgc_max_pool_forward / hgc_max_pool_output_size: NULL, BAD_DESC, TOO_LARGE before any GPU work."""
    mp = hgc.MaxPoolDesc
    assert ctypes.sizeof(mp) == 28
    assert hgc.max_pool_output_size_raw(mp(1, 64, 224, 224, 2, 2, 0)) == (0, 112, 112)
    assert hgc.max_pool_output_size_raw(mp(1, 96, 55, 55, 3, 2, 0)) == (0, 27, 27)
    assert hgc.max_pool_output_size_raw(mp(1, 64, 112, 112, 3, 2, 1)) == (0, 57, 57)     # rounded up
    assert hgc.max_pool_output_size_raw(mp(1, 1, 3, 3, 2, 2, 1)) == (0, 2, 2)             # last window in the padding: dropped
    assert hgc.max_pool_output_size_raw(None)[0] == -1
    good = mp(2, 3, 8, 8, 2, 2, 0)
    assert hgc.max_pool_forward_raw(None, FAKE, FAKE) == -1
    assert hgc.max_pool_forward_raw(good, 0, FAKE) == -1
    assert hgc.max_pool_forward_raw(good, FAKE, 0) == -1
    assert hgc.max_pool_forward_raw(mp(0, 3, 8, 8, 2, 2, 0), 0, FAKE) == -1               # NULL wins
    for bad in (mp(0, 3, 8, 8, 2, 2, 0), mp(1, 0, 8, 8, 2, 2, 0), mp(1, 1, 0, 8, 2, 2, 0), mp(1, 1, 8, -1, 2, 2, 0),
                mp(1, 1, 8, 8, 0, 2, 0), mp(1, 1, 8, 8, 2, 0, 0), mp(1, 1, 8, 8, 2, 2, -1), mp(1, 1, 8, 8, 2, 2, 2),
                mp(1, 1, 2, 8, 3, 1, 0)):
        assert hgc.max_pool_forward_raw(bad, FAKE, FAKE) == -2
        assert hgc.max_pool_output_size_raw(bad)[0] == -2
    assert hgc.max_pool_forward_raw(mp(1 << 10, 1 << 10, 1 << 6, 1 << 5, 2, 2, 0), FAKE, FAKE) == -3


def test_status_strings(lib):
    seen = {hgc.status_string(s) for s in (0, -1, -2, -3, -4, -5, -6)}
    assert len(seen) == 7 and hgc.status_string(0) == "ok"
    assert hgc.status_string(-99) == "unknown status"
    assert hgc.version() >= 100


def test_plans_for_every_benchmark_layer(lib):
    for name, fn in CONFIGS.items():
        for N in (1, 16):
            for L in fn(N):
                for ws in (False, True):
                    p = hgc.conv2d_plan(L, ws)
                    assert (p.Ho, p.Wo) == (L.Ho, L.Wo)
                    assert p.path in hgc.PATH_NAMES and p.grid >= 1 and p.block in (128, 256, 512)
                    assert p.lds_bytes <= 160 * 1024
                    if p.path in (hgc.PATH_IGEMM, hgc.PATH_IGEMM_SPLITK):
                        assert p.tile_n * p.tile_h * p.tile_w in (128, 256, 512) and p.tile_m in (32, 64, 128, 256)
                    if not ws:
                        assert p.workspace_bytes == 0 and p.split_k == 1
                    else:
                        assert hgc.conv2d_workspace_size(L) >= p.workspace_bytes
                    if L.G == L.C == L.M and L.k == 3:
                        assert p.path == hgc.PATH_DEPTHWISE


def test_forced_path_round_trip(lib):
    L = ConvLayer("f", 1, 64, 56, 56, 64, 3, 1, 1)
    try:
        assert hgc.set_forced_path(hgc.PATH_DIRECT) == hgc.PATH_AUTO
        assert hgc.conv2d_plan(L).path == hgc.PATH_DIRECT
        assert hgc.set_forced_path(hgc.PATH_IGEMM) == hgc.PATH_DIRECT
        assert hgc.conv2d_plan(L, True).path == hgc.PATH_IGEMM
        hgc.set_forced_path(hgc.PATH_DEPTHWISE)          # not applicable -> direct
        assert hgc.conv2d_plan(L).path == hgc.PATH_DIRECT
        hgc.set_forced_path(hgc.PATH_IGEMM, 9999)        # no such instantiation -> direct
        assert hgc.conv2d_plan(L).path == hgc.PATH_DIRECT
    finally:
        hgc.set_forced_path(hgc.PATH_AUTO)
    assert hgc.conv2d_plan(L).path == hgc.PATH_IGEMM


def test_binding_refuses_cpu_tensors(lib):
    torch = pytest.importorskip("torch")
    L = ConvLayer("c", 1, 4, 8, 8, 4, 3, 1, 1)
    x = torch.zeros(L.x_shape, dtype=torch.float16)
    w = torch.zeros(L.w_shape, dtype=torch.float16)
    b = torch.zeros(L.M, dtype=torch.float16)
    with pytest.raises(TypeError):
        hgc.conv2d_forward(L, x, w, b)


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1901_00858_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                with open(os.path.join(dirpath, f)) as fh:
                    text = fh.read()
                assert "oracle" not in text.lower(), f
    with open(os.path.join(ROOT, "oracle", "__init__.py")) as fh:
        assert "paper_1901_00858_amd" not in fh.read().replace("never imports the product package", "")


def test_instantiation_tables_are_joined_in_order(lib):
    """The implicit-GEMM tables are compiled in parts and joined: same length for both weight layouts,
    no instantiation twice, and the numbering that plans and remembered launch shapes refer to starts
    with the throughput tile."""
    for packed in (False, True):
        names = []
        while True:
            n = hgc.igemm_variant_name(len(names), packed)
            if not n:
                break
            names.append(n)
        assert len(names) >= 90 and len(set(names)) == len(names)
        assert names[0].startswith("igemm_kernel<3, 2, 4, 2, 4, 2, 4,"), names[0]
        assert all(n.split(",")[8].strip() == ("true" if packed else "false") for n in names)
        if packed:
            count = len(names)
        else:
            first = names
    assert count == len(first)
    assert hgc.igemm_variant_name(10 ** 6, True) == ""

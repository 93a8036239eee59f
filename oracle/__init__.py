"""Python face of the CPU oracle (oracle/conv2d_oracle.c, inner_product_oracle.c, batch_norm_oracle.c,
max_pool_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module,
and this module never imports the product package.

The oracle evaluates the layer's plain definition (Caffe convolution forward as
kept by the paper, Sections 2 and 5) in FP64 over FP16 inputs; see the C file's
header for the formula.  Here only: building/loading the shared object, argument
marshalling, and the two things a comparison needs on top of the raw sums --
the ReLU of the FP64 pre-activation and the tolerance
|gpu - oracle| <= 4e-3 * sum|w*x| + 1e-3 stated for this build.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "conv2d_oracle.c")
_SRC_IP = os.path.join(_DIR, "inner_product_oracle.c")
_SRC_BN = os.path.join(_DIR, "batch_norm_oracle.c")
_SRC_MP = os.path.join(_DIR, "max_pool_oracle.c")
_LIB = os.path.join(_DIR, "libhgo.so")
_lib = None

REL_TOL = 4e-3
ABS_TOL = 1e-3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp).  Returns the library path."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_IP), os.path.getmtime(_SRC_BN), os.path.getmtime(_SRC_MP))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, _SRC_IP, _SRC_BN, _SRC_MP, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.hgo_half_to_double.argtypes = [ctypes.c_uint16]
        lib.hgo_half_to_double.restype = ctypes.c_double
        lib.hgo_conv2d_forward.argtypes = [i32p, u16p, u16p, u16p, f64p, f64p]
        lib.hgo_conv2d_forward.restype = ctypes.c_int
        lib.hgo_conv2d_points.argtypes = [i32p, u16p, u16p, u16p, ctypes.c_longlong, i32p, f64p, f64p]
        lib.hgo_conv2d_points.restype = ctypes.c_int
        lib.hgo_inner_product_forward.argtypes = [i32p, u16p, u16p, u16p, f64p, f64p]
        lib.hgo_inner_product_forward.restype = ctypes.c_int
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.hgo_batch_norm_forward.argtypes = [i32p, ctypes.c_double, ctypes.c_double, u16p, f32p, f32p,
                                               f64p, f64p, f64p, f64p]
        lib.hgo_batch_norm_forward.restype = ctypes.c_int
        lib.hgo_batch_norm_fold.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double, u16p, u16p,
                                            f32p, f32p, f64p, f64p]
        lib.hgo_batch_norm_fold.restype = ctypes.c_int
        lib.hgo_max_pool_shape.argtypes = [i32p, i32p]
        lib.hgo_max_pool_shape.restype = ctypes.c_int
        lib.hgo_max_pool_forward.argtypes = [i32p, u16p, u16p]
        lib.hgo_max_pool_forward.restype = ctypes.c_int
        lib.hgo_num_threads.restype = ctypes.c_int
        lib.hgo_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _u16(a: Optional[np.ndarray]):
    if a is None:
        return None, ctypes.POINTER(ctypes.c_uint16)()
    a = np.ascontiguousarray(a, dtype=np.float16)
    return a, a.view(np.uint16).ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _desc(desc: Sequence[int]):
    d = np.asarray(desc, dtype=np.int32)
    assert d.shape == (11,), "desc = (N,C,H,W,num_output,kernel,stride,pad,group,bias,relu)"
    return d, d.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def out_shape(desc: Sequence[int]) -> Tuple[int, int, int, int]:
    N, C, H, W, M, k, s, p = [int(v) for v in desc[:8]]
    if s < 1 or k < 1 or H + 2 * p < k or W + 2 * p < k:
        raise ValueError("descriptor has no output")
    return (N, M, (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1)


def half_to_double(bits: int) -> float:
    return float(_load().hgo_half_to_double(int(bits)))


def num_threads() -> int:
    return int(_load().hgo_num_threads())


def set_num_threads(n: int) -> None:
    _load().hgo_set_num_threads(int(n))


def conv2d_forward(desc, x, w, b=None):
    """Full tensor: returns (pre, mag), FP64 arrays of shape [N][M][Ho][Wo].

    pre = bias + sum of products (before ReLU); mag = sum of |products|.
    """
    lib = _load()
    d, dp = _desc(desc)
    xk, xp = _u16(x)
    wk, wp = _u16(w)
    bk, bp = _u16(b if d[9] else None)
    if d[9] and b is None:
        raise ValueError("bias=1 needs b")
    shape = out_shape(d)
    pre = np.empty(shape, dtype=np.float64)
    mag = np.empty(shape, dtype=np.float64)
    f64p = ctypes.POINTER(ctypes.c_double)
    rc = lib.hgo_conv2d_forward(dp, xp, wp, bp, pre.ctypes.data_as(f64p), mag.ctypes.data_as(f64p))
    if rc:
        raise ValueError(f"oracle rejected the descriptor (rc={rc})")
    return pre, mag


def conv2d_points(desc, x, w, b, idx):
    """Selected outputs: idx is an int array [npts][4] of (n, m, oh, ow). Returns (pre, mag)."""
    lib = _load()
    d, dp = _desc(desc)
    xk, xp = _u16(x)
    wk, wp = _u16(w)
    bk, bp = _u16(b if d[9] else None)
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 4)
    n = idx.shape[0]
    pre = np.empty(n, dtype=np.float64)
    mag = np.empty(n, dtype=np.float64)
    f64p = ctypes.POINTER(ctypes.c_double)
    rc = lib.hgo_conv2d_points(dp, xp, wp, bp, n, idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                               pre.ctypes.data_as(f64p), mag.ctypes.data_as(f64p))
    if rc:
        raise ValueError(f"oracle rejected the request (rc={rc})")
    return pre, mag


def inner_product_forward(desc, x, w, b=None):
    """Inner-product layer (inner_product_oracle.c): desc = (N, K, M, bias, relu), x [N][K], w [M][K], b [M].

    Returns (pre, mag), FP64 arrays of shape [N][M]: bias + sum of products, and sum of |products|.
    """
    lib = _load()
    d = [int(v) for v in desc]
    if len(d) != 5:
        raise ValueError("desc = (N, K, M, bias, relu)")
    if d[0] < 1 or d[1] < 1 or d[2] < 1 or d[3] not in (0, 1) or d[4] not in (0, 1):
        raise ValueError("bad inner-product descriptor")
    if d[3] and b is None:
        raise ValueError("bias=1 needs b")
    x = np.asarray(x)
    w = np.asarray(w)
    if x.size != d[0] * d[1] or w.size != d[2] * d[1] or (d[3] and np.asarray(b).size != d[2]):
        raise ValueError("tensor sizes do not match the descriptor")
    dk = (ctypes.c_int32 * 5)(*d)
    xk, xp = _u16(x)
    wk, wp = _u16(w)
    bk, bp = _u16(b if d[3] else None)
    pre = np.empty((d[0], d[2]), dtype=np.float64)
    mag = np.empty((d[0], d[2]), dtype=np.float64)
    f64p = ctypes.POINTER(ctypes.c_double)
    rc = lib.hgo_inner_product_forward(dk, xp, wp, bp, pre.ctypes.data_as(f64p), mag.ctypes.data_as(f64p))
    if rc:
        raise ValueError(f"oracle rejected the descriptor (rc={rc})")
    return pre, mag


BN_REL_TOL = 1e-3      # of |y|: the one FP16 rounding at the store is 2^-11 = 4.9e-4 of it
BN_MAG_TOL = 2e-5      # of mag: FP32 statistics and the FP32 multiply-add, about 300 * 2^-24
BN_ABS_TOL = 1e-7      # FP16's smallest subnormal step is 6e-8


def batch_norm_forward(desc, x, eps=1e-5, mean=None, var=None, stat_scale=1.0, gamma=None, beta=None):
    """Batch-norm layer (batch_norm_oracle.c): desc = (N, C, H, W, use_global_stats, scale_bias, relu).

    x: FP16 [N][C][H][W]; mean/var (use_global_stats = 1) and gamma/beta (scale_bias = 1): FP32 [C].
    Returns (pre, mag, mean, var): FP64 [N][C][H][W] twice, then the statistics used, FP64 [C].
    """
    lib = _load()
    d = [int(v) for v in desc]
    if len(d) != 7:
        raise ValueError("desc = (N, C, H, W, use_global_stats, scale_bias, relu)")
    N, C, H, W = d[:4]
    if min(N, C, H, W) < 1:
        raise ValueError("bad batch-norm descriptor")
    x = np.asarray(x)
    if x.size != N * C * H * W:
        raise ValueError("tensor size does not match the descriptor")
    dk = (ctypes.c_int32 * 7)(*d)
    xk, xp = _u16(x)
    f32p = ctypes.POINTER(ctypes.c_float)
    f64p = ctypes.POINTER(ctypes.c_double)

    def pair(a, b, what):
        if a is None or b is None:
            raise ValueError(what)
        both = np.concatenate([np.asarray(a, dtype=np.float32).reshape(-1), np.asarray(b, dtype=np.float32).reshape(-1)])
        if both.size != 2 * C:
            raise ValueError(what)
        return np.ascontiguousarray(both)

    stats = pair(mean, var, "use_global_stats=1 needs mean and var of C values") if d[4] else None
    gb = pair(gamma, beta, "scale_bias=1 needs gamma and beta of C values") if d[5] else None
    pre = np.empty((N, C, H, W), dtype=np.float64)
    mag = np.empty((N, C, H, W), dtype=np.float64)
    mu = np.empty(C, dtype=np.float64)
    vv = np.empty(C, dtype=np.float64)
    rc = lib.hgo_batch_norm_forward(dk, float(eps), float(stat_scale), xp,
                                    stats.ctypes.data_as(f32p) if stats is not None else f32p(),
                                    gb.ctypes.data_as(f32p) if gb is not None else f32p(),
                                    pre.ctypes.data_as(f64p), mag.ctypes.data_as(f64p),
                                    mu.ctypes.data_as(f64p), vv.ctypes.data_as(f64p))
    if rc:
        raise ValueError(f"oracle rejected the descriptor (rc={rc})")
    return pre, mag, mu, vv


def batch_norm_fold(w, b, mean, var, eps=1e-5, stat_scale=1.0, gamma=None, beta=None):
    """Stored batch-norm statistics folded into a convolution's weights and bias (batch_norm_oracle.c).

    w: FP16 [M][...]; b: FP16 [M] or None; mean, var, gamma, beta: FP32 [M] (gamma and beta together or not at
    all).  Returns (w', b') in FP64, unrounded, w' shaped like w.
    """
    lib = _load()
    w = np.asarray(w)
    M = int(w.shape[0])
    per = int(w.size // M)
    stats = np.ascontiguousarray(np.concatenate([np.asarray(mean, dtype=np.float32).reshape(-1),
                                                 np.asarray(var, dtype=np.float32).reshape(-1)]))
    if stats.size != 2 * M or (gamma is None) != (beta is None):
        raise ValueError("mean and var need M values each; gamma and beta come together")
    gb = None
    if gamma is not None:
        gb = np.ascontiguousarray(np.concatenate([np.asarray(gamma, dtype=np.float32).reshape(-1),
                                                  np.asarray(beta, dtype=np.float32).reshape(-1)]))
        if gb.size != 2 * M:
            raise ValueError("gamma and beta need M values each")
    f32p = ctypes.POINTER(ctypes.c_float)
    f64p = ctypes.POINTER(ctypes.c_double)
    wk, wp = _u16(w)
    bk, bp = _u16(b)
    wo = np.empty(w.shape, dtype=np.float64)
    bo = np.empty(M, dtype=np.float64)
    rc = lib.hgo_batch_norm_fold(M, per, float(eps), float(stat_scale), wp, bp, stats.ctypes.data_as(f32p),
                                 gb.ctypes.data_as(f32p) if gb is not None else f32p(),
                                 wo.ctypes.data_as(f64p), bo.ctypes.data_as(f64p))
    if rc:
        raise ValueError(f"oracle rejected the request (rc={rc})")
    return wo, bo


def check_batch_norm(y, pre, mag, relu):
    """Compare an FP16 batch-norm result with the oracle: |y - ref| <= 1e-3 |ref| + 2e-5 mag + 1e-7.

    Returns (ok, worst ratio |err|/bound, index).
    """
    ref = np.maximum(pre, 0.0) if relu else pre
    bound = BN_REL_TOL * np.abs(ref) + BN_MAG_TOL * mag + BN_ABS_TOL
    yd = np.asarray(y).astype(np.float64).reshape(ref.shape)
    err = np.abs(yd - ref)
    ratio = np.where(~np.isfinite(yd), np.inf, err / bound)
    worst = int(np.argmax(ratio))
    r = float(ratio.reshape(-1)[worst])
    return bool(r <= 1.0), r, np.unravel_index(worst, ref.shape)


def max_pool_shape(desc):
    """(Ho, Wo) of Caffe's max pooling for desc = (N, C, H, W, kernel, stride, pad)."""
    d = (ctypes.c_int32 * 7)(*[int(v) for v in desc])
    o = (ctypes.c_int32 * 2)()
    if len(desc) != 7 or _load().hgo_max_pool_shape(d, o):
        raise ValueError("bad max-pool descriptor")
    return int(o[0]), int(o[1])


def max_pool_forward(desc, x):
    """Max pooling (max_pool_oracle.c): x FP16 [N][C][H][W] -> FP16 [N][C][Ho][Wo], exact."""
    ho, wo = max_pool_shape(desc)
    N, C, H, W = [int(v) for v in desc[:4]]
    x = np.asarray(x)
    if x.size != N * C * H * W:
        raise ValueError("tensor size does not match the descriptor")
    xk, xp = _u16(x)
    y = np.empty((N, C, ho, wo), dtype=np.float16)
    d = (ctypes.c_int32 * 7)(*[int(v) for v in desc])
    rc = _load().hgo_max_pool_forward(d, xp, y.view(np.uint16).ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    if rc:
        raise ValueError(f"oracle rejected the descriptor (rc={rc})")
    return y


def reference(pre: np.ndarray, mag: np.ndarray, relu: int):
    """(ref, bound): the FP64 expected output and the allowed absolute deviation.

    The bound is formed from the pre-ReLU taps only (the bias is not part of
    sum|w*x|); ReLU is 1-Lipschitz, so the same bound holds after it.
    """
    ref = np.maximum(pre, 0.0) if relu else pre
    return ref, REL_TOL * mag + ABS_TOL


def check(y, pre, mag, relu):
    """Compare an FP16 result with the oracle. Returns (ok, worst ratio |err|/bound, index)."""
    ref, bound = reference(pre, mag, relu)
    yd = np.asarray(y).astype(np.float64).reshape(ref.shape)
    err = np.abs(yd - ref)
    bad = ~np.isfinite(yd)
    ratio = np.where(bad, np.inf, err / bound)
    worst = int(np.argmax(ratio))
    r = float(ratio.reshape(-1)[worst])
    return bool(r <= 1.0), r, np.unravel_index(worst, ref.shape)

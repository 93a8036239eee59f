"""ctypes binding of include/hgc.h.  Argument marshalling only.

Tensors are torch CUDA tensors (torch is used for device memory and streams and
for nothing else); the functions pass their data pointers and the current
stream's handle to the C entry points of the same name.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libhgc.so")
_lib = None

PATH_AUTO, PATH_DIRECT, PATH_IGEMM, PATH_IGEMM_SPLITK, PATH_DEPTHWISE = 0, 1, 2, 3, 4
PATH_FIRST_LAYER = 5
PATH_POINTWISE = 6
PATH_NAMES = {1: "direct", 2: "igemm", 3: "igemm_splitk", 4: "depthwise", 5: "first_layer", 6: "pointwise"}


class HgcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = ""
        if status == -5:
            detail = " [" + load().hgc_last_launch_error().decode() + "]"
        super().__init__(f"{where}: {status_string(status)} (status {status}){detail}")


class ConvDesc(ctypes.Structure):
    """hgc_conv2d_desc: eleven int32 fields in host memory."""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "num_output", "kernel", "stride", "pad", "group", "bias", "relu")]

    @classmethod
    def make(cls, desc) -> "ConvDesc":
        if isinstance(desc, cls):
            return desc
        if hasattr(desc, "desc"):
            desc = desc.desc()
        vals = [int(v) for v in desc]
        if len(vals) != 11:
            raise ValueError("desc = (N,C,H,W,num_output,kernel,stride,pad,group,bias,relu)")
        return cls(*vals)

    def out_shape(self):
        ho = (self.H + 2 * self.pad - self.kernel) // self.stride + 1
        wo = (self.W + 2 * self.pad - self.kernel) // self.stride + 1
        return (self.N, self.num_output, ho, wo)


class InnerProductDesc(ctypes.Structure):
    """hgc_inner_product_desc: five int32 fields in host memory."""
    _fields_ = [(n, ctypes.c_int32) for n in ("N", "K", "num_output", "bias", "relu")]

    @classmethod
    def make(cls, desc) -> "InnerProductDesc":
        if isinstance(desc, cls):
            return desc
        vals = [int(v) for v in desc]
        if len(vals) != 5:
            raise ValueError("desc = (N, K, num_output, bias, relu)")
        return cls(*vals)


class BatchNormDesc(ctypes.Structure):
    """hgc_batch_norm_desc: seven int32 fields and two floats in host memory."""
    _fields_ = [(n, ctypes.c_int32) for n in ("N", "C", "H", "W", "use_global_stats", "scale_bias", "relu")] + \
               [("eps", ctypes.c_float), ("stat_scale", ctypes.c_float)]

    @classmethod
    def make(cls, desc, eps: float = 1e-5, stat_scale: float = 1.0) -> "BatchNormDesc":
        if isinstance(desc, cls):
            return desc
        vals = [int(v) for v in desc]
        if len(vals) != 7:
            raise ValueError("desc = (N, C, H, W, use_global_stats, scale_bias, relu)")
        return cls(*vals, float(eps), float(stat_scale))


class MaxPoolDesc(ctypes.Structure):
    """hgc_max_pool_desc: seven int32 fields in host memory."""
    _fields_ = [(n, ctypes.c_int32) for n in ("N", "C", "H", "W", "kernel", "stride", "pad")]

    @classmethod
    def make(cls, desc) -> "MaxPoolDesc":
        if isinstance(desc, cls):
            return desc
        vals = [int(v) for v in desc]
        if len(vals) != 7:
            raise ValueError("desc = (N, C, H, W, kernel, stride, pad)")
        return cls(*vals)


class Plan(ctypes.Structure):
    """hgc_plan."""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("path", "Ho", "Wo", "tile_m", "tile_h", "tile_w", "split_k", "variant", "grid", "block")] + \
               [("workspace_bytes", ctypes.c_int64), ("lds_bytes", ctypes.c_int64),
                ("tile_n", ctypes.c_int32), ("reserved", ctypes.c_int32)]

    def as_dict(self):
        d = {n: int(getattr(self, n)) for n, _ in self._fields_}
        d["path_name"] = PATH_NAMES.get(d["path"], "?")
        return d


def library_path() -> str:
    return _LIB_PATH


def load():
    """Load libhgc.so. Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_1901_00858_amd.build` "
            "(or __graft_entry__.build()); there is no fallback implementation")
    # PyTorch brings its own copy of the HIP runtime; whichever copy is loaded first serves the whole
    # process, and device memory and streams come from PyTorch's, so it has to be that one
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, dp = ctypes.c_void_p, ctypes.POINTER(ConvDesc)
    lib.hgc_conv2d_forward.argtypes = [dp, vp, vp, vp, vp, vp]
    lib.hgc_conv2d_forward.restype = ctypes.c_int32
    lib.hgc_conv2d_forward_ws.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hgc_conv2d_forward_ws.restype = ctypes.c_int32
    lib.hgc_conv2d_workspace_size.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
    lib.hgc_conv2d_workspace_size.restype = ctypes.c_int32
    lib.hgc_conv2d_plan.argtypes = [dp, ctypes.c_int32, ctypes.POINTER(Plan)]
    lib.hgc_conv2d_plan.restype = ctypes.c_int32
    lib.hgc_set_forced_path.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.hgc_set_forced_path.restype = ctypes.c_int32
    lib.hgc_conv2d_packed_weights_size.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
    lib.hgc_conv2d_packed_weights_size.restype = ctypes.c_int32
    lib.hgc_conv2d_pack_weights.argtypes = [dp, vp, vp, vp]
    lib.hgc_conv2d_pack_weights.restype = ctypes.c_int32
    lib.hgc_conv2d_forward_packed.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hgc_conv2d_forward_packed.restype = ctypes.c_int32
    lib.hgc_conv2d_tune.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_size_t, ctypes.c_int32, vp, ctypes.POINTER(Plan)]
    lib.hgc_conv2d_tune.restype = ctypes.c_int32
    lib.hgc_conv2d_set_launch_shape.argtypes = [dp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                ctypes.c_int32]
    lib.hgc_conv2d_set_launch_shape.restype = ctypes.c_int32
    lib.hgc_conv2d_tune_reset.argtypes = []
    lib.hgc_conv2d_tune_reset.restype = None
    lib.hgc_set_forced_tiling.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
    lib.hgc_set_forced_tiling.restype = None
    lib.hgc_inner_product_forward.argtypes = [ctypes.POINTER(InnerProductDesc), vp, vp, vp, vp, vp]
    lib.hgc_inner_product_forward.restype = ctypes.c_int32
    bp = ctypes.POINTER(BatchNormDesc)
    lib.hgc_batch_norm_workspace_size.argtypes = [bp, ctypes.POINTER(ctypes.c_size_t)]
    lib.hgc_batch_norm_workspace_size.restype = ctypes.c_int32
    lib.hgc_batch_norm_forward.argtypes = [bp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hgc_batch_norm_forward.restype = ctypes.c_int32
    lib.hgc_batch_norm_fold.argtypes = [dp, vp, vp, vp, vp, ctypes.c_float, ctypes.c_float, vp, vp, vp, vp, vp]
    lib.hgc_batch_norm_fold.restype = ctypes.c_int32
    mp = ctypes.POINTER(MaxPoolDesc)
    lib.hgc_max_pool_output_size.argtypes = [mp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    lib.hgc_max_pool_output_size.restype = ctypes.c_int32
    lib.hgc_max_pool_forward.argtypes = [mp, vp, vp, vp]
    lib.hgc_max_pool_forward.restype = ctypes.c_int32
    lib.hgc_status_string.argtypes = [ctypes.c_int32]
    lib.hgc_status_string.restype = ctypes.c_char_p
    lib.hgc_version.restype = ctypes.c_int32
    lib.hgc_igemm_variant_name.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_char_p, ctypes.c_int32]
    lib.hgc_igemm_variant_name.restype = ctypes.c_int32
    lib.hgc_last_launch_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().hgc_status_string(int(status)).decode()


def version() -> int:
    return int(load().hgc_version())


def set_forced_path(path: int = PATH_AUTO, tile_variant: int = -1) -> int:
    return int(load().hgc_set_forced_path(int(path), int(tile_variant)))


def set_forced_tiling(log2_tile_w: int = -1, split_k: int = -1, log2_tile_n: int = -1) -> None:
    load().hgc_set_forced_tiling(int(log2_tile_w), int(split_k), int(log2_tile_n))


def igemm_variant_name(variant: int, packed: bool = False) -> str:
    buf = ctypes.create_string_buffer(160)
    n = load().hgc_igemm_variant_name(1 if packed else 0, int(variant), buf, 160)
    return buf.value.decode() if n >= 0 else ""


def conv2d_workspace_size(desc) -> int:
    d = ConvDesc.make(desc)
    n = ctypes.c_size_t(0)
    st = load().hgc_conv2d_workspace_size(ctypes.byref(d), ctypes.byref(n))
    if st != 0:
        raise HgcError(st, "hgc_conv2d_workspace_size")
    return int(n.value)


def conv2d_plan(desc, with_workspace: bool = False, packed: bool = False) -> Plan:
    d = ConvDesc.make(desc)
    p = Plan()
    mode = 3 if packed else (1 if with_workspace else 0)
    st = load().hgc_conv2d_plan(ctypes.byref(d), mode, ctypes.byref(p))
    if st != 0:
        raise HgcError(st, "hgc_conv2d_plan")
    return p


def forward_raw(desc: Optional[ConvDesc], x: int, w: int, b: int, y: int, stream: int = 0) -> int:
    """hgc_conv2d_forward on raw addresses; returns the status (no exception)."""
    dref = ctypes.byref(desc) if desc is not None else None
    return int(load().hgc_conv2d_forward(dref, x or None, w or None, b or None, y or None, stream or None))


def forward_ws_raw(desc: Optional[ConvDesc], x: int, w: int, b: int, y: int, ws: int, ws_bytes: int,
                   stream: int = 0) -> int:
    dref = ctypes.byref(desc) if desc is not None else None
    return int(load().hgc_conv2d_forward_ws(dref, x or None, w or None, b or None, y or None,
                                            ws or None, int(ws_bytes), stream or None))


def _check_tensor(t, name, shape=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.float16 or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous float16 CUDA tensor")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")


def _marshal(desc, x, w, b, y):
    import torch
    d = ConvDesc.make(desc)
    cg = d.C // d.group if d.group > 0 and d.C % d.group == 0 else None
    _check_tensor(x, "x", (d.N, d.C, d.H, d.W))
    _check_tensor(w, "w", (d.num_output, cg, d.kernel, d.kernel) if cg else None)
    if d.bias:
        if b is None:
            raise ValueError("bias=1 needs b")
        _check_tensor(b, "b", (d.num_output,))
    if y is None:
        y = torch.empty(d.out_shape(), dtype=torch.float16, device=x.device)
    else:
        _check_tensor(y, "y", d.out_shape())
    stream = torch.cuda.current_stream(x.device).cuda_stream
    return d, y, stream


def conv2d_forward(desc, x, w, b=None, y=None):
    """hgc_conv2d_forward on torch tensors, on torch's current stream. Returns y."""
    d, y, stream = _marshal(desc, x, w, b, y)
    st = forward_raw(d, x.data_ptr(), w.data_ptr(), b.data_ptr() if (d.bias and b is not None) else 0,
                     y.data_ptr(), stream)
    if st != 0:
        raise HgcError(st, "hgc_conv2d_forward")
    return y


def conv2d_forward_ws(desc, x, w, b=None, y=None, workspace=None):
    """hgc_conv2d_forward_ws; `workspace` is a CUDA uint8 tensor (or None when 0 bytes are needed)."""
    d, y, stream = _marshal(desc, x, w, b, y)
    ws_ptr, ws_bytes = 0, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    st = forward_ws_raw(d, x.data_ptr(), w.data_ptr(), b.data_ptr() if (d.bias and b is not None) else 0,
                        y.data_ptr(), ws_ptr, ws_bytes, stream)
    if st != 0:
        raise HgcError(st, "hgc_conv2d_forward_ws")
    return y


def conv2d_packed_weights_size(desc) -> int:
    d = ConvDesc.make(desc)
    n = ctypes.c_size_t(0)
    st = load().hgc_conv2d_packed_weights_size(ctypes.byref(d), ctypes.byref(n))
    if st != 0:
        raise HgcError(st, "hgc_conv2d_packed_weights_size")
    return int(n.value)


def conv2d_pack_weights(desc, w, w_packed=None):
    """hgc_conv2d_pack_weights on torch tensors; returns the packed uint8 CUDA tensor."""
    import torch
    d = ConvDesc.make(desc)
    _check_tensor(w, "w")
    need = conv2d_packed_weights_size(d)
    if w_packed is None:
        w_packed = torch.empty(need, dtype=torch.uint8, device=w.device)
    if w_packed.numel() * w_packed.element_size() < need:
        raise ValueError("w_packed is too small")
    stream = torch.cuda.current_stream(w.device).cuda_stream
    st = int(load().hgc_conv2d_pack_weights(ctypes.byref(d), w.data_ptr(), w_packed.data_ptr(), stream or None))
    if st != 0:
        raise HgcError(st, "hgc_conv2d_pack_weights")
    return w_packed


def forward_packed_raw(desc: Optional[ConvDesc], x: int, wp: int, b: int, y: int, ws: int, ws_bytes: int,
                       stream: int = 0) -> int:
    dref = ctypes.byref(desc) if desc is not None else None
    return int(load().hgc_conv2d_forward_packed(dref, x or None, wp or None, b or None, y or None,
                                                ws or None, int(ws_bytes), stream or None))


def conv2d_forward_packed(desc, x, w_packed, b=None, y=None, workspace=None):
    """hgc_conv2d_forward_packed; w_packed comes from conv2d_pack_weights."""
    import torch
    d = ConvDesc.make(desc)
    _check_tensor(x, "x", (d.N, d.C, d.H, d.W))
    if d.bias:
        if b is None:
            raise ValueError("bias=1 needs b")
        _check_tensor(b, "b", (d.num_output,))
    if y is None:
        y = torch.empty(d.out_shape(), dtype=torch.float16, device=x.device)
    else:
        _check_tensor(y, "y", d.out_shape())
    ws_ptr, ws_bytes = 0, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    stream = torch.cuda.current_stream(x.device).cuda_stream
    st = forward_packed_raw(d, x.data_ptr(), w_packed.data_ptr(), b.data_ptr() if (d.bias and b is not None) else 0,
                            y.data_ptr(), ws_ptr, ws_bytes, stream)
    if st != 0:
        raise HgcError(st, "hgc_conv2d_forward_packed")
    return y


def tune_raw(desc: Optional[ConvDesc], x: int, w: int, b: int, y: int, ws: int, ws_bytes: int, packed: bool,
             stream: int = 0, plan: Optional[Plan] = None) -> int:
    dref = ctypes.byref(desc) if desc is not None else None
    pref = ctypes.byref(plan) if plan is not None else None
    return int(load().hgc_conv2d_tune(dref, x or None, w or None, b or None, y or None, ws or None,
                                      int(ws_bytes), 1 if packed else 0, stream or None, pref))


def conv2d_tune(desc, x, w, b=None, y=None, workspace=None, packed: bool = False) -> Plan:
    """hgc_conv2d_tune; w is the packed buffer when packed.  Returns the shape now in effect."""
    import torch
    d = ConvDesc.make(desc)
    _check_tensor(x, "x", (d.N, d.C, d.H, d.W))
    if d.bias:
        if b is None:
            raise ValueError("bias=1 needs b")
        _check_tensor(b, "b", (d.num_output,))
    if y is None:
        y = torch.empty(d.out_shape(), dtype=torch.float16, device=x.device)
    else:
        _check_tensor(y, "y", d.out_shape())
    ws_ptr, ws_bytes = 0, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    plan = Plan()
    st = tune_raw(d, x.data_ptr(), w.data_ptr(), b.data_ptr() if (d.bias and b is not None) else 0,
                  y.data_ptr(), ws_ptr, ws_bytes, packed, torch.cuda.current_stream(x.device).cuda_stream, plan)
    if st != 0:
        raise HgcError(st, "hgc_conv2d_tune")
    return plan


def conv2d_tune_reset() -> None:
    load().hgc_conv2d_tune_reset()


def conv2d_set_launch_shape(desc, packed: bool, variant: int, log2_tile_w: int, split_k: int,
                            log2_tile_n: int = 0) -> None:
    d = ConvDesc.make(desc)
    st = load().hgc_conv2d_set_launch_shape(ctypes.byref(d), 1 if packed else 0, int(variant), int(log2_tile_w),
                                            int(log2_tile_n), int(split_k))
    if st != 0:
        raise HgcError(st, "hgc_conv2d_set_launch_shape")


def inner_product_forward_raw(desc: Optional[InnerProductDesc], x: int, w: int, b: int, y: int, stream: int = 0) -> int:
    dref = ctypes.byref(desc) if desc is not None else None
    return int(load().hgc_inner_product_forward(dref, x or None, w or None, b or None, y or None, stream or None))


def inner_product_forward(desc, x, w, b=None, y=None):
    """hgc_inner_product_forward: x [N][K] (or any shape with N*K elements), w [M][K], b [M] -> y [N][M]."""
    import torch
    d = InnerProductDesc.make(desc)
    for t, name, count in ((x, "x", d.N * d.K), (w, "w", d.num_output * d.K)):
        _check_tensor(t, name)
        if t.numel() != count:
            raise ValueError(f"{name} has {t.numel()} elements, the descriptor needs {count}")
    if d.bias:
        if b is None:
            raise ValueError("bias=1 needs b")
        _check_tensor(b, "b", (d.num_output,))
    if y is None:
        y = torch.empty((d.N, d.num_output), dtype=torch.float16, device=x.device)
    else:
        _check_tensor(y, "y", (d.N, d.num_output))
    st = inner_product_forward_raw(d, x.data_ptr(), w.data_ptr(), b.data_ptr() if (d.bias and b is not None) else 0,
                                   y.data_ptr(), torch.cuda.current_stream(x.device).cuda_stream)
    if st != 0:
        raise HgcError(st, "hgc_inner_product_forward")
    return y


def batch_norm_workspace_size_raw(desc: Optional[BatchNormDesc]):
    """Returns (status, bytes)."""
    out = ctypes.c_size_t(0)
    dref = ctypes.byref(desc) if desc is not None else None
    st = int(load().hgc_batch_norm_workspace_size(dref, ctypes.byref(out)))
    return st, int(out.value)


def batch_norm_workspace_size(desc, eps: float = 1e-5, stat_scale: float = 1.0) -> int:
    st, n = batch_norm_workspace_size_raw(BatchNormDesc.make(desc, eps, stat_scale))
    if st != 0:
        raise HgcError(st, "hgc_batch_norm_workspace_size")
    return n


def batch_norm_forward_raw(desc: Optional[BatchNormDesc], x: int, mean: int, var: int, gamma: int, beta: int, y: int,
                           workspace: int, workspace_bytes: int, stream: int = 0) -> int:
    dref = ctypes.byref(desc) if desc is not None else None
    return int(load().hgc_batch_norm_forward(dref, x or None, mean or None, var or None, gamma or None, beta or None,
                                             y or None, workspace or None, int(workspace_bytes), stream or None))


def batch_norm_forward(desc, x, eps: float = 1e-5, mean=None, var=None, stat_scale: float = 1.0, gamma=None, beta=None,
                       y=None, workspace=None):
    """hgc_batch_norm_forward: x FP16 [N][C][H][W] -> y (same shape; pass y=x for in place).

    mean, var, gamma, beta: FP32 [C] device tensors.  With use_global_stats = 0, mean and var (if given)
    receive the batch statistics.  Returns y.
    """
    import torch
    d = BatchNormDesc.make(desc, eps, stat_scale)
    shape = (d.N, d.C, d.H, d.W)
    _check_tensor(x, "x", shape)
    if y is None:
        y = torch.empty(shape, dtype=torch.float16, device=x.device)
    else:
        _check_tensor(y, "y", shape)

    def f32(t, name, required):
        if t is None:
            if required:
                raise ValueError(f"{name} is required by the descriptor")
            return 0
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or t.numel() != d.C:
            raise ValueError(f"{name} must be a contiguous float32 device tensor of C elements")
        return t.data_ptr()

    pm, pv = f32(mean, "mean", d.use_global_stats == 1), f32(var, "var", d.use_global_stats == 1)
    pg, pb = f32(gamma, "gamma", d.scale_bias == 1), f32(beta, "beta", d.scale_bias == 1)
    need = batch_norm_workspace_size(d)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    st = batch_norm_forward_raw(d, x.data_ptr(), pm, pv, pg, pb, y.data_ptr(), workspace.data_ptr(),
                                workspace.numel() * workspace.element_size(),
                                torch.cuda.current_stream(x.device).cuda_stream)
    if st != 0:
        raise HgcError(st, "hgc_batch_norm_forward")
    return y


def max_pool_output_size_raw(desc: Optional[MaxPoolDesc]):
    """Returns (status, Ho, Wo)."""
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    dref = ctypes.byref(desc) if desc is not None else None
    st = int(load().hgc_max_pool_output_size(dref, ctypes.byref(ho), ctypes.byref(wo)))
    return st, int(ho.value), int(wo.value)


def max_pool_output_size(desc):
    st, ho, wo = max_pool_output_size_raw(MaxPoolDesc.make(desc))
    if st != 0:
        raise HgcError(st, "hgc_max_pool_output_size")
    return ho, wo


def max_pool_forward_raw(desc: Optional[MaxPoolDesc], x: int, y: int, stream: int = 0) -> int:
    dref = ctypes.byref(desc) if desc is not None else None
    return int(load().hgc_max_pool_forward(dref, x or None, y or None, stream or None))


def max_pool_forward(desc, x, y=None):
    """hgc_max_pool_forward: x FP16 [N][C][H][W] -> y FP16 [N][C][Ho][Wo]."""
    import torch
    d = MaxPoolDesc.make(desc)
    _check_tensor(x, "x", (d.N, d.C, d.H, d.W))
    ho, wo = max_pool_output_size(d)
    if y is None:
        y = torch.empty((d.N, d.C, ho, wo), dtype=torch.float16, device=x.device)
    else:
        _check_tensor(y, "y", (d.N, d.C, ho, wo))
    st = max_pool_forward_raw(d, x.data_ptr(), y.data_ptr(), torch.cuda.current_stream(x.device).cuda_stream)
    if st != 0:
        raise HgcError(st, "hgc_max_pool_forward")
    return y


def batch_norm_fold_raw(conv: Optional[ConvDesc], w: int, b: int, mean: int, var: int, stat_scale: float, eps: float,
                        gamma: int, beta: int, w_out: int, b_out: int, stream: int = 0) -> int:
    dref = ctypes.byref(conv) if conv is not None else None
    return int(load().hgc_batch_norm_fold(dref, w or None, b or None, mean or None, var or None, float(stat_scale),
                                          float(eps), gamma or None, beta or None, w_out or None, b_out or None,
                                          stream or None))


def batch_norm_fold(conv, w, b, mean, var, eps: float = 1e-5, stat_scale: float = 1.0, gamma=None, beta=None):
    """hgc_batch_norm_fold: returns (w_out, b_out), new FP16 device tensors; use them with bias = 1."""
    import torch
    d = ConvDesc.make(conv)
    _check_tensor(w, "w")
    if d.bias:
        _check_tensor(b, "b", (d.num_output,))
    for t, name in ((mean, "mean"), (var, "var"), (gamma, "gamma"), (beta, "beta")):
        if t is not None and (t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or t.numel() != d.num_output):
            raise ValueError(f"{name} must be a contiguous float32 device tensor of num_output elements")
    w_out = torch.empty_like(w)
    b_out = torch.empty(d.num_output, dtype=torch.float16, device=w.device)
    ptr = lambda t: 0 if t is None else t.data_ptr()
    st = batch_norm_fold_raw(d, w.data_ptr(), ptr(b) if d.bias else 0, ptr(mean), ptr(var), stat_scale, eps, ptr(gamma),
                             ptr(beta), w_out.data_ptr(), b_out.data_ptr(), torch.cuda.current_stream(w.device).cuda_stream)
    if st != 0:
        raise HgcError(st, "hgc_batch_norm_fold")
    return w_out, b_out

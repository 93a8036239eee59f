"""FP16 convolution-layer forward for MI355X: thin Python binding of libhgc.

The package holds the HIP sources (csrc/), the build step (build.py) and a
ctypes binding (binding.py) whose functions carry the C ABI's names and only
marshal arguments.  Every step of the computation runs in the HIP kernels;
there is no CPU fallback: loading fails loudly when libhgc.so is missing.
"""
from .binding import (  # noqa: F401
    ConvDesc, Plan, HgcError, PATH_AUTO, PATH_DIRECT, PATH_IGEMM, PATH_IGEMM_SPLITK,
    PATH_DEPTHWISE, PATH_FIRST_LAYER, PATH_POINTWISE, PATH_NAMES, load, library_path, conv2d_forward, conv2d_forward_ws,
    conv2d_workspace_size, conv2d_plan, set_forced_path, set_forced_tiling, status_string, version,
    forward_raw, forward_ws_raw, forward_packed_raw, conv2d_packed_weights_size, conv2d_pack_weights,
    conv2d_forward_packed, igemm_variant_name, conv2d_tune, conv2d_tune_reset, tune_raw, conv2d_set_launch_shape, InnerProductDesc,
    inner_product_forward, inner_product_forward_raw, BatchNormDesc, batch_norm_forward, batch_norm_forward_raw,
    batch_norm_workspace_size, batch_norm_workspace_size_raw, MaxPoolDesc, max_pool_forward, max_pool_forward_raw,
    max_pool_output_size, max_pool_output_size_raw, batch_norm_fold, batch_norm_fold_raw,
)

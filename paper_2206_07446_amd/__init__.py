"""MI355X-native conv hot path of NNV12-style cold inference: per-kernel weight
transformation and convolution execution behind the C ABI of include/nnv.h.

The Python layer only marshals arguments (torch tensors -> device pointers); every
step of the path runs in the HIP library libnnv.so.
"""
from .binding import (  # noqa: F401
    NnvError, ConvDesc, Timing, CacheIo, KINDS, DIRECT, IM2COL_GEMM, WINO_F2, WINO_F4, DEPTHWISE, WINO_F6, F32, F16,
    load, make_desc, nnv_layout_version, nnv_status_string, nnv_last_hip_error, nnv_kind_supported,
    nnv_transformed_bytes, nnv_workspace_bytes, nnv_transform_weights, nnv_transform_weights_grouped,
    nnv_conv_forward, nnv_conv_forward_relu, nnv_conv_forward_static, STATIC_SCRATCH_BYTES, nnv_conv_forward_grouped,
    nnv_conv_forward_grouped_workspace_bytes, FORWARD_RELU, nnv_time_layer, nnv_cold_stack, nnv_cache_write, nnv_cache_read, EXPORTS,
)

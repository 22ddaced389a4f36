"""SqueezeNet forward path for AMD MI355X: Python binding of libsq.so.

The functions here have the names of the C entry points in include/sq.h and do
argument marshalling only (tensor checks, output allocation, pointer passing);
every step of the computation runs in the library's HIP kernels.  PyTorch
supplies device memory and the current stream, nothing else.  There is no CPU
fallback: if the library is missing the import fails.
"""
from .binding import (  # noqa: F401
    SQ_ALGO_AUTO, SQ_ALGO_DIRECT, SQ_ALGO_VARIANT0, SQ_BF16, SQ_F32, SQ_SQUEEZENET_MAX_BATCH, SQ_SQUEEZENET_BF16_MAX_BATCH,
    SqError, lib,
    sq_avgpool_global, sq_conv2d_forward, sq_conv2d_forward_ex, sq_conv2d_forward_ws,
    sq_conv2d_workspace_bytes, sq_conv2d_strided_workspace_bytes, sq_conv2d_bf16_workspace_bytes, sq_conv_variant_count,
    sq_conv_variant_name, sq_fire_forward, sq_fire_workspace_bytes, sq_maxpool, sq_maxpool_conv2d_forward, sq_softmax,
    sq_profile_begin, sq_profile_end, sq_squeezenet_forward, sq_init, sq_set_dtype, sq_fire_packed_bytes, sq_fire_pack_weights,
    sq_fire_forward_packed, sq_classifier_forward, sq_fire_forward_static, SQ_FIRE_STATIC_SCRATCH_BYTES, sq_packed_weights_bytes, sq_pack_weights, sq_squeezenet_forward_packed,
    sq_blocked_map_bytes, sq_blocked_pack, sq_blocked_unpack, sq_blocked_kernel_bytes, sq_blocked_pack_kernels,
    sq_blocked_conv2d_forward, sq_blocked_kernel7_bytes, sq_blocked_pack_kernels7, sq_blocked_conv7s2_forward, sq_blocked_fire_forward, sq_blocked_pool_conv2d_forward,
    sq_blocked_maxpool, sq_blocked_avgpool_global, sq_squeezenet_bf16_packed_bytes,
    sq_squeezenet_bf16_pack_params, sq_squeezenet_bf16_workspace_bytes, sq_squeezenet_forward_bf16, sq_squeezenet_workspace_bytes, sq_strerror, TAP_NAMES, TAP_SHAPES,
    sq_tune_conv2d_forward_poolcols, sq_tune_fire_forward_poolcols, sq_tune_poolrows_conv2d_forward)

"""Dense ops of the TensorFlow.js paper (arxiv 1901.05350) for AMD MI355X (gfx950).

Thin Python binding over libtfx.so (hand-written HIP kernels behind a C ABI, see
include/tfx.h).  The functions here only marshal arguments: PyTorch provides device
memory and the current stream, every step of the computation runs in the HIP kernels.
There is no CPU fallback: if the library is missing or fails to load, calls raise.
"""
from .binding import (  # noqa: F401
    ACT_NONE, ACT_RELU, ACT_RELU6, PAD_SAME, PAD_VALID, TfxError, TfxVariant, MobileNetV1, MobileNetV1F16, lib, library_path,
    tfx_add, tfx_add_f16, tfx_batch_matmul, tfx_batch_matmul_f16, tfx_conv2d, tfx_conv2d_f16, tfx_conv2d_out_shape, tfx_depthwise_conv2d, tfx_depthwise_conv2d_f16,
    tfx_depthwise_conv2d_out_shape, tfx_matmul, tfx_matmul_out_shape, tfx_mobilenet_v1_forward,
    tfx_mobilenet_v1_variant_forward, tfx_mobilenet_v1_variant_workspace_bytes,
    tfx_mobilenet_v1_variant_forward_static, tfx_mobilenet_v1_static_scratch_bytes,
    tfx_mobilenet_v1_variant_features, tfx_mobilenet_v1_variant_features_shape, tfx_mobilenet_v1_features_f16,
    tfx_mobilenet_v1_workspace_bytes, tfx_status_string,
)

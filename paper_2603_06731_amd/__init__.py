"""libpbk for MI355X: Python binding of the C ABI declared in include/pbk.h.

Argument marshalling only: every step of the contraction runs in the HIP
kernels inside libpbk.so.  There is no CPU fallback: importing this package
without a built library raises.
"""
from .binding import (  # noqa: F401
    PBK_OK, PBK_F32, PBK_BF16, PBK_F16, PBK_FP8_E4M3, PBK_FP8_E5M2, PBK_INT8,
    PBK_EPI_NONE, PBK_EPI_BIAS, PBK_EPI_RELU, PBK_EPI_BIAS_RELU,
    PBK_EPI_BIAS_GELU_TANH, PBK_EPI_GELU_TANH,
    PbkError, lib, lib_path, pbk_matmul, pbk_batched_matmul, pbk_conv2d_nhwc, pbk_conv2d_nhwc_pad4,
    pbk_conv2d_transpose_nhwc, pbk_attention, pbk_attention_causal, pbk_matmul_int8, pbk_conv2d_nhwc_int8,
    pbk_matmul_residual, pbk_conv2d_nhwc_residual, pbk_matmul_int8_bn, pbk_conv2d_nhwc_int8_bn,
    pbk_status_string, pbk_version, pbk_last_kernel, pbk_force_kernel, check, EXPORTED_SYMBOLS,
)

"""libbatq: MI355X-native W4A4 MXFP4 linear layer with block-wise affine transforms.

The product is the C-ABI shared library built from ``csrc/`` (see include/batq.h);
this package is its thin ctypes binding.
"""
from .binding import (  # noqa: F401
    BatqError, Transform, Weight, batq_prepare_weight, batq_prepare_weight_minmax, batq_weight_import,
    batq_quantize_act,
    batq_gemm_mxfp4, batq_gemm_workspace, batq_linear, batq_linear_workspace, batq_linear_workspace_for, batq_scale_bytes, batq_scales_to_rowmajor,
    batq_code_bytes, batq_codes_to_rowmajor, batq_codes_from_rowmajor,
    batq_scales_from_rowmajor, batq_code8_bytes, batq_quantize_act_mxfp8, batq_codes8_to_rowmajor,
    batq_codes8_from_rowmajor, batq_gemm_a8w4, batq_linear_a8w4, batq_linear_a8w4_workspace, batq_row_rms_scale, batq_dequantize, batq_transform_apply, batq_kv_append, batq_kv_dequantize, batq_prepare_weight_gate_up, batq_gemm_glu, batq_linear_glu, APPLY_FORWARD, APPLY_INVERSE, APPLY_INVERSE_T,
    batq_quantize_act_ex, batq_linear_ex, lib, LIB_PATH, SYMBOLS, STATUS_NAMES, F32, BF16,
)

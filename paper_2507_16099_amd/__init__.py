"""MI355X-native dynamically scaled float8 linear layer (thin binding over
libfp8mi355.so).  Every step of the path runs in the library's HIP kernels;
this package only marshals arguments.  PyTorch supplies device memory and
streams."""
from .fp8 import (  # noqa: F401
    FP8_E4M3FN, FP8_E5M2, FP8_TENSOR, FP8_ROW, FP8_COL,
    FP8_POW2_SCALE, FP8_TRANSPOSE_OUT, FP8_OUT_FP32, FP8_GRAD_WEIGHT_HP, FP8_SAVE_FOR_BWD, FP8_EPILOGUE_SIGMOID,
    Fp8Error, Recipe, library_path, load_library, set_knob,
    fp8_amax, fp8_scale, fp8_cast, fp8_quantize, fp8_quantize_row_col, fp8_scaled_mm,
    fp8_linear_workspace_bytes, fp8_linear_fwd, fp8_linear_bwd,
    fp8_linear_prequantized_workspace_bytes, fp8_linear_fwd_prequantized, fp8_grad_weight_hp,
    FP8_STATIC_SCRATCH_BYTES, fp8_linear_fwd_prequantized_static,
    fp8_layernorm_quantize, fp8_block_quantize, fp8_block_linear_workspace_bytes, fp8_block_linear_fwd, fp8_block_quantize_t, fp8_block_quantize_row_col, fp8_block_linear_bwd_workspace_bytes, fp8_block_linear_bwd, fp8_linear_bwd_sigmoid_workspace_bytes, fp8_linear_bwd_sigmoid, fp8_mx_quantize, e8m0_plain_rows, fp8_mx_quantize_t, fp8_mx_quantize_row_col, fp8_mx_scaled_mm, fp8_mx_linear_workspace_bytes, fp8_mx_linear_fwd,
    fp8_mx_linear_bwd_workspace_bytes, fp8_mx_linear_bwd,
    fp8_last_error, fp8_version,
)

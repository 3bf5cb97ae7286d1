"""MI355X-native fine-grained W4A8 linear layer with integer group scales (Integer Scale, Eq. (2)).

The product is the C-ABI library built from csrc/ (declared in include/intscale.h); this package is its thin
Python binding.
"""
from .binding import (  # noqa: F401
    EXPORTED_SYMBOLS,
    IS_ALPHA_HEURISTIC,
    IS_ERR_HIP,
    IS_ERR_INVALID_ARG,
    IS_ERR_UNSUPPORTED,
    IS_ERR_WORKSPACE,
    IS_OK,
    IS_SCALE_NORM,
    IS_SCALE_RAW,
    IntScaleError,
    QuantizedWeights,
    is_gemm_grouped_workspace_bytes,
    is_gemm_safe_workspace_bytes,
    is_gemm_w4a8_floatscale,
    is_gemm_w4a8_floatscale_grouped,
    is_gemm_w4a8_intscale,
    is_gemm_w4a8_intscale_grouped,
    is_gemm_w4a8_intscale_safe,
    is_gemm_w8a8_floatscale,
    is_gemm_w8a8_intscale,
    is_gemm_w8a8_workspace_bytes,
    is_gemm_workspace_bytes,
    is_intscale_overflow_bound,
    is_probe_mfma_i8,
    is_probe_stream_read,
    is_quantize_act_int8_token,
    is_quantize_weights_int4_group,
    is_quantize_weights_int8_group,
    last_hip_error,
    library_path,
    load_library,
    status_string,
)

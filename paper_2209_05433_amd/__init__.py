"""MI355X-native scaled-FP8 matrix multiply path (amax -> scale -> cast -> FP8 GEMM ->
unscale) of arXiv 2209.05433, as hand-written HIP kernels behind a C ABI.

The functions re-exported here have the names and argument order of include/fp8mm.h and
only marshal arguments; the library is loaded on first use and its absence is an error.
"""
from .binding import (  # noqa: F401
    FP8_E4M3, FP8_E5M2, FP8_F32, FP8_BF16,
    FP8_OK, FP8_ERR_INVALID_ARG, FP8_ERR_UNSUPPORTED, FP8_ERR_DEVICE,
    EXPORTS, LIB_PATH, Fp8Error, lib,
    fp8_amax, fp8_amax_scale, fp8_amax_scale_multi, fp8_quantize_multi, FP8_MULTI_MAX, FP8_AMAX_WORKSPACE_BYTES, fp8_scale_from_amax_host, fp8_scale_from_amax,
    fp8_quantize, fp8_quantize_dscale, fp8_quantize_ex, fp8_dequantize, FP8_QUANT_NOSAT, fp8_gemm, fp8_gemm_dscale,
    fp8_gemm_mfma8, fp8_gemm_mfma8_dscale, fp8_gemm_ex, fp8_gemm_splitk, fp8_gemm_splitk_workspace_size, fp8_gemm_splitk_static, FP8_SPLITK_STATIC_BYTES, FP8_GEMM_MFMA8, fp8_gemm_fused, fp8_scaled_gemm, fp8_quantize_amax, fp8_quantize_sr, fp8_scale_from_amax_history, fp8_scale_from_amax_n,
    fp8_amax_rows, fp8_quantize_rows, fp8_quantize_transpose,
    FP8_OUT_F32, FP8_OUT_BF16, FP8_OUT_E4M3, FP8_OUT_E5M2, fp8_gemm_plan,
    FP8_PLAN_NO_GEMM, FP8_PLAN_FMA_KERNEL, FP8_PLAN_TILED_256x256, FP8_PLAN_TILED_256x128, FP8_PLAN_MFMA_ANY, FP8_PLAN_TILED_MIXED, FP8_PLAN_ELEMENTWISE_STORES,
    fp8_set_knob, fp8_get_knob, FP8_KNOB_CAST_PATH, FP8_KNOB_TILE_N, FP8_KNOB_GROUP_M, FP8_KNOB_GEMM_KERNEL, FP8_KNOB_SPLIT_K, FP8_KNOB_CAST_RUN, FP8_KNOB_PERSIST, FP8_KNOB_MIXED, FP8_PLAN_PERSISTENT,
    fp8_last_error, fp8_version,
)

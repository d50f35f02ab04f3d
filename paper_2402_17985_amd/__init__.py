"""FlattenQuant per-tensor-quantized linear layer for AMD MI355X (gfx950).

The product is libfq.so (HIP kernels behind the C ABI of include/fq.h); this package is its thin
Python binding.  PyTorch supplies device memory and streams only.
"""
from .binding import (FQ_BF16, FQ_F16, FQ_F32, FQ_I32, FqError, LIB_PATH, SYMBOLS, fq_act_workspace_bytes,
                      fq_bmm_i4, fq_bmm_i8, fq_channel_absmax, fq_flatten_plan, fq_flatten_plan_xw, fq_flatten_quant_act_peel,
                      fq_flatten_weights_split, fq_flatten_quant_act, fq_flatten_quant_act_noalloc, fq_noalloc_scratch_bytes,
                      fq_flatten_weights,
                      fq_gemm_bf16, fq_gemm_i4, fq_gemm_i4_bias, fq_gemm_i4_e3m2, fq_gemm_i8, fq_gemm_i8_bias, fq_gemm_select, fq_linear,
                      fq_linear_bias, fq_linear_fused_a_i8,
                      fq_linear_workspace_bytes, fq_smooth_scales, fq_threshold_boxplot, fq_version,
                      fq_weights_workspace_bytes, fq_peak_mfma, fq_peak_copy, fq_peak_gemm_ticks, fq_peak_wall_clock_khz, lib)
from .layer import FqLinear

__all__ = ["FQ_BF16", "FQ_F16", "FQ_F32", "FQ_I32", "FqError", "FqLinear", "LIB_PATH", "SYMBOLS",
           "fq_act_workspace_bytes", "fq_bmm_i4", "fq_bmm_i8", "fq_channel_absmax", "fq_flatten_plan", "fq_flatten_plan_xw",
           "fq_flatten_quant_act_peel", "fq_flatten_weights_split", "fq_flatten_quant_act",
           "fq_flatten_quant_act_noalloc", "fq_noalloc_scratch_bytes",
           "fq_flatten_weights", "fq_gemm_bf16", "fq_gemm_i4", "fq_gemm_i4_bias", "fq_gemm_i4_e3m2", "fq_gemm_i8", "fq_gemm_i8_bias", "fq_gemm_select", "fq_linear", "fq_linear_bias", "fq_linear_fused_a_i8",
           "fq_linear_workspace_bytes", "fq_smooth_scales", "fq_threshold_boxplot", "fq_version",
           "fq_weights_workspace_bytes", "fq_peak_mfma", "fq_peak_copy", "fq_peak_gemm_ticks", "fq_peak_wall_clock_khz", "lib"]

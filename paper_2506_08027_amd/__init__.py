"""MXFP8 linear-layer hot path for AMD MI355X (gfx950): quantize, block-scaled GEMM, dequantize.

The work is done by hand-written HIP kernels behind a C ABI (``include/mxfp8.h``,
``libmxfp8.so``); this package is the thin binding plus the seeded synthetic input generators.
"""
from .binding import (BF16, BOTH, COLWISE, DGRAD, E4M3, E5M2, F32, FPROP, ROWWISE, SCALE_OCP_V1, SCALE_ROUND_UP,  # noqa: F401
                      SCALES_ROWMAJOR, SCALES_TILED,
                      WGRAD, MXFP8Error, dequantize, gemm, gemm_bf16, gemm_grouped, gemm_quantize, load, mxfp8_gemm_bf16, mxfp8_gemm_grouped_ex, mxfp8_dequantize, mxfp8_dequantize_ex, mxfp8_gemm,
                      mxfp8_dequantize_mode_ex, mxfp8_gemm_ex, mxfp8_gemm_mode_ex, gemm_mode, mxfp8_gemm_quantize_ex, mxfp8_mfma_rate_probe, mxfp8_mfma_rate_probe_ex, mxfp8_mfma_layout_probe, mxfp8_copy_rate_probe, mxfp8_requantize_colwise_ex, requantize_colwise, mxfp8_quantize,
                      mxfp8_quantize_mode_ex, mxfp8_quantize_ex, mxfp8_fp4_quantize_ex, mxfp8_fp4_dequantize_ex, mxfp8_fp4_gemm_ex, E2M3, E3M2, mxfp8_fp6_quantize_ex, mxfp8_fp6_dequantize_ex, mxfp8_fp6_expand_ex, fp6_quantize, fp6_dequantize, fp6_expand, fp6_gemm, fp4_gemm, fp4_quantize, fp4_dequantize, mxfp8_scale_bytes, quantize, status_string)

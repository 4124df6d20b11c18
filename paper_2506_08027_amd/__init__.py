"""MXFP8 linear-layer hot path for AMD MI355X (gfx950): quantize, block-scaled GEMM, dequantize.

The work is done by hand-written HIP kernels behind a C ABI (``include/mxfp8.h``,
``libmxfp8.so``); this package is the thin binding plus the seeded synthetic input generators.
"""
from .binding import (BF16, BOTH, COLWISE, DGRAD, F32, FPROP, ROWWISE, WGRAD, MXFP8Error, dequantize,  # noqa: F401
                      gemm, load, mxfp8_dequantize, mxfp8_gemm, mxfp8_quantize, quantize, status_string)

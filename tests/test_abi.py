"""CPU checks of the C ABI: the shared library loads without a GPU, exports every function that
include/mxfp8.h declares, and its host-side validation rejects bad calls before anything is
launched (so these calls are safe on a machine with no GPU; valid calls are made only in the GPU
tests)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2506_08027_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2506_08027_amd.build import build_library
        build_library()
    return ctypes.CDLL(binding.LIB_PATH)


I64, P = ctypes.c_int64, ctypes.c_void_p
FAKE = P(0x1000)          # 16-byte aligned and never dereferenced: every call made with it fails validation first


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mxfp8.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mxfp8_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    assert declared_functions() == ["mxfp8_copy_rate_probe", "mxfp8_dequantize", "mxfp8_dequantize_ex", "mxfp8_dequantize_mode_ex",
                                    "mxfp8_fp4_dequantize_ex", "mxfp8_fp4_gemm_ex", "mxfp8_fp4_quantize_ex", "mxfp8_fp6_dequantize_ex", "mxfp8_fp6_expand_ex", "mxfp8_fp6_quantize_ex", "mxfp8_gemm", "mxfp8_gemm_bf16", "mxfp8_gemm_ex", "mxfp8_gemm_grouped_ex", "mxfp8_gemm_mode_ex", "mxfp8_gemm_quantize_ex", "mxfp8_mfma_layout_probe", "mxfp8_mfma_rate_probe", "mxfp8_mfma_rate_probe_ex", "mxfp8_quantize",
                                    "mxfp8_quantize_ex", "mxfp8_quantize_mode_ex", "mxfp8_requantize_colwise_ex", "mxfp8_scale_bytes",
                                    "mxfp8_status_string"]


def test_library_exports_every_declared_function(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_mirrors_the_header():
    import paper_2506_08027_amd as mx
    for name in declared_functions():
        if name != "mxfp8_status_string":
            assert callable(getattr(mx, name)), name
    assert callable(mx.status_string)
    assert (mx.ROWWISE, mx.COLWISE, mx.BOTH) == (1, 2, 3)
    assert (mx.FPROP, mx.DGRAD, mx.WGRAD) == (0, 1, 2)
    assert (mx.SCALES_ROWMAJOR, mx.SCALES_TILED) == (0, 1)
    assert (mx.E4M3, mx.E5M2) == (0, 1) and (mx.SCALE_ROUND_UP, mx.SCALE_OCP_V1) == (0, 1)


def test_scale_bytes_is_host_arithmetic(lib):
    f = lib.mxfp8_scale_bytes
    f.restype = ctypes.c_int64
    f.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
    assert f(8192, 4096, 0) == 8192 * 128 and f(8192, 4096, 1) == 8192 * 128
    assert f(100, 96, 0) == 300 and f(100, 96, 1) == 2 * 1 * 256        # 2 groups of 64 rows, 1 group of 4 blocks
    assert f(64, 160, 1) == 1 * 2 * 256 and f(0, 128, 1) == 0
    assert f(64, 100, 1) == -1 and f(-1, 128, 0) == -1 and f(64, 128, 2) == -1


def test_ex_entry_points_validate_the_layout(lib):
    q = lib.mxfp8_quantize_ex
    q.argtypes = [P, ctypes.c_int, I64, I64, I64, ctypes.c_int, P, P, P, P, ctypes.c_int, P]
    assert q(FAKE, 0, 32, 32, 32, 3, FAKE, FAKE, FAKE, FAKE, 2, None) == 5
    assert q(FAKE, 0, 32, 32, 32, 1, FAKE, P(0x1004), None, None, 1, None) == 3     # tiled scales: 16-byte aligned
    assert q(FAKE, 0, 33, 32, 32, 3, FAKE, FAKE, FAKE, FAKE, 1, None) == 2
    g = lib.mxfp8_gemm_ex
    g.argtypes = [ctypes.c_int, P, P, P, P, I64, I64, I64, P, ctypes.c_int, I64, ctypes.c_int, ctypes.c_int32, P]
    assert g(0, FAKE, FAKE, FAKE, FAKE, 64, 64, 128, FAKE, 0, 64, 9, 0, None) == 5
    assert g(0, FAKE, FAKE, FAKE, FAKE, 64, 64, 128, FAKE, 0, 64, 1, -3, None) == 5   # negative workgroup bound
    assert g(0, FAKE, FAKE, FAKE, FAKE, 64, 64, 96, FAKE, 0, 64, 1, 0, None) == 2
    f = lib.mxfp8_gemm_quantize_ex
    f.argtypes = [ctypes.c_int, P, P, P, P, I64, I64, I64, P, I64, ctypes.c_int, P, P, P, P, ctypes.c_int,
                  ctypes.c_int32, P]
    ok = (FAKE, FAKE, FAKE, FAKE)
    outs = (FAKE, FAKE, FAKE, FAKE)
    assert f(0, *ok, 256, 256, 256, FAKE, 256, 3, *outs, 3, 0, None) == 5           # layout
    assert f(0, *ok, 256, 256, 256, FAKE, 256, 0, *outs, 0, 0, None) == 5           # axis
    assert f(0, *ok, 256, 256, 256, FAKE, 256, 3, *outs, 0, -1, None) == 5          # negative workgroup bound
    assert f(0, *ok, 200, 256, 256, FAKE, 256, 3, *outs, 0, 0, None) == 2           # M not a multiple of the tile
    assert f(0, *ok, 256, 256, 128, FAKE, 256, 3, *outs, 0, 0, None) == 2           # fewer than two K steps
    assert f(0, *ok, 256, 256, 256, FAKE, 256, 1, None, FAKE, None, None, 0, 0, None) == 1
    assert f(0, *ok, 256, 256, 256, FAKE, 256, 2, None, None, FAKE, None, 0, 0, None) == 1
    assert f(0, *ok, 256, 256, 256, FAKE, 260, 3, *outs, 0, 0, None) == 3           # ldc * 2 not a multiple of 16
    assert f(0, *ok, 256, 256, 256, FAKE, 256, 1, FAKE, P(0x1004), None, None, 1, 0, None) == 3
    d = lib.mxfp8_dequantize_ex
    d.argtypes = [P, P, I64, I64, P, ctypes.c_int, I64, ctypes.c_int, P]
    assert d(FAKE, FAKE, 4, 64, FAKE, 0, 64, -1, None) == 5
    assert d(FAKE, FAKE, 4, 48, FAKE, 0, 48, 1, None) == 2


def test_mode_entry_points_and_rate_probe_validate(lib):
    q = lib.mxfp8_quantize_mode_ex
    q.argtypes = [P, ctypes.c_int, I64, I64, I64, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, P, P, P, ctypes.c_int, P]
    assert q(FAKE, 0, 32, 32, 32, 3, 2, 0, FAKE, FAKE, FAKE, FAKE, 0, None) == 5   # element format
    assert q(FAKE, 0, 32, 32, 32, 3, 1, 2, FAKE, FAKE, FAKE, FAKE, 0, None) == 5   # scale rule
    assert q(FAKE, 0, 32, 40, 40, 3, 1, 1, FAKE, FAKE, FAKE, FAKE, 0, None) == 2
    assert q(None, 0, 32, 32, 32, 1, 1, 1, FAKE, FAKE, None, None, 0, None) == 1
    d = lib.mxfp8_dequantize_mode_ex
    d.argtypes = [P, P, I64, I64, ctypes.c_int, P, ctypes.c_int, I64, ctypes.c_int, P]
    assert d(FAKE, FAKE, 4, 64, 7, FAKE, 0, 64, 0, None) == 5
    assert d(FAKE, FAKE, 4, 48, 1, FAKE, 0, 48, 0, None) == 2
    cp = lib.mxfp8_copy_rate_probe
    cp.argtypes = [P, P, I64, ctypes.c_int32, ctypes.c_int32, P]
    assert cp(FAKE, FAKE, 1024, 4, 5, None) == 5 and cp(FAKE, FAKE, 1024, 4, 3, None) == 2 and cp(FAKE, FAKE, 1000, 4, 0, None) == 2 and cp(FAKE, FAKE, 1024, 0, 0, None) == 2
    assert cp(None, FAKE, 1024, 4, 0, None) == 1 and cp(P(0x1008), FAKE, 1024, 4, 0, None) == 3 and cp(None, None, 0, 4, 0, None) == 0
    r = lib.mxfp8_mfma_rate_probe
    r.argtypes = [ctypes.c_int32, ctypes.c_int32, P, P]
    assert r(-1, 10, FAKE, None) == 2 and r(10, -1, FAKE, None) == 2 and r((1 << 20) + 1, 1, FAKE, None) == 2
    assert r(4, 10, None, None) == 1 and r(4, 10, P(0x1002), None) == 3 and r(0, 10, None, None) == 0
    rx = lib.mxfp8_mfma_rate_probe_ex
    rx.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, P, P]
    assert rx(4, 10, 6, FAKE, None) == 5 and rx(-1, 10, 4, FAKE, None) == 2 and rx(4, 10, 4, None, None) == 1 and rx(0, 10, 4, None, None) == 0


def test_status_strings(lib):
    lib.mxfp8_status_string.restype = ctypes.c_char_p
    seen = {lib.mxfp8_status_string(i) for i in range(7)}
    assert len(seen) == 7 and all(seen)
    assert lib.mxfp8_status_string(0) == b"ok"
    assert lib.mxfp8_status_string(99)  # never NULL




def test_quantize_validation_needs_no_gpu(lib):
    f = lib.mxfp8_quantize
    f.argtypes = [P, ctypes.c_int, I64, I64, I64, ctypes.c_int, P, P, P, P, P]
    assert f(FAKE, 7, 32, 32, 32, 3, FAKE, FAKE, FAKE, FAKE, None) == 4          # dtype
    assert f(FAKE, 0, 32, 32, 32, 4, FAKE, FAKE, FAKE, FAKE, None) == 5          # axis
    assert f(FAKE, 0, 33, 32, 32, 3, FAKE, FAKE, FAKE, FAKE, None) == 2          # rows % 32
    assert f(FAKE, 0, 32, 64, 32, 3, FAKE, FAKE, FAKE, FAKE, None) == 2          # ld < cols
    assert f(FAKE, 0, -32, 32, 32, 3, FAKE, FAKE, FAKE, FAKE, None) == 2
    assert f(FAKE, 0, 1 << 32, 32, 32, 3, FAKE, FAKE, FAKE, FAKE, None) == 2
    assert f(None, 0, 32, 32, 32, 3, FAKE, FAKE, FAKE, FAKE, None) == 1
    assert f(FAKE, 0, 32, 32, 32, 2, None, None, None, FAKE, None) == 1          # colwise needs q_colT
    assert f(P(0x1004), 0, 32, 32, 32, 1, FAKE, FAKE, None, None, None) == 3     # src alignment
    assert f(FAKE, 1, 32, 32, 36, 1, FAKE, FAKE, None, None, None) == 3          # BF16 ld: 72 bytes
    assert f(FAKE, 0, 0, 32, 32, 3, None, None, None, None, None) == 0           # nothing to do


def test_gemm_validation_needs_no_gpu(lib):
    f = lib.mxfp8_gemm
    f.argtypes = [ctypes.c_int, P, P, P, P, I64, I64, I64, P, ctypes.c_int, I64, P]
    ok = (FAKE, FAKE, FAKE, FAKE)
    assert f(3, *ok, 64, 64, 128, FAKE, 0, 64, None) == 5
    assert f(0, *ok, 64, 64, 128, FAKE, 2, 64, None) == 4
    assert f(0, *ok, 64, 64, 96, FAKE, 0, 64, None) == 2                         # K % 128
    assert f(0, *ok, 64, 64, 128, FAKE, 0, 63, None) == 2                        # ldc < N
    assert f(0, *ok, 64, 64, (1 << 24) + 128, FAKE, 0, 64, None) == 2            # K beyond the 32-bit tile offsets
    assert f(0, *ok, (1 << 30) + 1, 64, 128, FAKE, 0, 64, None) == 2
    assert f(0, *ok, 1 << 30, 1 << 30, 128, FAKE, 0, 1 << 30, None) == 2         # more tiles than a grid holds
    assert f(0, None, FAKE, FAKE, FAKE, 64, 64, 128, FAKE, 0, 64, None) == 1
    assert f(0, *ok, 64, 64, 128, None, 0, 64, None) == 1
    assert f(0, P(0x1008), FAKE, FAKE, FAKE, 64, 64, 128, FAKE, 0, 64, None) == 3
    assert f(0, *ok, 64, 64, 128, P(0x1002), 0, 64, None) == 3                   # FP32 c needs 4-byte alignment
    assert f(0, *ok, 0, 64, 128, None, 0, 64, None) == 0


def test_requantize_validation_needs_no_gpu(lib):
    f = lib.mxfp8_requantize_colwise_ex
    f.argtypes = [P, P, I64, I64, P, P, ctypes.c_int, P]
    assert f(FAKE, FAKE, 64, 64, FAKE, FAKE, 2, None) == 5
    assert f(FAKE, FAKE, 48, 64, FAKE, FAKE, 0, None) == 2 and f(FAKE, FAKE, 64, 48, FAKE, FAKE, 0, None) == 2
    assert f(None, FAKE, 64, 64, FAKE, FAKE, 0, None) == 1 and f(FAKE, FAKE, 64, 64, FAKE, None, 0, None) == 1
    assert f(P(0x1004), FAKE, 64, 64, FAKE, FAKE, 0, None) == 3
    assert f(None, None, 0, 64, None, None, 0, None) == 0


def test_layout_probe_validation_needs_no_gpu(lib):
    f = lib.mxfp8_mfma_layout_probe
    f.argtypes = [P, P, P, P, ctypes.c_int32, ctypes.c_int32, P, P]
    assert f(FAKE, FAKE, FAKE, FAKE, 1, 6, FAKE, None) == 5 and f(FAKE, FAKE, FAKE, FAKE, -1, 8, FAKE, None) == 2
    assert f(FAKE, FAKE, FAKE, FAKE, (1 << 16) + 1, 4, FAKE, None) == 2 and f(FAKE, None, FAKE, FAKE, 1, 4, FAKE, None) == 1
    assert f(P(0x1008), FAKE, FAKE, FAKE, 1, 8, FAKE, None) == 3 and f(FAKE, FAKE, P(0x1002), FAKE, 1, 8, FAKE, None) == 3
    assert f(None, None, None, None, 0, 8, None, None) == 0


def test_fp4_validation_needs_no_gpu(lib):
    f = lib.mxfp8_fp4_quantize_ex
    f.argtypes = [P, ctypes.c_int, I64, I64, I64, ctypes.c_int, P, P, P, P, ctypes.c_int, P]
    assert f(FAKE, 2, 64, 64, 64, 3, FAKE, FAKE, FAKE, FAKE, 0, None) == 4
    assert f(FAKE, 0, 64, 64, 64, 0, FAKE, FAKE, FAKE, FAKE, 0, None) == 5 and f(FAKE, 0, 64, 64, 64, 3, FAKE, FAKE, FAKE, FAKE, 2, None) == 5
    assert f(FAKE, 0, 48, 64, 64, 3, FAKE, FAKE, FAKE, FAKE, 0, None) == 2 and f(FAKE, 0, 64, 64, 32, 3, FAKE, FAKE, FAKE, FAKE, 0, None) == 2
    assert f(FAKE, 0, 64, 64, 64, 1, None, FAKE, None, None, 0, None) == 1 and f(FAKE, 0, 64, 64, 64, 2, None, None, FAKE, None, 0, None) == 1
    assert f(P(0x1004), 0, 64, 64, 64, 1, FAKE, FAKE, None, None, 0, None) == 3 and f(FAKE, 1, 64, 64, 68, 1, FAKE, FAKE, None, None, 0, None) == 3
    assert f(None, 0, 0, 64, 64, 3, None, None, None, None, 0, None) == 0
    g = lib.mxfp8_fp4_dequantize_ex
    g.argtypes = [P, P, I64, I64, P, ctypes.c_int, I64, ctypes.c_int, P]
    assert g(FAKE, FAKE, 64, 64, FAKE, 2, 64, 0, None) == 4 and g(FAKE, FAKE, 64, 64, FAKE, 0, 64, 2, None) == 5
    assert g(FAKE, FAKE, 64, 48, FAKE, 0, 64, 0, None) == 2 and g(FAKE, FAKE, 64, 64, FAKE, 0, 32, 0, None) == 2
    assert g(None, FAKE, 64, 64, FAKE, 0, 64, 0, None) == 1 and g(FAKE, FAKE, 64, 64, P(0x1008), 0, 64, 0, None) == 3
    assert g(None, None, 64, 0, None, 0, 64, 0, None) == 0


def test_gemm_mode_validation_needs_no_gpu(lib):
    f = lib.mxfp8_gemm_mode_ex
    f.argtypes = [ctypes.c_int, P, P, ctypes.c_int, P, P, ctypes.c_int, I64, I64, I64, P, ctypes.c_int, I64, ctypes.c_int, ctypes.c_int32, P]
    assert f(0, FAKE, FAKE, 2, FAKE, FAKE, 0, 64, 64, 128, FAKE, 0, 64, 0, 0, None) == 5 and f(0, FAKE, FAKE, 1, FAKE, FAKE, 3, 64, 64, 128, FAKE, 0, 64, 0, 0, None) == 5
    assert f(0, FAKE, FAKE, 1, FAKE, FAKE, 0, 64, 64, 128, FAKE, 2, 64, 0, 0, None) == 4 and f(0, FAKE, FAKE, 1, FAKE, FAKE, 0, 64, 64, 96, FAKE, 0, 64, 0, 0, None) == 2
    assert f(0, None, FAKE, 1, FAKE, FAKE, 1, 64, 64, 128, FAKE, 0, 64, 0, 0, None) == 1 and f(0, FAKE, FAKE, 1, P(0x1004), FAKE, 1, 64, 64, 128, FAKE, 0, 64, 0, 0, None) == 3
    assert f(0, None, None, 1, None, None, 0, 0, 64, 128, None, 0, 64, 0, 0, None) == 0


def test_fp6_validation_needs_no_gpu(lib):
    f = lib.mxfp8_fp6_quantize_ex
    f.argtypes = [P, ctypes.c_int, I64, I64, I64, ctypes.c_int, ctypes.c_int, P, P, P, P, ctypes.c_int, P]
    assert f(FAKE, 2, 64, 64, 64, 3, 0, FAKE, FAKE, FAKE, FAKE, 0, None) == 4
    assert f(FAKE, 0, 64, 64, 64, 3, 2, FAKE, FAKE, FAKE, FAKE, 0, None) == 5 and f(FAKE, 0, 64, 64, 64, 0, 0, FAKE, FAKE, FAKE, FAKE, 0, None) == 5
    assert f(FAKE, 0, 48, 64, 64, 3, 0, FAKE, FAKE, FAKE, FAKE, 0, None) == 2 and f(FAKE, 0, 64, 64, 32, 3, 1, FAKE, FAKE, FAKE, FAKE, 0, None) == 2
    assert f(FAKE, 0, 64, 64, 64, 1, 1, None, FAKE, None, None, 0, None) == 1 and f(P(0x1004), 0, 64, 64, 64, 1, 0, FAKE, FAKE, None, None, 0, None) == 3
    assert f(None, 0, 0, 64, 64, 3, 0, None, None, None, None, 0, None) == 0
    g = lib.mxfp8_fp6_dequantize_ex
    g.argtypes = [P, P, I64, I64, ctypes.c_int, P, ctypes.c_int, I64, ctypes.c_int, P]
    assert g(FAKE, FAKE, 64, 64, 0, FAKE, 2, 64, 0, None) == 4 and g(FAKE, FAKE, 64, 64, 2, FAKE, 0, 64, 0, None) == 5
    assert g(FAKE, FAKE, 64, 48, 0, FAKE, 0, 64, 0, None) == 2 and g(None, FAKE, 64, 64, 1, FAKE, 0, 64, 0, None) == 1
    assert g(FAKE, FAKE, 64, 64, 1, P(0x1008), 0, 64, 0, None) == 3 and g(None, None, 64, 0, 0, None, 0, 64, 0, None) == 0
    h = lib.mxfp8_fp6_expand_ex
    h.argtypes = [P, I64, I64, ctypes.c_int, P, P]
    assert h(FAKE, 64, 64, 2, FAKE, None) == 5 and h(FAKE, 64, 40, 0, FAKE, None) == 2 and h(FAKE, 64, 64, 0, None, None) == 1
    assert h(P(0x1008), 64, 64, 0, FAKE, None) == 3 and h(None, 0, 64, 1, None, None) == 0


def test_fp4_gemm_validation_needs_no_gpu(lib):
    f = lib.mxfp8_fp4_gemm_ex
    f.argtypes = [ctypes.c_int, P, P, P, P, I64, I64, I64, P, ctypes.c_int, I64, ctypes.c_int, ctypes.c_int32, P]
    ok = (FAKE, FAKE, FAKE, FAKE)
    assert f(0, *ok, 64, 64, 256, FAKE, 2, 64, 0, 0, None) == 4 and f(3, *ok, 64, 64, 256, FAKE, 0, 64, 0, 0, None) == 5
    assert f(0, *ok, 64, 64, 256, FAKE, 0, 64, 2, 0, None) == 5 and f(0, *ok, 64, 64, 256, FAKE, 0, 64, 0, -1, None) == 5
    assert f(0, *ok, 64, 64, 128, FAKE, 0, 64, 0, 0, None) == 2 and f(0, *ok, 64, 64, 256, FAKE, 0, 32, 0, 0, None) == 2
    assert f(0, None, FAKE, FAKE, FAKE, 64, 64, 256, FAKE, 0, 64, 0, 0, None) == 1 and f(0, *ok, 64, 64, 256, None, 0, 64, 0, 0, None) == 1
    assert f(0, P(0x1004), FAKE, FAKE, FAKE, 64, 64, 256, FAKE, 0, 64, 0, 0, None) == 3 and f(0, *ok, 64, 64, 256, P(0x1002), 0, 64, 0, 0, None) == 3
    assert f(0, None, None, None, None, 0, 64, 256, None, 0, 64, 0, 0, None) == 0


def test_grouped_gemm_validation_needs_no_gpu(lib):
    f = lib.mxfp8_gemm_grouped_ex
    f.argtypes = [ctypes.c_int, P, P, P, P, P, ctypes.c_int32, I64, I64, I64, P, ctypes.c_int, I64, ctypes.c_int, ctypes.c_int32, P]
    ok = (FAKE, FAKE, FAKE, FAKE, FAKE)
    assert f(0, *ok, 4, 512, 256, 256, FAKE, 2, 256, 0, 0, None) == 4             # output type
    assert f(3, *ok, 4, 512, 256, 256, FAKE, 0, 256, 0, 0, None) == 5             # no such pass
    assert f(2, *ok, 4, 512, 256, 320, FAKE, 0, 256, 0, 0, None) == 2             # weight-gradient form: K % 128
    assert f(2, *ok, 4, 512, 256, 256, P(0x1002), 0, 256, 0, 0, None) == 3        # ... c aligned to its element
    assert f(2, FAKE, FAKE, FAKE, FAKE, None, 4, 512, 256, 256, FAKE, 0, 256, 0, 0, None) == 1
    assert f(2, *ok, 4, 1 << 30, 1 << 30, 256, FAKE, 0, 1 << 30, 0, 0, None) == 2 # more workgroups than a grid holds
    assert f(0, *ok, 4, 512, 256, 256, FAKE, 0, 256, 2, 0, None) == 5             # scale layout
    assert f(0, *ok, 4, 512, 256, 256, FAKE, 0, 256, 0, -1, None) == 5
    assert f(0, *ok, 4, 512, 192, 256, FAKE, 0, 192, 0, 0, None) == 2             # N % 128
    assert f(0, *ok, 4, 512, 256, 128, FAKE, 0, 256, 0, 0, None) == 2             # K < 256
    assert f(0, *ok, 4, 512, 256, 320, FAKE, 0, 256, 0, 0, None) == 2             # K % 128
    assert f(0, *ok, 4097, 512, 256, 256, FAKE, 0, 256, 0, 0, None) == 2          # too many groups
    assert f(0, *ok, -1, 512, 256, 256, FAKE, 0, 256, 0, 0, None) == 2
    assert f(0, *ok, 4, 512, 256, 256, FAKE, 0, 255, 0, 0, None) == 2             # ldc < N
    assert f(0, FAKE, FAKE, FAKE, FAKE, None, 4, 512, 256, 256, FAKE, 0, 256, 0, 0, None) == 1
    assert f(0, *ok, 4, 512, 256, 256, None, 0, 256, 0, 0, None) == 1
    assert f(0, *ok, 4, 512, 256, 256, P(0x1008), 0, 256, 0, 0, None) == 3        # c must take 128-bit stores
    assert f(0, *ok, 4, 512, 256, 256, FAKE, 1, 260, 0, 0, None) == 3             # BF16 rows of 520 bytes
    assert f(0, FAKE, FAKE, FAKE, FAKE, P(0x1002), 4, 512, 256, 256, FAKE, 0, 256, 0, 0, None) == 3
    assert f(0, *ok, 0, 512, 256, 256, FAKE, 0, 256, 0, 0, None) == 0             # no groups: nothing to do
    assert f(0, *ok, 4, 0, 256, 256, None, 0, 256, 0, 0, None) == 0


def test_bf16_gemm_validation_needs_no_gpu(lib):
    f = lib.mxfp8_gemm_bf16
    f.argtypes = [P, P, I64, I64, I64, P, ctypes.c_int, I64, ctypes.c_int32, P]
    assert f(FAKE, FAKE, 64, 64, 64, FAKE, 2, 64, 0, None) == 4                  # output type
    assert f(FAKE, FAKE, 64, 64, 64, FAKE, 0, 64, -1, None) == 5                 # negative workgroup bound
    assert f(FAKE, FAKE, 64, 64, 96, FAKE, 0, 64, 0, None) == 2                  # K % 64
    assert f(FAKE, FAKE, 64, 64, 64, FAKE, 0, 63, 0, None) == 2                  # ldc < N
    assert f(FAKE, FAKE, 64, 64, (1 << 23) + 64, FAKE, 0, 64, 0, None) == 2      # row bytes beyond the 32-bit tile offsets
    assert f(None, FAKE, 64, 64, 64, FAKE, 0, 64, 0, None) == 1
    assert f(FAKE, FAKE, 64, 64, 64, None, 0, 64, 0, None) == 1
    assert f(P(0x1008), FAKE, 64, 64, 64, FAKE, 0, 64, 0, None) == 3
    assert f(FAKE, FAKE, 64, 64, 64, P(0x1002), 0, 64, 0, None) == 3
    assert f(FAKE, FAKE, 0, 64, 64, None, 0, 64, 0, None) == 0


def test_dequantize_validation_needs_no_gpu(lib):
    f = lib.mxfp8_dequantize
    f.argtypes = [P, P, I64, I64, P, ctypes.c_int, I64, P]
    assert f(FAKE, FAKE, 4, 48, FAKE, 0, 48, None) == 2
    assert f(FAKE, FAKE, 4, 64, FAKE, 0, 32, None) == 2
    assert f(FAKE, FAKE, 4, 64, FAKE, 5, 64, None) == 4
    assert f(None, FAKE, 4, 64, FAKE, 0, 64, None) == 1
    assert f(FAKE, FAKE, 4, 64, P(0x1008), 0, 64, None) == 3
    assert f(FAKE, FAKE, 4, 64, FAKE, 1, 68, None) == 3                          # BF16 ld: 136 bytes
    assert f(FAKE, FAKE, 0, 64, None, 0, 64, None) == 0

"""Thin ctypes binding of ``libmxfp8.so``: same names as the C ABI, argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the path (amax, scale,
element conversion, transposed column copy, block-scaled GEMM, decode) runs in the HIP kernels
behind the C entry points. There is no fallback: if the library is missing or an entry point
reports an error, a Python exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmxfp8.so")

OK = 0
F32, BF16 = 0, 1
ROWWISE, COLWISE, BOTH = 1, 2, 3
FPROP, DGRAD, WGRAD = 0, 1, 2
SCALES_ROWMAJOR, SCALES_TILED = 0, 1
E4M3, E5M2 = 0, 1
SCALE_ROUND_UP, SCALE_OCP_V1 = 0, 1
K_BLOCK = 32

_AXIS = {"rowwise": ROWWISE, "colwise": COLWISE, "both": BOTH, ROWWISE: ROWWISE, COLWISE: COLWISE, BOTH: BOTH}
_PASS = {"fprop": FPROP, "dgrad": DGRAD, "wgrad": WGRAD, FPROP: FPROP, DGRAD: DGRAD, WGRAD: WGRAD}

_lib = None


class MXFP8Error(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what} failed with status {code}: {status_string(code)}")
        self.code = code


def load() -> ctypes.CDLL:
    """Load the in-tree HIP library; fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2506_08027_amd.build` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.mxfp8_quantize.restype = ci
    lib.mxfp8_quantize.argtypes = [vp, ci, i64, i64, i64, ci, vp, vp, vp, vp, vp]
    lib.mxfp8_gemm.restype = ci
    lib.mxfp8_gemm.argtypes = [ci, vp, vp, vp, vp, i64, i64, i64, vp, ci, i64, vp]
    lib.mxfp8_dequantize.restype = ci
    lib.mxfp8_dequantize.argtypes = [vp, vp, i64, i64, vp, ci, i64, vp]
    lib.mxfp8_quantize_ex.restype = ci
    lib.mxfp8_quantize_ex.argtypes = [vp, ci, i64, i64, i64, ci, vp, vp, vp, vp, ci, vp]
    lib.mxfp8_gemm_ex.restype = ci
    lib.mxfp8_gemm_ex.argtypes = [ci, vp, vp, vp, vp, i64, i64, i64, vp, ci, i64, ci, ctypes.c_int32, vp]
    lib.mxfp8_gemm_quantize_ex.restype = ci
    lib.mxfp8_gemm_quantize_ex.argtypes = [ci, vp, vp, vp, vp, i64, i64, i64, vp, i64, ci, vp, vp, vp, vp, ci,
                                           ctypes.c_int32, vp]
    lib.mxfp8_dequantize_ex.restype = ci
    lib.mxfp8_dequantize_ex.argtypes = [vp, vp, i64, i64, vp, ci, i64, ci, vp]
    lib.mxfp8_scale_bytes.restype = i64
    lib.mxfp8_scale_bytes.argtypes = [i64, i64, ci]
    lib.mxfp8_quantize_mode_ex.restype = ci
    lib.mxfp8_quantize_mode_ex.argtypes = [vp, ci, i64, i64, i64, ci, ci, ci, vp, vp, vp, vp, ci, vp]
    lib.mxfp8_dequantize_mode_ex.restype = ci
    lib.mxfp8_dequantize_mode_ex.argtypes = [vp, vp, i64, i64, ci, vp, ci, i64, ci, vp]
    lib.mxfp8_requantize_colwise_ex.restype = ci
    lib.mxfp8_requantize_colwise_ex.argtypes = [vp, vp, i64, i64, vp, vp, ci, vp]
    lib.mxfp8_gemm_grouped_ex.restype = ci
    lib.mxfp8_gemm_grouped_ex.argtypes = [ci, vp, vp, vp, vp, vp, ctypes.c_int32, i64, i64, i64, vp, ci, i64, ci, ctypes.c_int32, vp]
    lib.mxfp8_gemm_bf16.restype = ci
    lib.mxfp8_gemm_bf16.argtypes = [vp, vp, i64, i64, i64, vp, ci, i64, ctypes.c_int32, vp]
    lib.mxfp8_mfma_rate_probe.restype = ci
    lib.mxfp8_fp4_quantize_ex.argtypes = [vp, ci, i64, i64, i64, ci, vp, vp, vp, vp, ci, vp]
    lib.mxfp8_fp4_quantize_ex.restype = ci
    lib.mxfp8_fp4_dequantize_ex.argtypes = [vp, vp, i64, i64, vp, ci, i64, ci, vp]
    lib.mxfp8_fp4_dequantize_ex.restype = ci
    lib.mxfp8_fp4_gemm_ex.argtypes = [ci, vp, vp, vp, vp, i64, i64, i64, vp, ci, i64, ci, ctypes.c_int32, vp]
    lib.mxfp8_fp4_gemm_ex.restype = ci
    lib.mxfp8_fp6_quantize_ex.argtypes = [vp, ci, i64, i64, i64, ci, ci, vp, vp, vp, vp, ci, vp]
    lib.mxfp8_fp6_quantize_ex.restype = ci
    lib.mxfp8_fp6_dequantize_ex.argtypes = [vp, vp, i64, i64, ci, vp, ci, i64, ci, vp]
    lib.mxfp8_fp6_dequantize_ex.restype = ci
    lib.mxfp8_fp6_expand_ex.argtypes = [vp, i64, i64, ci, vp, vp]
    lib.mxfp8_fp6_expand_ex.restype = ci
    lib.mxfp8_gemm_mode_ex.argtypes = [ci, vp, vp, ci, vp, vp, ci, i64, i64, i64, vp, ci, i64, ci, ctypes.c_int32, vp]
    lib.mxfp8_gemm_mode_ex.restype = ci
    lib.mxfp8_mfma_rate_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.mxfp8_copy_rate_probe.restype = ci
    lib.mxfp8_mfma_rate_probe_ex.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.mxfp8_mfma_rate_probe_ex.restype = ci
    lib.mxfp8_mfma_layout_probe.argtypes = [vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.mxfp8_mfma_layout_probe.restype = ci
    lib.mxfp8_copy_rate_probe.argtypes = [vp, vp, i64, ctypes.c_int32, ctypes.c_int32, vp]
    lib.mxfp8_status_string.restype = ctypes.c_char_p
    lib.mxfp8_status_string.argtypes = [ci]
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load().mxfp8_status_string(int(code)).decode()


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    raise TypeError(f"only float32 and bfloat16 are supported, got {t}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _need_cuda(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("all tensors must live in GPU memory")


# ---- raw entry points: same names and argument order as include/mxfp8.h -----------------------

def mxfp8_scale_bytes(rows: int, cols: int, scale_layout: int = SCALES_ROWMAJOR) -> int:
    """Bytes of the scale buffer of a [rows x cols] operand (host arithmetic in the library)."""
    n = load().mxfp8_scale_bytes(rows, cols, scale_layout)
    if n < 0:
        raise ValueError("bad shape or layout")
    return n


def _check_scales(s, rows, cols, scale_layout, what):
    if s.dtype != torch.uint8 or not s.is_contiguous():
        raise ValueError(f"{what} must be dense uint8")
    if scale_layout == SCALES_ROWMAJOR:
        if tuple(s.shape) != (rows, cols // K_BLOCK):
            raise ValueError(f"{what} must be [{rows} x {cols // K_BLOCK}]")
    elif scale_layout == SCALES_TILED and s.numel() < mxfp8_scale_bytes(rows, cols, scale_layout):
        raise ValueError(f"{what} holds {s.numel()} bytes, the tiled layout needs "
                         f"{mxfp8_scale_bytes(rows, cols, scale_layout)}")


def mxfp8_quantize(src, axis, q_row=None, s_row=None, q_colT=None, s_colT=None, stream=None) -> None:
    """src [rows x cols] float32/bfloat16 (row stride = leading dimension) -> the selected copies."""
    mxfp8_quantize_ex(src, axis, q_row, s_row, q_colT, s_colT, SCALES_ROWMAJOR, stream)


def mxfp8_quantize_ex(src, axis, q_row=None, s_row=None, q_colT=None, s_colT=None,
                      scale_layout=SCALES_ROWMAJOR, stream=None) -> None:
    """mxfp8_quantize with the scale bytes stored in `scale_layout` (tiled buffers: flat uint8 of
    mxfp8_scale_bytes(rows, cols) / mxfp8_scale_bytes(cols, rows) bytes)."""
    mxfp8_quantize_mode_ex(src, axis, E4M3, SCALE_ROUND_UP, q_row, s_row, q_colT, s_colT, scale_layout, stream)


def mxfp8_quantize_mode_ex(src, axis, element=E4M3, rule=SCALE_ROUND_UP, q_row=None, s_row=None, q_colT=None,
                           s_colT=None, scale_layout=SCALES_ROWMAJOR, stream=None) -> None:
    """mxfp8_quantize_ex with the element format (E4M3 / E5M2) and the scale rule (SCALE_ROUND_UP /
    SCALE_OCP_V1) of the paper's ablations."""
    _need_cuda(src, q_row, s_row, q_colT, s_colT)
    if src.dim() != 2 or (src.numel() and src.stride(1) != 1):
        raise ValueError("src must be 2-D with contiguous rows")
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else max(cols, 1)
    if scale_layout == SCALES_TILED:      # the library cannot see buffer sizes: check them here
        if s_row is not None and _AXIS[axis] & ROWWISE:
            _check_scales(s_row, rows, cols, scale_layout, "s_row")
        if s_colT is not None and _AXIS[axis] & COLWISE:
            _check_scales(s_colT, cols, rows, scale_layout, "s_colT")
    rc = load().mxfp8_quantize_mode_ex(_ptr(src), _dtype_code(src.dtype), rows, cols, ld, _AXIS[axis], element, rule,
                                       _ptr(q_row), _ptr(s_row), _ptr(q_colT), _ptr(s_colT), scale_layout,
                                       _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_quantize")


def mxfp8_gemm(pass_, a_q, a_s, b_q, b_s, c, stream=None) -> None:
    """c [M x N] (float32/bfloat16) = A [M x K] . B [N x K]^T with block scales [. x K/32]."""
    mxfp8_gemm_ex(pass_, a_q, a_s, b_q, b_s, c, SCALES_ROWMAJOR, 0, stream)


def mxfp8_gemm_ex(pass_, a_q, a_s, b_q, b_s, c, scale_layout=SCALES_ROWMAJOR, max_workgroups=0, stream=None) -> None:
    """mxfp8_gemm with both scale operands stored in `scale_layout`, on at most `max_workgroups` compute
    units (0 = all)."""
    _need_cuda(a_q, a_s, b_q, b_s, c)
    M, K = a_q.shape
    N, Kb = b_q.shape
    if K != Kb:
        raise ValueError("operand shapes disagree")
    _check_scales(a_s, M, K, scale_layout, "a_s")
    _check_scales(b_s, N, K, scale_layout, "b_s")
    if tuple(c.shape) != (M, N) or (c.numel() and c.stride(1) != 1):
        raise ValueError("c must be [M x N] with contiguous rows")
    for t in (a_q, a_s, b_q, b_s):
        if not t.is_contiguous() or t.dtype != torch.uint8:
            raise ValueError("quantized operands must be dense uint8")
    ldc = c.stride(0) if M > 1 else max(N, 1)
    rc = load().mxfp8_gemm_ex(_PASS[pass_], _ptr(a_q), _ptr(a_s), _ptr(b_q), _ptr(b_s), M, N, K, _ptr(c),
                              _dtype_code(c.dtype), ldc, scale_layout, max_workgroups, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_gemm")


def mxfp8_gemm_mode_ex(pass_, a_q, a_s, a_element, b_q, b_s, b_element, c, scale_layout=SCALES_ROWMAJOR, max_workgroups=0,
                       stream=None) -> None:
    """mxfp8_gemm_ex with the element format (E4M3 / E5M2) of each operand chosen by the caller."""
    _need_cuda(a_q, a_s, b_q, b_s, c)
    M, K = a_q.shape
    N, Kb = b_q.shape
    if K != Kb:
        raise ValueError("operand shapes disagree")
    _check_scales(a_s, M, K, scale_layout, "a_s")
    _check_scales(b_s, N, K, scale_layout, "b_s")
    if tuple(c.shape) != (M, N) or (c.numel() and c.stride(1) != 1):
        raise ValueError("c must be [M x N] with contiguous rows")
    for t in (a_q, a_s, b_q, b_s):
        if not t.is_contiguous() or t.dtype != torch.uint8:
            raise ValueError("quantized operands must be dense uint8")
    ldc = c.stride(0) if M > 1 else max(N, 1)
    rc = load().mxfp8_gemm_mode_ex(_PASS[pass_], _ptr(a_q), _ptr(a_s), a_element, _ptr(b_q), _ptr(b_s), b_element, M, N, K,
                                   _ptr(c), _dtype_code(c.dtype), ldc, scale_layout, max_workgroups, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_gemm_mode_ex")


def mxfp8_requantize_colwise_ex(q_row, s_row, q_colT, s_colT, scale_layout=SCALES_ROWMAJOR, stream=None) -> None:
    """Column copy (q_colT [cols x rows], s_colT) derived from the row copy (q_row [rows x cols], s_row) of a tensor."""
    _need_cuda(q_row, s_row, q_colT, s_colT)
    rows, cols = q_row.shape
    _check_scales(s_row, rows, cols, scale_layout, "s_row")
    _check_scales(s_colT, cols, rows, scale_layout, "s_colT")
    if tuple(q_colT.shape) != (cols, rows):
        raise ValueError("q_colT must be [cols x rows]")
    for t in (q_row, s_row, q_colT, s_colT):
        if not t.is_contiguous() or t.dtype != torch.uint8:
            raise ValueError("quantized tensors must be dense uint8")
    rc = load().mxfp8_requantize_colwise_ex(_ptr(q_row), _ptr(s_row), rows, cols, _ptr(q_colT), _ptr(s_colT), scale_layout,
                                            _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_requantize_colwise_ex")


def mxfp8_gemm_grouped_ex(pass_, a_q, a_s, b_q, b_s, group_ends, c, scale_layout=SCALES_ROWMAJOR, max_workgroups=0,
                          stream=None) -> None:
    """Grouped products over expert-sorted tokens; group_ends = int32 GPU tensor of E non-decreasing token numbers.
    fprop / dgrad: a_q [M x K] (tokens are rows), b_q [E x N x K] and b_s (E scale operands, each in `scale_layout`),
    c [M x N]. wgrad: a_q [M x K], b_q [N x K] (tokens are the K axis of both), c [E x M x N]."""
    _need_cuda(a_q, a_s, b_q, b_s, group_ends, c)
    wgrad = _PASS[pass_] == WGRAD
    M, K = a_q.shape
    E = group_ends.numel()
    if group_ends.dtype != torch.int32 or not group_ends.is_contiguous():
        raise ValueError("group_ends must be contiguous int32")
    _check_scales(a_s, M, K, scale_layout, "a_s")
    if wgrad:
        N, Kb = b_q.shape
        _check_scales(b_s, N, K, scale_layout, "b_s")
        if tuple(c.shape) != (E, M, N) or (c.numel() and (c.stride(2) != 1 or c.stride(0) != M * c.stride(1))):
            raise ValueError("c must be [E x M x N] with contiguous rows and experts M rows apart")
        ldc = c.stride(1) if M > 1 else max(N, 1)
    else:
        Eb, N, Kb = b_q.shape
        if Eb != E or b_s.numel() != E * mxfp8_scale_bytes(N, K, scale_layout):
            raise ValueError("b_q must be [E x N x K] with one scale operand per group in b_s")
        if tuple(c.shape) != (M, N) or (c.numel() and c.stride(1) != 1):
            raise ValueError("c must be [M x N] with contiguous rows")
        ldc = c.stride(0) if M > 1 else max(N, 1)
    if K != Kb:
        raise ValueError("operands disagree on K")
    for t in (a_q, a_s, b_q, b_s):
        if not t.is_contiguous() or t.dtype != torch.uint8:
            raise ValueError("quantized operands must be dense uint8")
    rc = load().mxfp8_gemm_grouped_ex(_PASS[pass_], _ptr(a_q), _ptr(a_s), _ptr(b_q), _ptr(b_s), _ptr(group_ends), E, M, N, K,
                                      _ptr(c), _dtype_code(c.dtype), ldc, scale_layout, max_workgroups, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_gemm_grouped_ex")


def mxfp8_gemm_bf16(a, b, c, max_workgroups=0, stream=None) -> None:
    """c [M x N] (float32 or bfloat16) = a [M x K] * b[N x K]^T for dense bfloat16 operands: the GEMM of the
    simulated MX path."""
    _need_cuda(a, b, c)
    M, K = a.shape
    N, Kb = b.shape
    if K != Kb or a.dtype != torch.bfloat16 or b.dtype != torch.bfloat16 or not a.is_contiguous() or not b.is_contiguous():
        raise ValueError("operands must be dense bfloat16 and agree in K")
    if tuple(c.shape) != (M, N) or (c.numel() and c.stride(1) != 1):
        raise ValueError("c must be [M x N] with contiguous rows")
    ldc = c.stride(0) if M > 1 else max(N, 1)
    rc = load().mxfp8_gemm_bf16(_ptr(a), _ptr(b), M, N, K, _ptr(c), _dtype_code(c.dtype), ldc, max_workgroups,
                                _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_gemm_bf16")


def mxfp8_gemm_quantize_ex(pass_, a_q, a_s, b_q, b_s, c, axis, cq_row=None, cs_row=None, cq_colT=None, cs_colT=None,
                           scale_layout=SCALES_ROWMAJOR, max_workgroups=0, stream=None) -> None:
    """mxfp8_gemm_ex with bfloat16 c [M x N] plus the MXFP8 copies of c selected by `axis`:
    cq_row [M x N] / cs_row and cq_colT [N x M] / cs_colT."""
    _need_cuda(a_q, a_s, b_q, b_s, c, cq_row, cs_row, cq_colT, cs_colT)
    M, K = a_q.shape
    N, Kb = b_q.shape
    if K != Kb or c.dtype != torch.bfloat16 or tuple(c.shape) != (M, N) or (c.numel() and c.stride(1) != 1):
        raise ValueError("c must be bfloat16 [M x N] with contiguous rows, operands must agree in K")
    _check_scales(a_s, M, K, scale_layout, "a_s")
    _check_scales(b_s, N, K, scale_layout, "b_s")
    ax = _AXIS[axis]
    for want, q, s, rows, cols, what in ((ax & ROWWISE, cq_row, cs_row, M, N, "row"), (ax & COLWISE, cq_colT, cs_colT, N, M, "colT")):
        if want and q is not None and s is not None:
            if tuple(q.shape) != (rows, cols) or not q.is_contiguous() or q.dtype != torch.uint8:
                raise ValueError(f"cq_{what} must be dense uint8 [{rows} x {cols}]")
            _check_scales(s, rows, cols, scale_layout, f"cs_{what}")
    for t in (a_q, b_q):
        if not t.is_contiguous() or t.dtype != torch.uint8:
            raise ValueError("element tensors must be dense uint8")
    ldc = c.stride(0) if M > 1 else max(N, 1)
    rc = load().mxfp8_gemm_quantize_ex(_PASS[pass_], _ptr(a_q), _ptr(a_s), _ptr(b_q), _ptr(b_s), M, N, K, _ptr(c), ldc,
                                       ax, _ptr(cq_row), _ptr(cs_row), _ptr(cq_colT), _ptr(cs_colT), scale_layout,
                                       max_workgroups, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_gemm_quantize_ex")


def mxfp8_dequantize(q, s, dst, stream=None) -> None:
    """dst [rows x cols] (float32/bfloat16) = E4M3(q) * 2^(s - 127), blocks along a row."""
    mxfp8_dequantize_ex(q, s, dst, SCALES_ROWMAJOR, stream)


def mxfp8_dequantize_ex(q, s, dst, scale_layout=SCALES_ROWMAJOR, stream=None, element=E4M3) -> None:
    """mxfp8_dequantize with s stored in `scale_layout` and the element bytes in `element` format."""
    _need_cuda(q, s, dst)
    rows, cols = q.shape
    if tuple(dst.shape) != (rows, cols):
        raise ValueError("shapes disagree")
    _check_scales(s, rows, cols, scale_layout, "s")
    if not q.is_contiguous() or q.dtype != torch.uint8:
        raise ValueError("q must be dense uint8")
    if dst.numel() and dst.stride(1) != 1:
        raise ValueError("dst rows must be contiguous")
    ld = dst.stride(0) if rows > 1 else max(cols, 1)
    rc = load().mxfp8_dequantize_mode_ex(_ptr(q), _ptr(s), rows, cols, element, _ptr(dst), _dtype_code(dst.dtype), ld,
                                         scale_layout, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_dequantize")


def mxfp8_mfma_rate_probe(workgroups: int, iterations: int, sink, stream=None) -> float:
    """Enqueue the register-only matrix-instruction loop; returns the flop it performs (time it yourself)."""
    _need_cuda(sink)
    if sink.dtype != torch.float32 or sink.numel() < workgroups * 256 or not sink.is_contiguous():
        raise ValueError("sink must be a dense float32 tensor of workgroups * 256 elements")
    rc = load().mxfp8_mfma_rate_probe(workgroups, iterations, _ptr(sink), _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_mfma_rate_probe")
    return workgroups * 4.0 * iterations * 64 * 65536


def mxfp8_mfma_rate_probe_ex(workgroups: int, iterations: int, element_bits: int, sink, stream=None) -> float:
    """mxfp8_mfma_rate_probe on 8-bit (E4M3) or 4-bit (E2M1) operands; returns the flop it performs."""
    _need_cuda(sink)
    if sink.dtype != torch.float32 or sink.numel() < workgroups * 256 or not sink.is_contiguous():
        raise ValueError("sink must be a dense float32 tensor of workgroups * 256 elements")
    rc = load().mxfp8_mfma_rate_probe_ex(workgroups, iterations, element_bits, _ptr(sink), _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_mfma_rate_probe_ex")
    return workgroups * 4.0 * iterations * 64 * 65536


def mxfp8_mfma_layout_probe(a_regs, b_regs, a_scale_regs, b_scale_regs, element_bits, out, stream=None) -> None:
    """One scaled 16x16x128 matrix instruction per experiment: a_regs / b_regs int32 [X x 64 x 8], scale registers
    int32 [X x 64], out float32 [X x 64 x 4]."""
    _need_cuda(a_regs, b_regs, a_scale_regs, b_scale_regs, out)
    X = a_regs.shape[0]
    for t, shape, dt in ((a_regs, (X, 64, 8), torch.int32), (b_regs, (X, 64, 8), torch.int32), (a_scale_regs, (X, 64), torch.int32),
                         (b_scale_regs, (X, 64), torch.int32), (out, (X, 64, 4), torch.float32)):
        if tuple(t.shape) != shape or t.dtype != dt or not t.is_contiguous():
            raise ValueError("operand registers int32 [X x 64 x 8], scale registers int32 [X x 64], out float32 [X x 64 x 4], dense")
    rc = load().mxfp8_mfma_layout_probe(_ptr(a_regs), _ptr(b_regs), _ptr(a_scale_regs), _ptr(b_scale_regs), X, element_bits,
                                        _ptr(out), _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_mfma_layout_probe")


def mxfp8_copy_rate_probe(src, dst, workgroups, mode=0, stream=None) -> int:
    """Copies src to dst (dense GPU tensors of the same size in bytes) with the library's plain copy kernel;
    returns the bytes moved (read + written)."""
    _need_cuda(src, dst)
    nbytes = src.numel() * src.element_size()
    if not src.is_contiguous() or not dst.is_contiguous() or dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst must be dense and of the same size")
    rc = load().mxfp8_copy_rate_probe(_ptr(src), _ptr(dst), nbytes, workgroups, mode, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_copy_rate_probe")
    return 2 * nbytes


def mxfp8_dequantize_mode_ex(q, s, element, dst, scale_layout=SCALES_ROWMAJOR, stream=None) -> None:
    """mxfp8_dequantize_ex for element bytes in `element` format (E4M3 / E5M2)."""
    mxfp8_dequantize_ex(q, s, dst, scale_layout, stream, element)


def mxfp8_fp4_quantize_ex(src, axis, q_row=None, s_row=None, q_colT=None, s_colT=None,
                          scale_layout=SCALES_ROWMAJOR, stream=None) -> None:
    """src [rows x cols] float32/bfloat16 -> MXFP4 copies: q_row [rows x cols/2], q_colT [cols x rows/2] (two E2M1
    codes per byte), scales as for MXFP8."""
    _need_cuda(src, q_row, s_row, q_colT, s_colT)
    if src.dim() != 2 or (src.numel() and src.stride(1) != 1):
        raise ValueError("src must be 2-D with contiguous rows")
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else max(cols, 1)
    ax = _AXIS[axis]
    for want, q, s, r, c, what in ((ax & ROWWISE, q_row, s_row, rows, cols, "row"), (ax & COLWISE, q_colT, s_colT, cols, rows, "colT")):
        if want and q is not None and s is not None:   # the library cannot see buffer sizes: check them here
            if q.dtype != torch.uint8 or not q.is_contiguous() or q.numel() != r * c // 2:
                raise ValueError(f"q_{what} must be dense uint8 with {r * c // 2} bytes")
            _check_scales(s, r, c, scale_layout, f"s_{what}")
    rc = load().mxfp8_fp4_quantize_ex(_ptr(src), _dtype_code(src.dtype), rows, cols, ld, ax, _ptr(q_row), _ptr(s_row),
                                      _ptr(q_colT), _ptr(s_colT), scale_layout, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_fp4_quantize_ex")


def mxfp8_fp4_dequantize_ex(q, s, dst, scale_layout=SCALES_ROWMAJOR, stream=None) -> None:
    """q [rows x cols/2] packed E2M1 codes, s its scales -> dst [rows x cols] float32/bfloat16."""
    _need_cuda(q, s, dst)
    rows, cols = dst.shape
    if q.dtype != torch.uint8 or not q.is_contiguous() or tuple(q.shape) != (rows, cols // 2):
        raise ValueError(f"q must be dense uint8 [{rows} x {cols // 2}]")
    _check_scales(s, rows, cols, scale_layout, "s")
    if dst.numel() and dst.stride(1) != 1:
        raise ValueError("dst rows must be contiguous")
    ld = dst.stride(0) if rows > 1 else max(cols, 1)
    rc = load().mxfp8_fp4_dequantize_ex(_ptr(q), _ptr(s), rows, cols, _ptr(dst), _dtype_code(dst.dtype), ld, scale_layout,
                                        _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_fp4_dequantize_ex")


def mxfp8_fp4_gemm_ex(pass_, a_q, a_s, b_q, b_s, c, scale_layout=SCALES_ROWMAJOR, max_workgroups=0, stream=None) -> None:
    """c [M x N] (float32/bfloat16) = A . B^T for MXFP4 operands a_q [M x K/2], b_q [N x K/2] (packed E2M1 codes) with
    block scales [. x K/32] in `scale_layout`."""
    _need_cuda(a_q, a_s, b_q, b_s, c)
    M, Kh = a_q.shape
    N, Kb = b_q.shape
    if Kh != Kb:
        raise ValueError("operand shapes disagree")
    K = 2 * Kh
    _check_scales(a_s, M, K, scale_layout, "a_s")
    _check_scales(b_s, N, K, scale_layout, "b_s")
    if tuple(c.shape) != (M, N) or (c.numel() and c.stride(1) != 1):
        raise ValueError("c must be [M x N] with contiguous rows")
    for t in (a_q, a_s, b_q, b_s):
        if not t.is_contiguous() or t.dtype != torch.uint8:
            raise ValueError("quantized operands must be dense uint8")
    ldc = c.stride(0) if M > 1 else max(N, 1)
    rc = load().mxfp8_fp4_gemm_ex(_PASS[pass_], _ptr(a_q), _ptr(a_s), _ptr(b_q), _ptr(b_s), M, N, K, _ptr(c),
                                  _dtype_code(c.dtype), ldc, scale_layout, max_workgroups, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_fp4_gemm_ex")


E2M3, E3M2 = 0, 1   # mxfp8_fp6_element


def mxfp8_fp6_quantize_ex(src, axis, element, q_row=None, s_row=None, q_colT=None, s_colT=None,
                          scale_layout=SCALES_ROWMAJOR, stream=None) -> None:
    """src [rows x cols] float32/bfloat16 -> MXFP6 copies: q_row [rows x cols*3/4], q_colT [cols x rows*3/4] (32 six-bit
    codes per 24 bytes), scales as for MXFP8. element: E2M3 or E3M2."""
    _need_cuda(src, q_row, s_row, q_colT, s_colT)
    if src.dim() != 2 or (src.numel() and src.stride(1) != 1):
        raise ValueError("src must be 2-D with contiguous rows")
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else max(cols, 1)
    ax = _AXIS[axis]
    for want, q, s, r, c, what in ((ax & ROWWISE, q_row, s_row, rows, cols, "row"), (ax & COLWISE, q_colT, s_colT, cols, rows, "colT")):
        if want and q is not None and s is not None:   # the library cannot see buffer sizes: check them here
            if q.dtype != torch.uint8 or not q.is_contiguous() or q.numel() != r * c // 4 * 3:
                raise ValueError(f"q_{what} must be dense uint8 with {r * c // 4 * 3} bytes")
            _check_scales(s, r, c, scale_layout, f"s_{what}")
    rc = load().mxfp8_fp6_quantize_ex(_ptr(src), _dtype_code(src.dtype), rows, cols, ld, ax, element, _ptr(q_row), _ptr(s_row),
                                      _ptr(q_colT), _ptr(s_colT), scale_layout, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_fp6_quantize_ex")


def mxfp8_fp6_dequantize_ex(q, s, element, dst, scale_layout=SCALES_ROWMAJOR, stream=None) -> None:
    """q [rows x cols*3/4] packed 6-bit codes, s its scales -> dst [rows x cols] float32/bfloat16."""
    _need_cuda(q, s, dst)
    rows, cols = dst.shape
    if q.dtype != torch.uint8 or not q.is_contiguous() or tuple(q.shape) != (rows, cols // 4 * 3):
        raise ValueError(f"q must be dense uint8 [{rows} x {cols // 4 * 3}]")
    _check_scales(s, rows, cols, scale_layout, "s")
    if dst.numel() and dst.stride(1) != 1:
        raise ValueError("dst rows must be contiguous")
    ld = dst.stride(0) if rows > 1 else max(cols, 1)
    rc = load().mxfp8_fp6_dequantize_ex(_ptr(q), _ptr(s), rows, cols, element, _ptr(dst), _dtype_code(dst.dtype), ld,
                                        scale_layout, _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_fp6_dequantize_ex")


def mxfp8_fp6_expand_ex(q, element, q_e4m3, stream=None) -> None:
    """q [rows x cols*3/4] packed 6-bit codes -> q_e4m3 [rows x cols] E4M3 bytes of the same values."""
    _need_cuda(q, q_e4m3)
    rows, cols = q_e4m3.shape
    for t, shape in ((q, (rows, cols // 4 * 3)), (q_e4m3, (rows, cols))):
        if t.dtype != torch.uint8 or not t.is_contiguous() or tuple(t.shape) != shape:
            raise ValueError("q must be dense uint8 [rows x cols*3/4], q_e4m3 dense uint8 [rows x cols]")
    rc = load().mxfp8_fp6_expand_ex(_ptr(q), rows, cols, element, _ptr(q_e4m3), _stream(stream))
    if rc != OK:
        raise MXFP8Error(rc, "mxfp8_fp6_expand_ex")


# ---- conveniences that only allocate the outputs ----------------------------------------------

def quantize(src, axis="both", scale_layout=SCALES_ROWMAJOR, element=E4M3, rule=SCALE_ROUND_UP):
    """Allocate outputs and call mxfp8_quantize_ex. Returns a dict with the selected copies:
    'q_row' [R x C], 's_row' [R x C/32], 'q_colT' [C x R], 's_colT' [C x R/32] (uint8); with
    tiled scales 's_row' and 's_colT' are flat buffers of mxfp8_scale_bytes bytes."""
    rows, cols = src.shape
    ax = _AXIS[axis]
    out = {}
    u8 = dict(dtype=torch.uint8, device=src.device)
    tiled = scale_layout != SCALES_ROWMAJOR
    if ax & ROWWISE:
        out["q_row"] = torch.empty((rows, cols), **u8)
        out["s_row"] = torch.empty((mxfp8_scale_bytes(rows, cols, scale_layout),) if tiled
                                   else (rows, cols // K_BLOCK), **u8)
    if ax & COLWISE:
        out["q_colT"] = torch.empty((cols, rows), **u8)
        out["s_colT"] = torch.empty((mxfp8_scale_bytes(cols, rows, scale_layout),) if tiled
                                    else (cols, rows // K_BLOCK), **u8)
    mxfp8_quantize_mode_ex(src, ax, element, rule, out.get("q_row"), out.get("s_row"), out.get("q_colT"),
                           out.get("s_colT"), scale_layout)
    return out


def gemm(pass_, a_q, a_s, b_q, b_s, out_dtype=torch.float32, scale_layout=SCALES_ROWMAJOR, max_workgroups=0):
    c = torch.empty((a_q.shape[0], b_q.shape[0]), dtype=out_dtype, device=a_q.device)
    mxfp8_gemm_ex(pass_, a_q, a_s, b_q, b_s, c, scale_layout, max_workgroups)
    return c


def requantize_colwise(q_row, s_row, scale_layout=SCALES_ROWMAJOR):
    """Allocate and return {'q_colT', 's_colT'} derived from a row copy (see mxfp8_requantize_colwise_ex)."""
    rows, cols = q_row.shape
    u8 = dict(dtype=torch.uint8, device=q_row.device)
    tiled = scale_layout != SCALES_ROWMAJOR
    out = {"q_colT": torch.empty((cols, rows), **u8),
           "s_colT": torch.empty((mxfp8_scale_bytes(cols, rows, scale_layout),) if tiled else (cols, rows // K_BLOCK), **u8)}
    mxfp8_requantize_colwise_ex(q_row, s_row, out["q_colT"], out["s_colT"], scale_layout)
    return out


def gemm_grouped(pass_, a_q, a_s, b_q, b_s, group_ends, out_dtype=torch.float32, scale_layout=SCALES_ROWMAJOR, max_workgroups=0):
    """Allocates the output of mxfp8_gemm_grouped_ex and calls it: c [M x N] for fprop / dgrad (filled with NaN
    first: rows that belong to no group are not written), c [E x M x N] for wgrad."""
    if _PASS[pass_] == WGRAD:
        c = torch.empty((group_ends.numel(), a_q.shape[0], b_q.shape[0]), dtype=out_dtype, device=a_q.device)
    else:
        c = torch.full((a_q.shape[0], b_q.shape[1]), float("nan"), dtype=out_dtype, device=a_q.device)
    mxfp8_gemm_grouped_ex(pass_, a_q, a_s, b_q, b_s, group_ends, c, scale_layout, max_workgroups)
    return c


def gemm_bf16(a, b, out_dtype=torch.float32, max_workgroups=0):
    c = torch.empty((a.shape[0], b.shape[0]), dtype=out_dtype, device=a.device)
    mxfp8_gemm_bf16(a, b, c, max_workgroups)
    return c


def gemm_quantize(pass_, a_q, a_s, b_q, b_s, axis="both", scale_layout=SCALES_ROWMAJOR, max_workgroups=0):
    """Allocate the outputs of mxfp8_gemm_quantize_ex and return them as a dict: 'c' (bfloat16 [M x N]) and,
    as selected by `axis`, 'q_row', 's_row', 'q_colT', 's_colT' of c (same conventions as quantize)."""
    M, N = a_q.shape[0], b_q.shape[0]
    ax = _AXIS[axis]
    u8 = dict(dtype=torch.uint8, device=a_q.device)
    tiled = scale_layout != SCALES_ROWMAJOR
    out = {"c": torch.empty((M, N), dtype=torch.bfloat16, device=a_q.device)}
    if ax & ROWWISE:
        out["q_row"] = torch.empty((M, N), **u8)
        out["s_row"] = torch.empty((mxfp8_scale_bytes(M, N, scale_layout),) if tiled else (M, N // K_BLOCK), **u8)
    if ax & COLWISE:
        out["q_colT"] = torch.empty((N, M), **u8)
        out["s_colT"] = torch.empty((mxfp8_scale_bytes(N, M, scale_layout),) if tiled else (N, M // K_BLOCK), **u8)
    mxfp8_gemm_quantize_ex(pass_, a_q, a_s, b_q, b_s, out["c"], ax, out.get("q_row"), out.get("s_row"),
                           out.get("q_colT"), out.get("s_colT"), scale_layout, max_workgroups)
    return out


def dequantize(q, s, out_dtype=torch.float32, scale_layout=SCALES_ROWMAJOR, element=E4M3):
    dst = torch.empty(tuple(q.shape), dtype=out_dtype, device=q.device)
    mxfp8_dequantize_ex(q, s, dst, scale_layout, element=element)
    return dst


def fp4_quantize(src, axis="both", scale_layout=SCALES_ROWMAJOR):
    """Allocate outputs and call mxfp8_fp4_quantize_ex; keys as for quantize(), element buffers half as wide."""
    rows, cols = src.shape
    ax = _AXIS[axis]
    out = {}
    u8 = dict(dtype=torch.uint8, device=src.device)
    tiled = scale_layout != SCALES_ROWMAJOR
    if ax & ROWWISE:
        out["q_row"] = torch.empty((rows, cols // 2), **u8)
        out["s_row"] = torch.empty((mxfp8_scale_bytes(rows, cols, scale_layout),) if tiled else (rows, cols // K_BLOCK), **u8)
    if ax & COLWISE:
        out["q_colT"] = torch.empty((cols, rows // 2), **u8)
        out["s_colT"] = torch.empty((mxfp8_scale_bytes(cols, rows, scale_layout),) if tiled else (cols, rows // K_BLOCK), **u8)
    mxfp8_fp4_quantize_ex(src, ax, out.get("q_row"), out.get("s_row"), out.get("q_colT"), out.get("s_colT"), scale_layout)
    return out


def fp4_dequantize(q, s, out_dtype=torch.float32, scale_layout=SCALES_ROWMAJOR):
    dst = torch.empty((q.shape[0], q.shape[1] * 2), dtype=out_dtype, device=q.device)
    mxfp8_fp4_dequantize_ex(q, s, dst, scale_layout)
    return dst


def fp4_gemm(pass_, a_q, a_s, b_q, b_s, out_dtype=torch.float32, scale_layout=SCALES_ROWMAJOR, max_workgroups=0):
    c = torch.empty((a_q.shape[0], b_q.shape[0]), dtype=out_dtype, device=a_q.device)
    mxfp8_fp4_gemm_ex(pass_, a_q, a_s, b_q, b_s, c, scale_layout, max_workgroups)
    return c


def fp6_quantize(src, element, axis="both", scale_layout=SCALES_ROWMAJOR):
    """Allocate outputs and call mxfp8_fp6_quantize_ex; keys as for quantize(), element buffers 3/4 as wide."""
    rows, cols = src.shape
    ax = _AXIS[axis]
    out = {}
    u8 = dict(dtype=torch.uint8, device=src.device)
    tiled = scale_layout != SCALES_ROWMAJOR
    if ax & ROWWISE:
        out["q_row"] = torch.empty((rows, cols // 4 * 3), **u8)
        out["s_row"] = torch.empty((mxfp8_scale_bytes(rows, cols, scale_layout),) if tiled else (rows, cols // K_BLOCK), **u8)
    if ax & COLWISE:
        out["q_colT"] = torch.empty((cols, rows // 4 * 3), **u8)
        out["s_colT"] = torch.empty((mxfp8_scale_bytes(cols, rows, scale_layout),) if tiled else (cols, rows // K_BLOCK), **u8)
    mxfp8_fp6_quantize_ex(src, ax, element, out.get("q_row"), out.get("s_row"), out.get("q_colT"), out.get("s_colT"), scale_layout)
    return out


def fp6_dequantize(q, s, element, out_dtype=torch.float32, scale_layout=SCALES_ROWMAJOR):
    dst = torch.empty((q.shape[0], q.shape[1] // 3 * 4), dtype=out_dtype, device=q.device)
    mxfp8_fp6_dequantize_ex(q, s, element, dst, scale_layout)
    return dst


def fp6_expand(q, element):
    q8 = torch.empty((q.shape[0], q.shape[1] // 3 * 4), dtype=torch.uint8, device=q.device)
    mxfp8_fp6_expand_ex(q, element, q8)
    return q8


def fp6_gemm(pass_, a_q, a_s, a_element, b_q, b_s, b_element, out_dtype=torch.float32, scale_layout=SCALES_ROWMAJOR, max_workgroups=0):
    """Product of two MXFP6 operands: both expanded to E4M3 bytes, then the MXFP8 product with the operands' own scales."""
    return gemm(pass_, fp6_expand(a_q, a_element), a_s, fp6_expand(b_q, b_element), b_s, out_dtype, scale_layout, max_workgroups)


def gemm_mode(pass_, a_q, a_s, a_element, b_q, b_s, b_element, out_dtype=torch.float32, scale_layout=SCALES_ROWMAJOR, max_workgroups=0):
    c = torch.empty((a_q.shape[0], b_q.shape[0]), dtype=out_dtype, device=a_q.device)
    mxfp8_gemm_mode_ex(pass_, a_q, a_s, a_element, b_q, b_s, b_element, c, scale_layout, max_workgroups)
    return c

"""CPU oracle for the MXFP8 linear-layer path: numpy front end of ``mxfp8_oracle.c``.

TEST INFRASTRUCTURE ONLY. The tests, the smoke check and the benchmark's ``cpu_baseline`` leg call
this; the HIP library and its Python binding never do, and nothing here touches the GPU.

All arithmetic lives in the C file (the paper's definitions, Section 2, Section 3.3, Algorithm 1,
Appendix A.1-A.3, written out in double precision). This module only compiles it with gcc, loads
it with ctypes and moves numpy arrays in and out. BF16 tensors travel as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mxfp8_oracle.c")
_LIB = os.path.join(_HERE, "libmxfp8_oracle.so")

K_BLOCK = 32


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over rows/columns only). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    u8p = ctypes.POINTER(ctypes.c_uint8)
    i64 = ctypes.c_int64
    vp = ctypes.c_void_p
    lib.mxo_threads.restype = ctypes.c_int
    lib.mxo_e4m3_decode.restype = ctypes.c_double
    lib.mxo_e4m3_decode.argtypes = [ctypes.c_uint8]
    lib.mxo_e4m3_encode.restype = ctypes.c_uint8
    lib.mxo_e4m3_encode.argtypes = [ctypes.c_double]
    lib.mxo_scale_byte.restype = ctypes.c_int
    lib.mxo_scale_byte.argtypes = [ctypes.c_double]
    lib.mxo_round_to_bf16.restype = ctypes.c_uint16
    lib.mxo_round_to_bf16.argtypes = [ctypes.c_double]
    for name in ("mxo_quantize_rowwise_f32", "mxo_quantize_colwise_f32",
                 "mxo_quantize_rowwise_bf16", "mxo_quantize_colwise_bf16"):
        fn = getattr(lib, name)
        fn.restype = None
        fn.argtypes = [vp, i64, i64, i64, u8p, u8p]
    lib.mxo_dequantize_f64.restype = None
    lib.mxo_dequantize_f64.argtypes = [u8p, u8p, i64, i64, vp]
    lib.mxo_dequantize_f32.restype = None
    lib.mxo_dequantize_f32.argtypes = [u8p, u8p, i64, i64, vp, i64]
    lib.mxo_dequantize_bf16.restype = None
    lib.mxo_dequantize_bf16.argtypes = [u8p, u8p, i64, i64, vp, i64]
    lib.mxo_e5m2_decode.restype = ctypes.c_double
    lib.mxo_e5m2_decode.argtypes = [ctypes.c_uint8]
    lib.mxo_e5m2_encode.restype = ctypes.c_uint8
    lib.mxo_e5m2_encode.argtypes = [ctypes.c_double]
    lib.mxo_scale_byte_mode.restype = ctypes.c_int
    lib.mxo_scale_byte_mode.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_int]
    lib.mxo_quantize_rowwise_mode_f32.restype = None
    lib.mxo_quantize_rowwise_mode_f32.argtypes = [vp, i64, i64, i64, u8p, u8p, ctypes.c_int, ctypes.c_int]
    lib.mxo_dequantize_mode_f64.restype = None
    lib.mxo_dequantize_mode_f64.argtypes = [u8p, u8p, i64, i64, vp, ctypes.c_int]
    lib.mxo_matmul_nt_bf16_rows.restype = None
    lib.mxo_matmul_nt_bf16_rows.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, vp]
    lib.mxo_gemm_rows_f64.restype = ctypes.c_int
    lib.mxo_gemm_rows_f64.argtypes = [u8p, u8p, u8p, u8p, i64, i64, i64, vp, i64, vp, vp]
    _lib = lib
    return lib


def _u8(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def threads() -> int:
    """Number of host threads the C loops use (OpenMP default: all cores given to the process)."""
    return int(_load().mxo_threads())


def e4m3_decode(code: int) -> float:
    return float(_load().mxo_e4m3_decode(int(code) & 0xFF))


def e4m3_encode(t: float) -> int:
    return int(_load().mxo_e4m3_encode(float(t)))


def scale_byte(amax: float) -> int:
    return int(_load().mxo_scale_byte(float(amax)))


def round_to_bf16_bits(x: float) -> int:
    return int(_load().mxo_round_to_bf16(float(x)))


def _check_src(src: np.ndarray):
    if src.ndim != 2:
        raise ValueError("source must be 2-D")
    if src.dtype == np.float32:
        kind = "f32"
    elif src.dtype == np.uint16:
        kind = "bf16"
    else:
        raise TypeError("source must be float32 or uint16 (BF16 bit patterns)")
    if src.strides[1] != src.itemsize or src.strides[0] % src.itemsize:
        raise ValueError("source rows must be contiguous")
    return kind, src.strides[0] // src.itemsize


def quantize_rowwise(src: np.ndarray):
    """[rows x cols] -> (q [rows x cols] u8, s [rows x cols/32] u8); blocks run along a row."""
    kind, ld = _check_src(src)
    rows, cols = src.shape
    if cols % K_BLOCK:
        raise ValueError("cols must be a multiple of 32")
    q = np.empty((rows, cols), np.uint8)
    s = np.empty((rows, cols // K_BLOCK), np.uint8)
    getattr(_load(), "mxo_quantize_rowwise_" + kind)(src.ctypes.data, rows, cols, ld, _u8(q), _u8(s))
    return q, s


def quantize_colwise(src: np.ndarray):
    """[rows x cols] -> (qT [cols x rows] u8, sT [cols x rows/32] u8); blocks run down a column."""
    kind, ld = _check_src(src)
    rows, cols = src.shape
    if rows % K_BLOCK:
        raise ValueError("rows must be a multiple of 32")
    qT = np.empty((cols, rows), np.uint8)
    sT = np.empty((cols, rows // K_BLOCK), np.uint8)
    getattr(_load(), "mxo_quantize_colwise_" + kind)(src.ctypes.data, rows, cols, ld, _u8(qT), _u8(sT))
    return qT, sT


def _check_qs(q: np.ndarray, s: np.ndarray):
    q = np.ascontiguousarray(q, np.uint8)
    s = np.ascontiguousarray(s, np.uint8)
    if q.ndim != 2 or q.shape[1] % K_BLOCK or s.shape != (q.shape[0], q.shape[1] // K_BLOCK):
        raise ValueError("q must be [rows x cols], s [rows x cols/32]")
    return q, s


def dequantize(q: np.ndarray, s: np.ndarray, dtype: str = "f64") -> np.ndarray:
    """Decoded values Q * 2^(S-127); 'f64' exact, 'f32'/'bf16' rounded once (bf16 as uint16)."""
    q, s = _check_qs(q, s)
    rows, cols = q.shape
    lib = _load()
    if dtype == "f64":
        out = np.empty((rows, cols), np.float64)
        lib.mxo_dequantize_f64(_u8(q), _u8(s), rows, cols, out.ctypes.data)
    elif dtype == "f32":
        out = np.empty((rows, cols), np.float32)
        lib.mxo_dequantize_f32(_u8(q), _u8(s), rows, cols, out.ctypes.data, cols)
    elif dtype == "bf16":
        out = np.empty((rows, cols), np.uint16)
        lib.mxo_dequantize_bf16(_u8(q), _u8(s), rows, cols, out.ctypes.data, cols)
    else:
        raise ValueError(dtype)
    return out


def gemm_rows(a_q, a_s, b_q, b_s, rows):
    """Rows ``rows`` of C = A * B^T over decoded operands in double: returns (C, sum|a*b|)."""
    a_q, a_s = _check_qs(a_q, a_s)
    b_q, b_s = _check_qs(b_q, b_s)
    M, K = a_q.shape
    N, Kb = b_q.shape
    if K != Kb:
        raise ValueError("operands disagree on K")
    idx = np.ascontiguousarray(rows, np.int64)
    if idx.size and (idx.min() < 0 or idx.max() >= M):
        raise ValueError("row index out of range")
    C = np.empty((idx.size, N), np.float64)
    A = np.empty((idx.size, N), np.float64)
    rc = _load().mxo_gemm_rows_f64(_u8(a_q), _u8(a_s), _u8(b_q), _u8(b_s), M, N, K,
                                   idx.ctypes.data, idx.size, C.ctypes.data, A.ctypes.data)
    if rc != 0:
        raise MemoryError("oracle GEMM could not allocate its decoded operands")
    return C, A


def gemm(a_q, a_s, b_q, b_s):
    """All of C = A * B^T (see gemm_rows)."""
    return gemm_rows(a_q, a_s, b_q, b_s, np.arange(np.asarray(a_q).shape[0]))


# ---- single-copy storage (Section 5): the column copy derived from the row copy -----------------------------
def requantize_colwise(q_row: np.ndarray, s_row: np.ndarray):
    """Column copy of a tensor of which only the MXFP8 row copy (q_row [rows x cols], s_row) was kept: every
    element is decoded exactly (Q_i * X, in double, then FP32 without rounding) and the decoded tensor is
    quantized down its columns like any FP32 source (FP32 being the widest source format of Section 3.3, a
    decoded magnitude beyond it counts as +-Inf, as it would in such a source). Returns (qT [cols x rows], sT [cols x rows/32])."""
    v = dequantize(q_row, s_row, "f64")
    with np.errstate(over="ignore"):
        v32 = v.astype(np.float32)  # exact, except that magnitudes beyond FP32 (scale bytes >= 247 only) become +-Inf
    ok = np.isfinite(v32)
    if not np.array_equal(v32[ok].astype(np.float64), v[ok]):
        raise ValueError("a decoded value is not an FP32 number")   # cannot happen: 4 significant bits, >= 2^-136
    return quantize_colwise(v32)


# ---- grouped product (Appendix A.4: mixture-of-experts layers) ------------------------------------------
def grouped_gemm(a_q, a_s, b_q, b_s, group_ends):
    """Expert-batched tokens: the rows of A are sorted by expert, rows [group_ends[e-1], group_ends[e]) belong to
    expert e, and every expert has its own B: b_q [E x N x K], b_s [E x N x K/32]. Row m of expert e gives
    C[m, :] = A[m, :] . B_e^T, the same block-scaled dot products as gemm(). Returns (C, sum|a*b|), [M x N].
    Rows at or beyond group_ends[-1] belong to no expert and come back as NaN."""
    a_q, a_s = _check_qs(a_q, a_s)
    b_q, b_s = np.ascontiguousarray(b_q), np.ascontiguousarray(b_s)
    ends = [int(e) for e in group_ends]
    if b_q.ndim != 3 or b_q.shape[0] != len(ends) or b_s.shape[:2] != b_q.shape[:2]:
        raise ValueError("one B operand per group expected")
    M = a_q.shape[0]
    C = np.full((M, b_q.shape[1]), np.nan)
    A = np.full((M, b_q.shape[1]), np.nan)
    start = 0
    for e, end in enumerate(ends):
        if not start <= end <= M:
            raise ValueError("group ends must be non-decreasing and at most M")
        if end > start:
            C[start:end], A[start:end] = gemm_rows(a_q, a_s, b_q[e], b_s[e], np.arange(start, end))
        start = end
    return C, A


def grouped_gemm_wgrad(a_q, a_s, b_q, b_s, group_ends):
    """The weight-gradient product of the same layer: A = dY_colT [M x T], B = X_colT [N x T], tokens (the
    reduction axis) sorted by expert; expert e owns columns [group_ends[e-1], group_ends[e]) of both operands,
    which must be whole 32-token blocks. Returns (C, sum|a*b|), each [E x M x N]: one dW per expert (zeros for an
    expert without tokens)."""
    a_q, a_s = _check_qs(a_q, a_s)
    b_q, b_s = _check_qs(b_q, b_s)
    ends = [int(e) for e in group_ends]
    M, N = a_q.shape[0], b_q.shape[0]
    C = np.zeros((len(ends), M, N))
    A = np.zeros((len(ends), M, N))
    start = 0
    for e, end in enumerate(ends):
        if not start <= end <= a_q.shape[1] or start % K_BLOCK or end % K_BLOCK:
            raise ValueError("group ends must be non-decreasing multiples of 32 and at most K")
        if end > start:
            sl, bl = slice(start, end), slice(start // K_BLOCK, end // K_BLOCK)
            C[e], A[e] = gemm(a_q[:, sl], a_s[:, bl], b_q[:, sl], b_s[:, bl])
        start = end
    return C, A


# ---- simulated MX path (Section 3.1): BF16 -> MXFP8 -> BF16 round trip, then a BF16 product -----------
def roundtrip_bf16(src: np.ndarray, axis: str = "row") -> np.ndarray:
    """BF16 source (uint16 bit patterns, [rows x cols]) converted to MXFP8 along `axis` and straight back
    to BF16 (round to nearest even of Q_i * X): what the paper's simulated runs feed to the GEMM.
    'row': blocks along a row, result [rows x cols]; 'col': blocks down a column, result stored
    transposed [cols x rows] like the column copy itself."""
    src = np.ascontiguousarray(src)
    if src.dtype != np.uint16:
        raise TypeError("BF16 bit patterns (uint16) expected")
    q, s = quantize_rowwise(src) if axis == "row" else quantize_colwise(src)
    return dequantize(q, s, "bf16")


def matmul_nt_bf16_rows(a: np.ndarray, b: np.ndarray, rows):
    """Rows ``rows`` of C = A * B^T for BF16 operands given as uint16 bit patterns ([M x K], [N x K]),
    in double: returns (C, sum|a*b|)."""
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    if a.dtype != np.uint16 or b.dtype != np.uint16 or a.ndim != 2 or b.ndim != 2:
        raise TypeError("two 2-D arrays of BF16 bit patterns (uint16) expected")
    M, K = a.shape
    N, Kb = b.shape
    if K != Kb:
        raise ValueError("operands disagree on K")
    idx = np.ascontiguousarray(rows, np.int64)
    if idx.size and (idx.min() < 0 or idx.max() >= M):
        raise ValueError("row index out of range")
    C = np.empty((idx.size, N), np.float64)
    A = np.empty((idx.size, N), np.float64)
    _load().mxo_matmul_nt_bf16_rows(a.ctypes.data, b.ctypes.data, M, N, K, idx.ctypes.data, idx.size,
                                    C.ctypes.data, A.ctypes.data)
    return C, A


def matmul_nt_bf16(a: np.ndarray, b: np.ndarray):
    """All of C = A * B^T (see matmul_nt_bf16_rows)."""
    return matmul_nt_bf16_rows(a, b, np.arange(np.asarray(a).shape[0]))


# ---- ablation arms of the paper (E5M2 elements, OCP v1 scale rule): not part of the recipe ----------
_FMT = {"e4m3": 0, "e5m2": 1}
_RULE = {"up": 0, "ocp": 1}


def e5m2_decode(code: int) -> float:
    return _load().mxo_e5m2_decode(int(code))


def e5m2_encode(t: float) -> int:
    return _load().mxo_e5m2_encode(float(t))


def scale_byte_mode(amax: float, fmt: str = "e4m3", rule: str = "up") -> int:
    """Scale byte under the element format and the scale rule ('up' = Algorithm 1, 'ocp' = OCP v1)."""
    return _load().mxo_scale_byte_mode(float(amax), _FMT[fmt], _RULE[rule])


def quantize_rowwise_mode(src: np.ndarray, fmt: str = "e4m3", rule: str = "up"):
    """Row-wise quantization of an FP32 tensor under (fmt, rule): (q, s) like quantize_rowwise."""
    kind, ld = _check_src(src)
    if kind != "f32":
        raise TypeError("FP32 source only")
    rows, cols = src.shape
    if cols % K_BLOCK:
        raise ValueError("cols must be a multiple of 32")
    q = np.empty((rows, cols), np.uint8)
    s = np.empty((rows, cols // K_BLOCK), np.uint8)
    _load().mxo_quantize_rowwise_mode_f32(src.ctypes.data, rows, cols, ld, _u8(q), _u8(s), _FMT[fmt], _RULE[rule])
    return q, s


def dequantize_mode(q: np.ndarray, s: np.ndarray, fmt: str = "e4m3") -> np.ndarray:
    """Decoded values under the element format, in double."""
    _check_qs(q, s)
    rows, cols = q.shape
    out = np.empty((rows, cols), np.float64)
    _load().mxo_dequantize_mode_f64(_u8(q), _u8(s), rows, cols, out.ctypes.data, _FMT[fmt])
    return out


def gemm_mode(a_q, a_s, a_fmt, b_q, b_s, b_fmt):
    """C = A * B^T with each operand's elements in its own FP8 format ('e4m3' or 'e5m2'; Section 3.2.2 compares
    them per tensor type): the block-scaled sum of Section 2 / Appendix A.3 written as the product of the decoded
    operands in double (every decoded value and every product of two is exact there). Returns (C, sum|a*b|)."""
    da, db = dequantize_mode(a_q, a_s, a_fmt), dequantize_mode(b_q, b_s, b_fmt)
    if da.shape[1] != db.shape[1]:
        raise ValueError("operands disagree on K")
    with np.errstate(invalid="ignore", over="ignore"):
        return da @ db.T, np.abs(da) @ np.abs(db).T

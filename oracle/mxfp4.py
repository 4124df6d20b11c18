"""MXFP4 (E2M1 elements, UE8M0 block scales, K = 32: Table 1) reference arithmetic on the CPU, in numpy float64.

THIS FILE IS TEST INFRASTRUCTURE, like the rest of oracle/: only the tests, the smoke check and the benchmark's
cpu_baseline leg may use it; the product never does, and the two share no code.

The recipe of the paper is MXFP8; Table 1 lists MXFP4 as the narrower member of the same family, and everything
here is the paper's conversion (Section 3.3, Algorithm 1, Appendix A.1 and A.2) with the E2M1 constants put in:
  - elements: sign, 2 exponent bits (bias 1), 1 mantissa bit; exponent field 0 is subnormal (0 or 0.5); the
    eight magnitudes are 0, 0.5, 1, 1.5, 2, 3, 4, 6 (max normal 1.5 * 2^2, min subnormal 2^-1: Table 1); there
    is no NaN and no Inf code;
  - scale: the smallest n with amax <= 6 * 2^n, clamped to [-127, 127], stored as n + 127 (Algorithm 1 with
    destmax = 6); 0xFF marks a NaN block (the only place a NaN can live);
  - elements of a block: RNE(V_i / X) to the nearest magnitude, ties to the even code, saturating at +-6;
  - storage: two codes per byte, the element with the even index in the low nibble (OCP MX v1.0 packing).
Readings where the paper is silent (parity unpinned, same choices as for MXFP8): a block containing a NaN gets
scale 0xFF and zero codes; a block with +-Inf and no NaN gets scale byte 254, its infinities saturate to +-6 and
its finite values are divided by 2^127; the sign bit of every input is kept.
Layouts as for MXFP8 with half the element bytes: rowwise q [rows x cols/2], s [rows x cols/32]; colwise (blocks of
32 rows) stored transposed: qT [cols x rows/2], sT [cols x rows/32].
"""
import numpy as np

K_BLOCK = 32
E2M1_MAX = 6.0


def e2m1_decode(code):
    """Value of a 4-bit code (array or scalar), by the format's definition."""
    code = np.asarray(code, np.int64)
    e, m = (code >> 1) & 3, code & 1
    mag = np.where(e == 0, m * 0.5, (1.0 + 0.5 * m) * np.exp2((e - 1).astype(np.float64)))
    return np.where(code & 8, -mag, mag)


def e2m1_encode(t):
    """Nearest code to t (float64 array): round to nearest, ties to the even code, saturating; the sign bit is kept
    (also for zero). NaN has no code: callers never pass one (NaN blocks are handled by the scale)."""
    t = np.asarray(t, np.float64)
    mags = e2m1_decode(np.arange(8))
    a = np.minimum(np.abs(t), E2M1_MAX)
    d = np.abs(a[..., None] - mags)                       # distance to each of the eight magnitudes
    best = d.min(-1, keepdims=True)
    cand = d == best                                      # one candidate, or two neighbours at a tie
    even = cand & (np.arange(8) % 2 == 0)
    pick = np.where(cand.sum(-1, keepdims=True) > 1, even, cand)
    code = pick.argmax(-1)
    return (code | np.where(np.signbit(t), 8, 0)).astype(np.uint8)


def scale_byte(amax):
    """n + 127 for the smallest n in [-127, 127] with amax <= 6 * 2^n (array in, array out); NaN -> 0xFF."""
    amax = np.asarray(amax, np.float64)
    n = np.full(amax.shape, 127, np.int64)
    for k in range(126, -128, -1):                        # the smallest qualifying n: walk down while it still qualifies
        n = np.where(amax <= np.ldexp(E2M1_MAX, k), k, n)
    return np.where(np.isnan(amax), 0xFF, n + 127).astype(np.uint8)


def _widen(src):
    src = np.asarray(src)
    if src.dtype == np.uint16:                            # BF16 bit patterns
        return (src.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if src.dtype == np.float32:
        return src.astype(np.float64)
    raise TypeError("source must be float32 or uint16 (BF16 bit patterns)")


def quantize_rowwise(src):
    """[rows x cols] -> (q [rows x cols/2] u8, s [rows x cols/32] u8); blocks run along a row."""
    v = _widen(src)
    rows, cols = v.shape
    if cols % K_BLOCK:
        raise ValueError("cols must be a multiple of 32")
    blk = v.reshape(rows, cols // K_BLOCK, K_BLOCK)
    a = np.abs(blk)
    has_nan = np.isnan(a).any(-1)
    amax = np.where(np.isnan(a), 0.0, a).max(-1)
    s = np.where(has_nan, 0xFF, scale_byte(amax)).astype(np.uint8)
    n = s.astype(np.int64) - 127
    with np.errstate(invalid="ignore"):
        codes = e2m1_encode(np.ldexp(np.where(np.isnan(blk), 0.0, blk), -n[..., None]))   # V_i / X, exact (or Inf)
    codes = np.where(has_nan[..., None], 0, codes).reshape(rows, cols)
    q = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    return q, s


def quantize_colwise(src):
    """[rows x cols] -> (qT [cols x rows/2] u8, sT [cols x rows/32] u8); blocks run down a column."""
    src = np.asarray(src)
    return quantize_rowwise(np.ascontiguousarray(src.T))


def unpack(q):
    """[rows x cols/2] bytes -> [rows x cols] codes."""
    q = np.asarray(q, np.uint8)
    out = np.empty((q.shape[0], q.shape[1] * 2), np.uint8)
    out[:, 0::2] = q & 0xF
    out[:, 1::2] = q >> 4
    return out


def dequantize(q, s):
    """Decoded values Q_i * 2^(S - 127) in float64 (NaN for a 0xFF scale)."""
    codes = unpack(q)
    s = np.asarray(s, np.uint8)
    scale = np.repeat(np.where(s == 0xFF, np.nan, np.exp2(s.astype(np.float64) - 127.0)), K_BLOCK, axis=1)
    return e2m1_decode(codes) * scale


def gemm(a_q, a_s, b_q, b_s):
    """C = A * B^T for MXFP4 operands A [M x K/2], B [N x K/2] (blocks along K): the block-scaled sum of Section 2
    and Appendix A.3, C[m, n] = sum_b 2^(a_s[m,b] + b_s[n,b] - 254) * sum_{i<32} P_a[m,32b+i] * P_b[n,32b+i], written
    as the product of the decoded operands in float64 (every decoded value and every product of two is exact there;
    the sum rounds at 2^-53 per addition). Returns (C, sum|a*b|) for tolerances; a 0xFF scale makes its row NaN."""
    da, db = dequantize(a_q, a_s), dequantize(b_q, b_s)
    if da.shape[1] != db.shape[1]:
        raise ValueError("operands disagree on K")
    with np.errstate(invalid="ignore", over="ignore"):
        return da @ db.T, np.abs(da) @ np.abs(db).T

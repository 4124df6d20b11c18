"""MXFP6 (E2M3 or E3M2 elements, UE8M0 block scales, K = 32: Table 1) reference arithmetic on the CPU, in numpy float64.

THIS FILE IS TEST INFRASTRUCTURE, like the rest of oracle/: only the tests, the smoke check and the benchmark's
cpu_baseline leg may use it; the product never does, and the two share no code.

The recipe of the paper is MXFP8; Table 1 lists MXFP6 between MXFP8 and MXFP4, and everything here is the paper's
conversion (Section 3.3, Algorithm 1, Appendix A.1 and A.2) with the 6-bit constants put in:
  - E2M3: sign, 2 exponent bits (bias 1), 3 mantissa bits; largest magnitude 1.875 * 2^2 = 7.5, smallest subnormal
    2^-3; E3M2: sign, 3 exponent bits (bias 3), 2 mantissa bits; largest magnitude 1.75 * 2^4 = 28, smallest
    subnormal 2^-4. Exponent field 0 is subnormal; there is no NaN and no Inf code.
    Reading: Table 1 prints 2^-3 as the smallest subnormal of E3M2 as well, but its own binade count for that row
    (8.8 = log2(28 / 2^-4)) and the format's definition (bias 3, two mantissa bits) give 2^-4; the table's E2M3 row
    (5.9 = log2(7.5 / 2^-3)) is consistent. The definition is followed.
  - scale: the smallest n with amax <= destmax * 2^n (destmax = 7.5 or 28), clamped to [-127, 127], stored as
    n + 127 (Algorithm 1); 0xFF marks a NaN block (the only place a NaN can live);
  - elements: RNE(V_i / X) to the nearest representable magnitude, ties to the even code, saturating at destmax;
  - storage: the 32 six-bit codes of a block are packed into 24 bytes as one little-endian 192-bit string, code i
    in bits 6i .. 6i+5 (the order in which the 6-bit matrix instructions of gfx950 take a block).
Readings where the paper is silent (parity unpinned, same choices as for MXFP8 and MXFP4): a block containing a
NaN gets scale 0xFF and zero codes; a block with +-Inf and no NaN gets scale byte 254, its infinities saturate to
+-destmax and its finite values are divided by 2^127; the sign bit of every input is kept.
Layouts: rowwise q [rows x cols*3/4], s [rows x cols/32]; colwise (blocks of 32 rows) stored transposed:
qT [cols x rows*3/4], sT [cols x rows/32].
"""
import numpy as np

K_BLOCK = 32
FORMATS = {"e2m3": (2, 3), "e3m2": (3, 2)}     # exponent bits, mantissa bits


def _em(fmt):
    return FORMATS[fmt]


def decode(code, fmt):
    """Value of a 6-bit code (array or scalar), by the format's definition."""
    E, M = _em(fmt)
    bias = (1 << (E - 1)) - 1
    code = np.asarray(code, np.int64)
    e, m = (code >> M) & ((1 << E) - 1), code & ((1 << M) - 1)
    frac = m / float(1 << M)
    mag = np.where(e == 0, frac * 2.0 ** (1 - bias), (1.0 + frac) * np.exp2((e - bias).astype(np.float64)))
    return np.where(code & 32, -mag, mag)


def dest_max(fmt):
    return float(decode(31, fmt))


def encode(t, fmt):
    """Nearest code to t (float64 array): round to nearest, ties to the even code, saturating; the sign bit is kept
    (also for zero). NaN has no code: callers never pass one (NaN blocks are handled by the scale)."""
    t = np.asarray(t, np.float64)
    mags = decode(np.arange(32), fmt)                    # increasing with the code
    a = np.minimum(np.abs(t), mags[-1])
    d = np.abs(a[..., None] - mags)                       # distance to each of the 32 magnitudes
    best = d.min(-1, keepdims=True)
    cand = d == best                                      # one candidate, or two neighbours at a tie
    even = cand & (np.arange(32) % 2 == 0)
    pick = np.where(cand.sum(-1, keepdims=True) > 1, even, cand)
    code = pick.argmax(-1)
    return (code | np.where(np.signbit(t), 32, 0)).astype(np.uint8)


def scale_byte(amax, fmt):
    """n + 127 for the smallest n in [-127, 127] with amax <= destmax * 2^n (array in, array out); NaN -> 0xFF."""
    amax = np.asarray(amax, np.float64)
    top = dest_max(fmt)
    n = np.full(amax.shape, 127, np.int64)
    for k in range(126, -128, -1):                        # the smallest qualifying n: walk down while it still qualifies
        n = np.where(amax <= np.ldexp(top, k), k, n)
    return np.where(np.isnan(amax), 0xFF, n + 127).astype(np.uint8)


def _widen(src):
    src = np.asarray(src)
    if src.dtype == np.uint16:                            # BF16 bit patterns
        return (src.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if src.dtype == np.float32:
        return src.astype(np.float64)
    raise TypeError("source must be float32 or uint16 (BF16 bit patterns)")


def pack(codes):
    """[rows x cols] 6-bit codes -> [rows x cols*3/4] bytes: per block of 32 one little-endian 192-bit string."""
    codes = np.asarray(codes, np.uint8)
    rows, cols = codes.shape
    bits = ((codes[..., None] >> np.arange(6)) & 1).astype(np.uint8).reshape(rows, cols * 6)   # LSB first
    return np.packbits(bits, axis=1, bitorder="little")


def unpack(q):
    """[rows x cols*3/4] bytes -> [rows x cols] codes."""
    q = np.asarray(q, np.uint8)
    bits = np.unpackbits(q, axis=1, bitorder="little").reshape(q.shape[0], -1, 6)
    return (bits << np.arange(6, dtype=np.uint8)).sum(-1).astype(np.uint8)


def quantize_rowwise(src, fmt):
    """[rows x cols] -> (q [rows x cols*3/4] u8, s [rows x cols/32] u8); blocks run along a row."""
    v = _widen(src)
    rows, cols = v.shape
    if cols % K_BLOCK:
        raise ValueError("cols must be a multiple of 32")
    blk = v.reshape(rows, cols // K_BLOCK, K_BLOCK)
    a = np.abs(blk)
    has_nan = np.isnan(a).any(-1)
    amax = np.where(np.isnan(a), 0.0, a).max(-1)
    s = np.where(has_nan, 0xFF, scale_byte(amax, fmt)).astype(np.uint8)
    n = s.astype(np.int64) - 127
    with np.errstate(invalid="ignore"):
        codes = encode(np.ldexp(np.where(np.isnan(blk), 0.0, blk), -n[..., None]), fmt)   # V_i / X, exact (or Inf)
    codes = np.where(has_nan[..., None], 0, codes).reshape(rows, cols).astype(np.uint8)
    return pack(codes), s


def quantize_colwise(src, fmt):
    """[rows x cols] -> (qT [cols x rows*3/4] u8, sT [cols x rows/32] u8); blocks run down a column."""
    return quantize_rowwise(np.ascontiguousarray(np.asarray(src).T), fmt)


def dequantize(q, s, fmt):
    """Decoded values Q_i * 2^(S - 127) in float64 (NaN for a 0xFF scale)."""
    codes = unpack(q)
    s = np.asarray(s, np.uint8)
    scale = np.repeat(np.where(s == 0xFF, np.nan, np.exp2(s.astype(np.float64) - 127.0)), K_BLOCK, axis=1)
    return decode(codes, fmt) * scale


def gemm(a_q, a_s, b_q, b_s, fmt_a, fmt_b=None):
    """C = A * B^T for MXFP6 operands (blocks along K): the block-scaled sum of Section 2 and Appendix A.3 written
    as the product of the decoded operands in float64 (every decoded value and every product of two is exact
    there). Returns (C, sum|a*b|)."""
    da, db = dequantize(a_q, a_s, fmt_a), dequantize(b_q, b_s, fmt_b or fmt_a)
    if da.shape[1] != db.shape[1]:
        raise ValueError("operands disagree on K")
    with np.errstate(invalid="ignore", over="ignore"):
        return da @ db.T, np.abs(da) @ np.abs(db).T

"""Pins for the CPU oracle: everything here checks ``oracle/`` against something other than itself
-- constants the paper prints, closed forms, exact integer arithmetic, invariants, a library cast
inside the range where it is a special case of the method, and brute force on tiny inputs.
No GPU is used."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2506_08027_amd import synth_inputs as si


# ------------------------------------------------------------------------------------------------
# Format constants (Section 2, Table 1)
# ------------------------------------------------------------------------------------------------

def _golden(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "table1_e4m3_ue8m0.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def test_e4m3_table_matches_paper_constants(golden_dir):
    g = _golden(golden_dir)
    vals = np.array([oracle.e4m3_decode(c) for c in range(256)])
    nan_codes = [c for c in range(256) if math.isnan(vals[c])]
    assert nan_codes == [0x7F, 0xFF]                      # one NaN pattern per sign, no Inf
    assert int(g["e4m3_nan_patterns_per_sign"]) == 1 and int(g["e4m3_has_infinity"]) == 0
    assert not np.isinf(vals).any()
    finite = vals[~np.isnan(vals)]
    vmax = g["e4m3_max_normal_significand"] * 2.0 ** g["e4m3_max_normal_exponent"]
    assert vmax == 448.0 and finite.max() == vmax and finite.min() == -vmax
    pos = finite[finite > 0]
    assert pos.min() == 2.0 ** g["e4m3_min_subnormal_exponent"]
    assert round(math.log2(pos.max() / pos.min()), 1) == g["e4m3_binades"]
    # strictly increasing with the code inside each sign; negative half mirrors the positive one
    assert np.all(np.diff(vals[0:0x7F]) > 0)
    assert np.array_equal(vals[0x80:0xFF], -vals[0x00:0x7F])
    assert vals[0] == 0 and math.copysign(1.0, vals[0x80]) == -1.0
    # 253 distinct finite values (+0 and -0 coincide)
    assert len(np.unique(finite)) == 253


def test_e4m3_decode_agrees_with_library_type():
    """The OCP 'e4m3fn' type in PyTorch decodes the same 256 codes."""
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = np.array([oracle.e4m3_decode(c) for c in range(256)])
    assert np.array_equal(np.isnan(lib), np.isnan(ours))
    m = ~np.isnan(lib)
    assert np.array_equal(lib[m], ours[m])
    assert np.array_equal(np.signbit(lib[m]), np.signbit(ours[m]))


def test_ue8m0_range(golden_dir):
    g = _golden(golden_dir)
    assert oracle.scale_byte(0.0) - g["ue8m0_bias"] == g["ue8m0_min_exponent"]
    assert oracle.scale_byte(float("inf")) - g["ue8m0_bias"] == g["ue8m0_max_exponent"]
    assert oracle.scale_byte(float("nan")) == 0xFF
    q = np.full((1, 32), 0x38, np.uint8)      # 1.0
    for sbyte in range(255):
        d = oracle.dequantize(q, np.array([[sbyte]], np.uint8))
        assert np.all(d == 2.0 ** (sbyte - 127))
    assert np.isnan(oracle.dequantize(q, np.array([[255]], np.uint8))).all()


# ------------------------------------------------------------------------------------------------
# Scale rule (Algorithm 1, Appendix A.1)
# ------------------------------------------------------------------------------------------------

def test_scale_closed_form_at_448_times_power_of_two():
    """amax = 448*2^k maps exactly onto the format maximum (not bumped); the next FP32 above needs
    the next power of two; the one below does not."""
    for k in list(range(-127, 120)):
        a = np.float32(448.0 * 2.0 ** k)
        assert oracle.scale_byte(float(a)) == k + 127
        up = np.nextafter(a, np.float32(np.inf))
        if np.isfinite(up):
            assert oracle.scale_byte(float(up)) == min(k + 1, 127) + 127
        down = np.nextafter(a, np.float32(0))
        assert oracle.scale_byte(float(down)) == k + 127
    # lower clamp: everything at or below 448*2^-127, all FP32 subnormals and zero included
    for a in (0.0, 2.0 ** -149, 2.0 ** -126, 448.0 * 2.0 ** -127, 448.0 * 2.0 ** -130):
        assert oracle.scale_byte(a) == 0
    # largest finite FP32 stays well below the upper end
    assert oracle.scale_byte(float(np.finfo(np.float32).max)) == 247


def _exact_ceil_log2_ratio(bits: int) -> int:
    """ceil(log2(amax/448)) for a positive finite FP32 bit pattern, in exact rational arithmetic."""
    e = bits >> 23
    m = bits & 0x7FFFFF
    amax = Fraction(m, 1 << 23) * Fraction(2) ** -126 if e == 0 else \
        (1 + Fraction(m, 1 << 23)) * Fraction(2) ** (e - 127)
    ratio = amax / 448
    n = -400
    while Fraction(2) ** n < ratio:
        n += 1
    return n


def test_scale_equals_exact_ceil_log2_on_random_fp32():
    rng = np.random.default_rng(11)
    bits = rng.integers(1, 0x7F800000, 3000, dtype=np.int64)
    edge = []
    for e in (1, 8, 9, 100, 127, 135, 254):
        for m in (0, 1, 0x5FFFFF, 0x600000, 0x600001, 0x7FFFFF):
            edge.append((e << 23) | m)
    for b in list(bits) + edge:
        a = float(np.array([b], np.uint32).view(np.float32)[0])
        n = max(-127, min(127, _exact_ceil_log2_ratio(int(b))))
        assert oracle.scale_byte(a) == n + 127, hex(int(b))


@pytest.mark.parametrize("biased_exp", [1, 8, 9, 100, 127, 254])
def test_scale_bit_rule_over_all_mantissas(biased_exp):
    """Across all 2^23 mantissas of a binade the rule is a step at mantissa 1.75: the scale byte is
    e-8 up to and including 1.75 and e-7 above it (Appendix A.1: non powers of two round up), and it
    is the OCP-v1 round-down exponent plus 0 or 1 (Section 3.3)."""
    e = biased_exp
    # the byte can only change where amax crosses 448*2^n, i.e. at mantissa field 0x600000
    probe = np.array([0, 1, 0x2AAAAA, 0x5FFFFF, 0x600000, 0x600001, 0x700000, 0x7FFFFF], np.uint32)
    dense = np.arange(0x600000 - 2048, 0x600000 + 2048, dtype=np.uint32)
    rng = np.random.default_rng(e)
    m = np.unique(np.concatenate([probe, dense, rng.integers(0, 1 << 23, 20000).astype(np.uint32)]))
    vals = ((np.uint32(e) << 23) | m).view(np.float32).astype(np.float64)
    got = np.array([oracle.scale_byte(v) for v in vals])
    want = np.maximum(0, e - 8 + (m > 0x600000))
    assert np.array_equal(got, want)
    ocp_floor = np.maximum(0, e - 8)        # floor(log2 amax) - 8, biased, clamped the same way
    assert set(np.unique(got - ocp_floor)) <= {0, 1}
    assert np.array_equal((got - ocp_floor) == 1, (m > 0x600000) & (e - 8 + 1 > 0))


def test_no_overflow_and_tight_scale_invariants():
    """Section 3.3: after scaling no value exceeds 448, and X is the smallest such power of two."""
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((64, 256)) * np.exp(rng.uniform(-80, 80, (64, 1)))).astype(np.float32)
    q, s = oracle.quantize_rowwise(x)
    assert s.max() <= 247
    n = s.astype(np.int64) - 127
    amax = np.abs(x.astype(np.float64)).reshape(64, 8, 32).max(-1)
    scaled = amax * 2.0 ** (-n.astype(np.float64))
    assert np.all(scaled <= 448.0)
    unclamped = s > 0
    assert np.all(scaled[unclamped] > 224.0)
    d = oracle.dequantize(q, s)
    assert np.all(np.abs(d) <= 448.0 * 2.0 ** np.repeat(n, 32, axis=1).astype(np.float64))
    # error bounds of an E4M3 grid: relative 2^-4 in the normal range, absolute 2^-10 * X below it
    X = 2.0 ** np.repeat(n, 32, axis=1).astype(np.float64)
    t = np.abs(x.astype(np.float64)) / X
    err = np.abs(d - x.astype(np.float64)) / X
    normal = t >= 2.0 ** -6
    assert np.all(err[normal] <= t[normal] * 2.0 ** -4)
    assert np.all(err[~normal] <= 2.0 ** -10)
    # the block maximum itself always lands in the top binade [256, 448] (or the block is clamped)
    top = np.abs(oracle.dequantize(q, s) / X).reshape(64, 8, 32).max(-1)
    assert np.all(top[unclamped] >= 224.0)


# ------------------------------------------------------------------------------------------------
# Element conversion (Section 3.3, Appendix A.2)
# ------------------------------------------------------------------------------------------------

def test_encoder_matches_library_rne_cast_inside_range():
    """For |t| <= 448 the conversion is the standard round-to-nearest-even cast to OCP e4m3."""
    rng = np.random.default_rng(3)
    vals = np.array([oracle.e4m3_decode(c) for c in range(0x7F)])
    mids = (vals[:-1] + vals[1:]) / 2              # every tie point
    eps = np.concatenate([np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf)])
    bf = si.bf16_bits_to_f32(np.arange(0, 0x7F80, dtype=np.uint16)).astype(np.float64)
    rnd = rng.uniform(-448, 448, 20000)
    small = rng.uniform(-1, 1, 20000) * 2.0 ** rng.integers(-30, 0, 20000)
    t = np.concatenate([vals, -vals, mids, -mids, eps, -eps, bf[bf <= 448], -bf[bf <= 448], rnd, small])
    t = t[np.abs(t) <= 448.0]
    # the library casts from FP32: keep only probes FP32 holds exactly so both sides see one value
    t = t[t.astype(np.float32).astype(np.float64) == t]
    lib = torch.from_numpy(t.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    ours = np.array([oracle.e4m3_encode(x) for x in t], np.uint8)
    assert np.array_equal(lib, ours)


def test_encoder_ties_saturation_sign():
    enc = oracle.e4m3_encode
    assert enc(0.0) == 0x00 and enc(-0.0) == 0x80
    assert enc(2.0 ** -10) == 0x00           # halfway between 0 and 2^-9: even code is 0
    assert enc(-(2.0 ** -10)) == 0x80
    assert enc(3 * 2.0 ** -10) == 0x02       # halfway between codes 1 and 2
    assert enc(np.nextafter(2.0 ** -10, 1)) == 0x01
    assert enc(448.0) == 0x7E and enc(-448.0) == 0xFE
    assert enc(432.0) == 0x7E                # halfway between 416 (0x7D) and 448 (0x7E)
    assert enc(400.0) == 0x7C                # halfway between 384 (0x7C) and 416 (0x7D)
    for big in (448.0000001, 464.0, 480.0, 1e30, float("inf")):
        assert enc(big) == 0x7E and enc(-big) == 0xFE
    assert enc(float("nan")) == 0x7F and enc(-float("nan")) == 0x7F   # one canonical NaN byte (reading R5)
    assert enc(1.0) == 0x38 and enc(1.0625) == 0x38 and enc(1.1875) == 0x3A  # ties to even mantissa


def test_every_code_round_trips_under_every_reachable_scale():
    """Exact round trip: a block of representable values decodes back to itself (values; the
    stored scale may be smaller than the one the block was built with)."""
    vals = np.array([oracle.e4m3_decode(c) for c in list(range(0x7F)) + list(range(0x80, 0xFF))])
    for n in (-127, -126, -100, -10, 0, 3, 64, 118, 119):
        blocks = []
        for start in range(0, len(vals), 31):
            v = list(vals[start:start + 31])
            v += [0.0] * (31 - len(v)) + [448.0]        # pivot keeps the scale at 2^n
            blocks.append(v)
        x = (np.array(blocks, np.float64) * 2.0 ** n).astype(np.float32)
        assert np.array_equal(x.astype(np.float64), np.array(blocks) * 2.0 ** n)  # exact in FP32
        q, s = oracle.quantize_rowwise(x)
        assert np.all(s == n + 127)
        assert np.array_equal(oracle.dequantize(q, s), x.astype(np.float64))
        # and through the FP32-rounded decode
        assert np.array_equal(oracle.dequantize(q, s, "f32"), x)


def test_idempotence_and_power_of_two_invariance():
    x = si.activations(64, 256, seed=7, bf16=False)
    q, s = oracle.quantize_rowwise(x)
    d = oracle.dequantize(q, s, "f32")
    q2, s2 = oracle.quantize_rowwise(d)
    assert np.array_equal(oracle.dequantize(q2, s2, "f32"), d)
    for k in (-20, 5, 60):
        qk, sk = oracle.quantize_rowwise((x.astype(np.float64) * 2.0 ** k).astype(np.float32))
        assert np.array_equal(qk, q)
        assert np.array_equal(sk.astype(int), s.astype(int) + k)


def test_all_bf16_patterns_against_exact_integer_rounding():
    """Every finite BF16 value as an element of a block whose scale is pinned to 1 by a pivot of
    448: compare with round-half-even done in integer arithmetic on the E4M3 grid."""
    bits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    f = si.bf16_bits_to_f32(bits)
    keep = np.isfinite(f) & (np.abs(f) <= 448)
    bits = bits[keep]
    pad = (-len(bits)) % 31
    bits = np.concatenate([bits, np.zeros(pad, np.uint16)])
    blk = bits.reshape(-1, 31)
    pivot = np.full((blk.shape[0], 1), si.to_bf16_bits(np.array([448.0], np.float32))[0], np.uint16)
    src = np.ascontiguousarray(np.concatenate([blk, pivot], axis=1))
    q, s = oracle.quantize_rowwise(src)
    assert np.all(s == 127)
    got = oracle.dequantize(q, s)[:, :31].ravel()
    x = si.bf16_bits_to_f32(blk.ravel()).astype(np.float64)
    # expected: grid spacing is 2^(max(e,-6)-3) where e = floor(log2|x|)
    want = np.empty_like(x)
    for i, v in enumerate(x):
        a = abs(v)
        if a == 0:
            want[i] = v
            continue
        e = max(math.frexp(a)[1] - 1, -6)
        step = Fraction(2) ** (e - 3)
        k = Fraction(a) / step
        fl = k.numerator // k.denominator
        rem = k - fl
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
            fl += 1
        want[i] = math.copysign(float(fl * step), v)
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), np.signbit(want))


# ------------------------------------------------------------------------------------------------
# Row / column copies (Section 3.2) and special blocks
# ------------------------------------------------------------------------------------------------

def test_colwise_is_rowwise_of_the_transpose():
    x = si.tiny_with_specials(256, 0)
    qT, sT = oracle.quantize_colwise(x)
    q2, s2 = oracle.quantize_rowwise(np.ascontiguousarray(x.T))
    assert np.array_equal(qT, q2) and np.array_equal(sT, s2)
    xb = si.activations(64, 96, seed=1)
    qT, sT = oracle.quantize_colwise(xb)
    q2, s2 = oracle.quantize_rowwise(np.ascontiguousarray(xb.T))
    assert np.array_equal(qT, q2) and np.array_equal(sT, s2)


def test_leading_dimension_is_honoured():
    x = si.activations(32, 128, seed=9, bf16=False)
    view = x[:, 32:96]
    q, s = oracle.quantize_rowwise(view)
    q2, s2 = oracle.quantize_rowwise(np.ascontiguousarray(view))
    assert np.array_equal(q, q2) and np.array_equal(s, s2)
    for v in (view, si.to_bf16_bits(x)[:, 32:96]):
        qT, sT = oracle.quantize_colwise(v)
        qT2, sT2 = oracle.quantize_colwise(np.ascontiguousarray(v))
        assert np.array_equal(qT, qT2) and np.array_equal(sT, sT2)


def test_special_blocks():
    for name, v in si.special_blocks(0):
        q, s = oracle.quantize_rowwise(v.reshape(1, 32).copy())
        q, s = q[0], int(s[0, 0])
        if name == "zero":
            assert s == 0 and np.array_equal(q, np.where(np.signbit(v), 0x80, 0).astype(np.uint8))
        elif name.startswith("subnormal"):
            assert s == 0
            # elements are scaled by 2^127, not flushed: anything above 2^-137 gives a nonzero code
            nz = np.abs(v.astype(np.float64)) > 2.0 ** -137
            assert np.all((q[nz] & 0x7F) != 0) and np.all((q[~nz] & 0x7F) == 0)
        elif name.startswith("amax448p"):
            k = int(name[len("amax448p"):].split("_")[0])
            n = k + 1 if name.endswith("_up") else k
            assert s == max(n, -127) + 127
            top = np.abs(np.array([oracle.e4m3_decode(c) for c in q])).max()
            if n >= -127 and not name.endswith("_up") and not name.endswith("_down"):
                assert top == 448.0
            if name.endswith("_up") and n >= -127:
                assert top == 224.0
        elif name in ("nan", "nan_inf"):
            assert s == 0xFF and np.all(q == 0x7F)
        elif name in ("pinf", "ninf", "inf_big"):
            assert s == 254
            inf = np.isinf(v)
            assert np.array_equal(q[inf], np.where(v[inf] > 0, 0x7E, 0xFE).astype(np.uint8))
            d = oracle.dequantize(q.reshape(1, 32), np.array([[s]], np.uint8), "f32")[0]
            assert np.array_equal(d[inf], v[inf])          # Inf survives the round trip
            # finite neighbours were divided by 2^127: their codes are below 2 in magnitude
            assert np.all(np.abs([oracle.e4m3_decode(c) for c in q[~inf]]) <= 2.0)
            assert np.array_equal(d[~inf].astype(np.float64),
                                  np.array([oracle.e4m3_decode(c) for c in q[~inf]]) * 2.0 ** 127)


# ------------------------------------------------------------------------------------------------
# Decode and output rounding
# ------------------------------------------------------------------------------------------------

def test_bf16_rounding_helper_matches_library():
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(5000) * np.exp(rng.uniform(-90, 88, 5000)),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.4e38, 3.39e38, 1e-40, 9.2e-41, 4.6e-41]])
    x = x.astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    ours = np.array([oracle.round_to_bf16_bits(float(v)) for v in x], np.uint16)
    assert np.array_equal(lib, ours)


def test_dequantize_all_codes_all_scales_against_library():
    """256 codes x every scale byte: FP32 decode equals the library decode times 2^(S-127)."""
    codes = np.tile(np.arange(256, dtype=np.uint8), 1).reshape(8, 32)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for sbyte in range(255):
        s = np.full((8, 1), sbyte, np.uint8)
        got = oracle.dequantize(codes, s, "f64")
        want = lib * 2.0 ** (sbyte - 127)
        m = ~np.isnan(want)
        assert np.array_equal(np.isnan(got), np.isnan(want))
        assert np.array_equal(got[m], want[m])
        g32 = oracle.dequantize(codes, s, "f32")
        assert np.array_equal(g32[m], want[m].astype(np.float32))
        g16 = oracle.dequantize(codes, s, "bf16")
        w16 = torch.from_numpy(want.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(g16[m], w16[m])


# ------------------------------------------------------------------------------------------------
# Block-scaled GEMM (Section 2, Appendix A.3)
# ------------------------------------------------------------------------------------------------

def test_gemm_equals_library_matmul_of_decoded_operands():
    a = si.activations(48, 256, seed=21)
    b = si.weights(40, 256, seed=22)
    a_q, a_s = oracle.quantize_rowwise(a)
    b_q, b_s = oracle.quantize_rowwise(b)
    C, A = oracle.gemm(a_q, a_s, b_q, b_s)
    da, db = oracle.dequantize(a_q, a_s), oracle.dequantize(b_q, b_s)
    ref = da @ db.T
    ref_abs = np.abs(da) @ np.abs(db).T
    assert np.allclose(C, ref, rtol=0, atol=1e-12 * ref_abs.max())
    assert np.allclose(A, ref_abs, rtol=1e-13)
    # the block-scaled form of Appendix A.3: per-block integer dot products, scale applied per block
    m, n = 5, 7
    acc = Fraction(0)
    for blk in range(256 // 32):
        p = Fraction(0)
        for i in range(32):
            k = blk * 32 + i
            p += Fraction(oracle.e4m3_decode(a_q[m, k])) * Fraction(oracle.e4m3_decode(b_q[n, k]))
        acc += p * Fraction(2) ** (int(a_s[m, blk]) - 127 + int(b_s[n, blk]) - 127)
    assert abs(float(acc) - C[m, n]) <= 2.0 ** -50 * A[m, n]


def test_gemm_one_hot_selects_columns_and_small_integers_are_exact():
    rng = np.random.default_rng(8)
    a = si.activations(32, 128, seed=31)
    a_q, a_s = oracle.quantize_rowwise(a)
    onehot = np.zeros((16, 128), np.float32)
    cols = rng.choice(128, 16, replace=False)
    onehot[np.arange(16), cols] = 1.0
    b_q, b_s = oracle.quantize_rowwise(onehot)
    C, _ = oracle.gemm(a_q, a_s, b_q, b_s)
    assert np.array_equal(C, oracle.dequantize(a_q, a_s)[:, cols])
    ia = rng.integers(-2, 3, (32, 128)).astype(np.float32)
    ib = rng.integers(-2, 3, (24, 128)).astype(np.float32)
    C, A = oracle.gemm(*oracle.quantize_rowwise(ia), *oracle.quantize_rowwise(ib))
    assert np.array_equal(C, (ia.astype(np.int64) @ ib.astype(np.int64).T).astype(np.float64))
    assert np.array_equal(A, (np.abs(ia).astype(np.int64) @ np.abs(ib).astype(np.int64).T).astype(np.float64))


def test_gemm_rows_subset_and_transposed_operand_roles():
    """dgrad and wgrad use the column copies: with them stored transposed every pass is the same
    K-contiguous product (Section 3.2, Figure 2)."""
    x = si.activations(64, 96, seed=41)         # [T x H]
    w = si.weights(32, 96, seed=42)             # [O x H]
    dy = si.gradients(64, 32, seed=43, spikes=True)   # [T x O]
    xq, xs = oracle.quantize_rowwise(x)
    wq, ws = oracle.quantize_rowwise(w)
    y, _ = oracle.gemm(xq, xs, wq, ws)
    assert y.shape == (64, 32)
    sub, _ = oracle.gemm_rows(xq, xs, wq, ws, [3, 60])
    assert np.array_equal(sub, y[[3, 60]])
    # dgrad: dX[T x H] = dY_row[T x O] . W_colT[H x O]^T
    wqT, wsT = oracle.quantize_colwise(w)
    dq, ds = oracle.quantize_rowwise(dy)
    dx, _ = oracle.gemm(dq, ds, wqT, wsT)
    ref = oracle.dequantize(dq, ds) @ oracle.dequantize(wqT, wsT).T
    assert dx.shape == (64, 96) and np.allclose(dx, ref, rtol=1e-12, atol=1e-30)
    # wgrad: dW[O x H] = dY_colT[O x T] . X_colT[H x T]^T
    dqT, dsT = oracle.quantize_colwise(dy)
    xqT, xsT = oracle.quantize_colwise(x)
    dw, _ = oracle.gemm(dqT, dsT, xqT, xsT)
    ref = oracle.dequantize(dqT, dsT) @ oracle.dequantize(xqT, xsT).T
    assert dw.shape == (32, 96) and np.allclose(dw, ref, rtol=1e-12, atol=1e-30)
    # and the quantized product tracks the unquantized one to E4M3 precision
    full = si.bf16_bits_to_f32(x).astype(np.float64) @ si.bf16_bits_to_f32(w).astype(np.float64).T
    assert np.linalg.norm(y - full) / np.linalg.norm(full) < 0.06

"""Pins of the oracle's MXFP4 arithmetic (Table 1: E2M1 elements; conversion of Section 3.3 / Algorithm 1 /
Appendix A.1, A.2 with the E2M1 constants). CPU only."""
import math
import os
from fractions import Fraction

import numpy as np

import oracle
from oracle import mxfp4
from paper_2506_08027_amd import synth_inputs as si

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table1_e2m1.txt")


def test_table_matches_the_paper_constants():
    c = dict(line.split() for line in open(GOLDEN) if line.strip() and not line.startswith("#"))
    vals = mxfp4.e2m1_decode(np.arange(16))
    pos = vals[:8]
    assert list(pos) == [0, 0.5, 1, 1.5, 2, 3, 4, 6] and list(vals[8:]) == [-v for v in pos]
    assert pos.max() == float(c["e2m1_max_normal_significand"]) * 2.0 ** int(c["e2m1_max_normal_exponent"])
    assert pos[pos > 0].min() == 2.0 ** int(c["e2m1_min_subnormal_exponent"])
    assert abs(math.log2(pos.max() / pos[pos > 0].min()) - float(c["e2m1_binades"])) < 0.05
    assert int(c["e2m1_exponent_bits"]) + int(c["e2m1_mantissa_bits"]) + 1 == 4


def test_encoder_is_round_to_nearest_even_and_saturates():
    mags = [Fraction(x) for x in (0, 0.5, 1, 1.5, 2, 3, 4, 6)]
    grid = np.array([0.0, 0.5, 1, 1.5, 2, 3, 4, 6])
    mids = (grid[:-1] + grid[1:]) / 2
    t = np.concatenate([grid, mids, np.nextafter(mids, 0), np.nextafter(mids, 10), np.random.default_rng(0).uniform(0, 7, 2000),
                        [6.0000001, 7, 100, 1e30, np.inf]])
    got = mxfp4.e2m1_encode(np.concatenate([t, -t]))
    for x, code in zip(np.concatenate([t, -t]), got):
        a = min(Fraction(abs(x)) if np.isfinite(x) else Fraction(10 ** 40), Fraction(6))
        best = min(abs(a - m) for m in mags)
        cands = [i for i, m in enumerate(mags) if abs(a - m) == best]
        want = [i for i in cands if i % 2 == 0][0] if len(cands) > 1 else cands[0]
        assert code & 7 == want and bool(code & 8) == bool(np.signbit(x)), (x, code)
    assert mxfp4.e2m1_encode(np.array([-0.0]))[0] == 8 and mxfp4.e2m1_encode(np.array([0.2]))[0] == 0
    assert list(mxfp4.e2m1_encode(np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]))) == [0, 2, 2, 4, 4, 6, 6]   # every tie


def test_scale_rule_closed_form_and_neighbours():
    for k in list(range(-127, 128)):
        edge = np.float64(6.0) * 2.0 ** k
        want = k + 127
        assert mxfp4.scale_byte(np.array([edge]))[0] == want
        assert mxfp4.scale_byte(np.array([np.nextafter(edge, np.inf)]))[0] == min(want + 1, 254)
        assert mxfp4.scale_byte(np.array([np.nextafter(edge, 0)]))[0] == want
    rng = np.random.default_rng(1)
    a = np.abs(rng.standard_normal(2000)) * 2.0 ** rng.integers(-60, 60, 2000)
    for x, b in zip(a, mxfp4.scale_byte(a)):
        n = int(b) - 127
        assert Fraction(x) <= 6 * Fraction(2) ** n and (n == -127 or Fraction(x) > 6 * Fraction(2) ** (n - 1))   # smallest such n
    assert list(mxfp4.scale_byte(np.array([0.0, np.nan, np.inf]))) == [0, 0xFF, 254]


def test_quantize_layout_packing_tightness_and_round_trip():
    x = np.asarray(si.activations(64, 128, seed=2, bf16=False), np.float32)
    q, s = mxfp4.quantize_rowwise(x)
    assert q.shape == (64, 64) and s.shape == (64, 4)
    # packing: element 2i in the low nibble of byte i
    v = x[0, :32].astype(np.float64)
    n = int(s[0, 0]) - 127
    codes = mxfp4.e2m1_encode(np.ldexp(v, -n))
    assert q[0, 0] == (codes[0] | (codes[1] << 4)) and q[0, 15] == (codes[30] | (codes[31] << 4))
    # tightness: the block maximum lands in (3, 6] after scaling, i.e. on code 6 or 7 ... and nothing saturates
    blk = np.abs(x.astype(np.float64)).reshape(64, 4, 32).max(-1)
    scaled = blk / np.exp2(s.astype(np.float64) - 127)
    assert ((scaled > 3) & (scaled <= 6)).all()
    d = mxfp4.dequantize(q, s)
    amax = np.repeat(blk, 32, axis=1)
    assert (np.abs(d - x) <= amax / 3 + 1e-300).all()       # half of the widest step (4 -> 6) is 1 X, and X < amax / 3
    # a fixed point in value: quantizing the decoded tensor decodes to the same tensor (the pair (code, scale) may
    # differ: a block whose maximum rounded down to 3 X is re-scaled to 6 X / 2)
    q2, s2 = mxfp4.quantize_rowwise(d.astype(np.float32))
    assert np.array_equal(mxfp4.dequantize(q2, s2), d)
    # BF16 sources are widened exactly; the column copy is the row copy of the transpose
    xb = si.activations(64, 128, seed=3)
    qb, sb = mxfp4.quantize_rowwise(xb)
    qf, sf = mxfp4.quantize_rowwise(si.bf16_bits_to_f32(xb))
    assert np.array_equal(qb, qf) and np.array_equal(sb, sf)
    qT, sT = mxfp4.quantize_colwise(x)
    qt2, st2 = mxfp4.quantize_rowwise(np.ascontiguousarray(x.T))
    assert qT.shape == (128, 32) and np.array_equal(qT, qt2) and np.array_equal(sT, st2)


def test_special_blocks():
    x = np.ones((1, 96), np.float32)
    x[0, 3] = np.nan
    x[0, 40] = -np.inf
    x[0, 64:96] = 0.0
    x[0, 70] = -0.0
    q, s = mxfp4.quantize_rowwise(x)
    assert s[0, 0] == 0xFF and (q[0, :16] == 0).all()                                  # NaN block
    assert s[0, 1] == 254 and mxfp4.unpack(q)[0, 40] == 0xF and (np.delete(mxfp4.unpack(q)[0, 32:64], 8) == 0).all()   # Inf -> -6, 1 / 2^127 -> 0
    assert s[0, 2] == 0 and mxfp4.unpack(q)[0, 70] == 8 and mxfp4.unpack(q)[0, 71] == 0     # zero block, sign of zero kept
    d = mxfp4.dequantize(q, s)
    assert np.isnan(d[0, :32]).all() and d[0, 40] == -6.0 * 2.0 ** 127 and (d[0, 64:] == 0).all()


def test_product_of_decoded_operands_reduces_to_the_bf16_product():
    """Q_i * X has 2 significant bits: decoding to BF16 is exact, so the MXFP4 product is the oracle's BF16 product
    of the decoded operands (the route the GPU tests use), and agrees with a library matmul."""
    a = np.asarray(si.activations(16, 128, seed=2, bf16=False), np.float32)
    b = np.asarray(si.weights(24, 128, seed=4, bf16=False), np.float32)
    da, db = mxfp4.dequantize(*mxfp4.quantize_rowwise(a)), mxfp4.dequantize(*mxfp4.quantize_rowwise(b))
    ba, bb = si.to_bf16_bits(da.astype(np.float32)), si.to_bf16_bits(db.astype(np.float32))
    assert np.array_equal(si.bf16_bits_to_f32(ba).astype(np.float64), da) and np.array_equal(si.bf16_bits_to_f32(bb).astype(np.float64), db)
    C, A = oracle.matmul_nt_bf16(ba, bb)
    ref = da @ db.T
    assert np.allclose(C, ref, rtol=0, atol=1e-13 * np.abs(ref).max()) and np.allclose(A, np.abs(da) @ np.abs(db).T, rtol=1e-13)


def test_gemm_is_the_block_scaled_sum_written_out():
    """Brute force on a tiny case: the double loop over blocks and elements of Section 2's definition, with the
    scale applied per block pair, in exact rational arithmetic."""
    from fractions import Fraction
    rng = np.random.default_rng(9)
    M, N, K = 3, 4, 64
    a = (rng.standard_normal((M, K)) * np.exp2(rng.integers(-6, 6, (M, 1)))).astype(np.float32)
    b = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    (a_q, a_s), (b_q, b_s) = mxfp4.quantize_rowwise(a), mxfp4.quantize_rowwise(b)
    C, A = mxfp4.gemm(a_q, a_s, b_q, b_s)
    ca, cb = mxfp4.unpack(a_q), mxfp4.unpack(b_q)
    val = [Fraction(x) for x in (0, 0.5, 1, 1.5, 2, 3, 4, 6)]
    for m in range(M):
        for n in range(N):
            tot, tot_abs = Fraction(0), Fraction(0)
            for blk in range(K // 32):
                inner = inner_abs = Fraction(0)
                for i in range(32):
                    x, y = int(ca[m, 32 * blk + i]), int(cb[n, 32 * blk + i])
                    p = val[x & 7] * val[y & 7]
                    inner += -p if (x ^ y) & 8 else p
                    inner_abs += p
                sc = Fraction(2) ** (int(a_s[m, blk]) + int(b_s[n, blk]) - 254)
                tot += sc * inner
                tot_abs += sc * inner_abs
            assert abs(Fraction(C[m, n]) - tot) <= Fraction(2) ** -45 * tot_abs and Fraction(A[m, n]) == tot_abs
    a_s[1, 0] = 0xFF
    C, _ = mxfp4.gemm(a_q, a_s, b_q, b_s)
    assert np.isnan(C[1]).all() and not np.isnan(C[[0, 2]]).any()

"""Pins of oracle/mxfp6.py (MXFP6: Table 1 with the conversion of Section 3.3 / Algorithm 1 / Appendix A.1, A.2):
the paper's constants, the library FP8 grids that contain the two 6-bit grids, exact rational arithmetic for the
encoder and the product, closed forms for the scale, bit-level examples for the packing."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import mxfp6
from paper_2506_08027_amd import synth_inputs as si

HERE = os.path.dirname(os.path.abspath(__file__))
FMTS = ["e2m3", "e3m2"]


def _golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "table1_mxfp6.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


@pytest.mark.parametrize("fmt", FMTS)
def test_table_matches_the_paper_constants(fmt):
    g = _golden()
    E, M = mxfp6.FORMATS[fmt]
    assert (E, M) == (g[f"{fmt}_exponent_bits"], g[f"{fmt}_mantissa_bits"]) and E + M == 5
    mags = mxfp6.decode(np.arange(32), fmt)
    assert mags[-1] == g[f"{fmt}_max_normal_significand"] * 2.0 ** g[f"{fmt}_max_normal_exponent"] == mxfp6.dest_max(fmt)
    key = f"{fmt}_min_subnormal_exponent" + ("_by_definition" if fmt == "e3m2" else "")
    assert mags[1] == 2.0 ** g[key] and mags[0] == 0
    assert round(math.log2(mags[-1] / mags[1]), 1) == g[f"{fmt}_binades"]       # the column that decides the E3M2 reading
    assert np.array_equal(mxfp6.decode(np.arange(32) | 32, fmt), -mags) and (np.diff(mags) > 0).all()


@pytest.mark.parametrize("fmt,lib,step", [("e2m3", torch.float8_e4m3fn, 2.0 ** -3), ("e3m2", torch.float8_e5m2, 2.0 ** -4)])
def test_grid_is_the_library_fp8_grid_cut_to_the_format(fmt, lib, step):
    """E2M3 has E4M3's three mantissa bits, E3M2 has E5M2's two: the 6-bit magnitudes are exactly the FP8 values (as
    the library decodes them) that do not exceed the format's maximum and are multiples of its smallest subnormal."""
    fp8 = torch.arange(256, dtype=torch.uint8).view(lib).float().numpy().astype(np.float64)
    fp8 = fp8[np.isfinite(fp8) & (fp8 >= 0)]
    want = np.unique(fp8[(fp8 <= mxfp6.dest_max(fmt)) & (np.round(fp8 / step) == fp8 / step)])
    assert np.array_equal(want, mxfp6.decode(np.arange(32), fmt))


@pytest.mark.parametrize("fmt,lib,lo", [("e2m3", torch.float8_e4m3fn, 1.0), ("e3m2", torch.float8_e5m2, 0.25)])
def test_encoder_against_the_library_cast_in_the_normal_range(fmt, lib, lo):
    """Between the smallest normal and the maximum the 6-bit grid IS the FP8 grid, so RNE must agree with the library's."""
    rng = np.random.default_rng(1)
    top = mxfp6.dest_max(fmt)
    t = np.concatenate([rng.uniform(lo, top, 20000), np.linspace(lo, top, 4097)]).astype(np.float32)
    t = np.concatenate([t, -t])
    got = mxfp6.decode(mxfp6.encode(t.astype(np.float64), fmt), fmt)
    assert np.array_equal(got, torch.from_numpy(t).to(lib).float().numpy().astype(np.float64))


@pytest.mark.parametrize("fmt", FMTS)
def test_encoder_is_round_to_nearest_even_and_saturates(fmt):
    """Exact rationals on a grid that holds every code, every midpoint and points beside them."""
    mags = [Fraction(float(x)) for x in mxfp6.decode(np.arange(32), fmt)]
    grid = [Fraction(k, 256) for k in range(0, 40 * 256 + 1, 1)] if fmt == "e3m2" else [Fraction(k, 256) for k in range(0, 10 * 256 + 1)]
    t = np.array([float(x) for x in grid])
    got = mxfp6.encode(t, fmt)
    for x, c in zip(grid, got):
        d = [abs(x - m) for m in mags]
        best = min(d)
        cands = [i for i, v in enumerate(d) if v == best]
        want = cands[0] if len(cands) == 1 else [i for i in cands if i % 2 == 0][0]
        if x >= mags[-1]:
            want = 31
        assert c == want, (x, c, want)
    assert np.array_equal(mxfp6.encode(-t, fmt), got | 32)                           # sign kept, -0 included
    assert mxfp6.encode(np.array([np.inf, -np.inf, 1e30]), fmt).tolist() == [31, 63, 31]


@pytest.mark.parametrize("fmt", FMTS)
def test_scale_rule_closed_form_and_neighbours(fmt):
    top = mxfp6.dest_max(fmt)
    for k in range(-127, 128, 7):
        a = np.float32(np.ldexp(top, k)) if k < 125 else None
        if a is None or not np.isfinite(a) or float(a) != math.ldexp(top, k):
            continue
        assert mxfp6.scale_byte(float(a), fmt) == k + 127
        assert mxfp6.scale_byte(float(np.nextafter(a, np.float32(0))), fmt) == k + 127
        assert mxfp6.scale_byte(float(np.nextafter(a, np.float32(np.inf))), fmt) == min(k + 128, 254)
        assert mxfp6.scale_byte(float(a) / 2 * (1 + 2.0 ** -20), fmt) == k + 127       # just above the previous boundary
    assert mxfp6.scale_byte(0.0, fmt) == 0 and mxfp6.scale_byte(np.nan, fmt) == 0xFF and mxfp6.scale_byte(np.inf, fmt) == 254
    assert mxfp6.scale_byte(2.0 ** -149, fmt) == 0
    # exact rational ceil(log2(amax / destmax)) on random magnitudes
    rng = np.random.default_rng(2)
    for a in np.exp2(rng.uniform(-120, 120, 300)).astype(np.float32):
        n = int(mxfp6.scale_byte(float(a), fmt)) - 127
        assert Fraction(float(a)) <= Fraction(top) * Fraction(2) ** n and Fraction(float(a)) > Fraction(top) * Fraction(2) ** (n - 1)


def test_packing_bit_order():
    codes = np.zeros((1, 32), np.uint8)
    codes[0, 0], codes[0, 1], codes[0, 2], codes[0, 5], codes[0, 31] = 1, 1, 63, 0b101010, 0b100001
    q = mxfp6.pack(codes)
    assert q.shape == (1, 24)
    assert q[0, 0] == 0x41 and q[0, 1] == 0xF0 and q[0, 2] == 0x03          # bits 0, 6, 12..17
    assert q[0, 3] == 0x80 and q[0, 4] == 0x0A                               # code 5 in bits 30..35
    assert q[0, 23] == 0b10000100                                             # code 31 in bits 186..191
    rng = np.random.default_rng(3)
    c = rng.integers(0, 64, (5, 96)).astype(np.uint8)
    assert np.array_equal(mxfp6.unpack(mxfp6.pack(c)), c)


@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_tightness_round_trip_transpose_and_specials(fmt):
    E, M = mxfp6.FORMATS[fmt]
    x = np.asarray(si.activations(96, 128, seed=2, bf16=False), np.float32)
    x[3, 32:64] = 0.0
    x[3, 33] = -0.0
    q, s = mxfp6.quantize_rowwise(x, fmt)
    assert q.shape == (96, 96) and s.shape == (96, 4)
    codes = mxfp6.unpack(q).reshape(96, 4, 32)
    top = (codes & 31).max(-1)
    amax = np.abs(x).reshape(96, 4, 32).max(-1)
    half = int(mxfp6.encode(np.array(mxfp6.dest_max(fmt) / 2), fmt))
    assert ((top >= half) | (amax == 0)).all()                                  # amax / X lies in (destmax / 2, destmax]
    d = mxfp6.dequantize(q, s, fmt)
    X = np.repeat(np.exp2(s.astype(np.float64) - 127), 32, axis=1)
    top_spacing = 2.0 ** (math.floor(math.log2(mxfp6.dest_max(fmt))) - M)
    assert (np.abs(d - x) <= X * top_spacing / 2).all()                        # half a step of the top binade at worst
    assert np.signbit(d[3, 33]) and not np.signbit(d[3, 32]) and (s[3, 1] == 0)
    qT, sT = mxfp6.quantize_colwise(x, fmt)
    q2, s2 = mxfp6.quantize_rowwise(np.ascontiguousarray(x.T), fmt)
    assert np.array_equal(qT, q2) and np.array_equal(sT, s2)
    bf = si.to_bf16_bits(x)
    assert np.array_equal(mxfp6.quantize_rowwise(bf, fmt)[0], mxfp6.quantize_rowwise(si.bf16_bits_to_f32(bf), fmt)[0])
    y = x[:2].copy()
    y[0, 5], y[0, 40], y[1, 70], y[1, 71] = np.nan, np.inf, -np.inf, 3.0
    q, s = mxfp6.quantize_rowwise(y, fmt)
    c = mxfp6.unpack(q)
    assert s[0, 0] == 0xFF and (c[0, :32] == 0).all() and s[0, 1] == 254 and c[0, 40] == 31 and (c[0, 32:40] & 31 == 0).all()
    assert s[1, 2] == 254 and c[1, 70] == 63 and c[1, 71] == 0
    assert np.isnan(mxfp6.dequantize(q, s, fmt)[0, :32]).all()


@pytest.mark.parametrize("fmt", FMTS)
def test_gemm_is_the_block_scaled_sum_and_reduces_to_the_mxfp8_product(fmt):
    """Brute force in exact rationals on a tiny case; and, since every 6-bit value is an E4M3 value, the product
    equals the MXFP8 oracle's product of the operands re-encoded as E4M3 bytes under the same scales (the route
    the GPU takes)."""
    rng = np.random.default_rng(9)
    M_, N_, K = 3, 4, 64
    a = (rng.standard_normal((M_, K)) * np.exp2(rng.integers(-6, 6, (M_, 1)))).astype(np.float32)
    b = (rng.standard_normal((N_, K)) * 0.05).astype(np.float32)
    (a_q, a_s), (b_q, b_s) = mxfp6.quantize_rowwise(a, fmt), mxfp6.quantize_rowwise(b, fmt)
    C, A = mxfp6.gemm(a_q, a_s, b_q, b_s, fmt)
    ca, cb = mxfp6.unpack(a_q), mxfp6.unpack(b_q)
    val = [Fraction(float(x)) for x in mxfp6.decode(np.arange(64), fmt)]
    for m in range(M_):
        for n in range(N_):
            tot, tot_abs = Fraction(0), Fraction(0)
            for blk in range(K // 32):
                inner = sum(val[int(ca[m, 32 * blk + i])] * val[int(cb[n, 32 * blk + i])] for i in range(32))
                inner_abs = sum(abs(val[int(ca[m, 32 * blk + i])] * val[int(cb[n, 32 * blk + i])]) for i in range(32))
                sc = Fraction(2) ** (int(a_s[m, blk]) + int(b_s[n, blk]) - 254)
                tot += sc * inner
                tot_abs += sc * inner_abs
            assert abs(Fraction(C[m, n]) - tot) <= Fraction(2) ** -45 * tot_abs and Fraction(A[m, n]) == tot_abs
    # expansion to E4M3 bytes: exact, and the MXFP8 oracle then computes the same product
    e4 = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    def expand(q):
        v = mxfp6.decode(mxfp6.unpack(q), fmt)
        by = torch.from_numpy(v.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(e4[by], v)                                        # no rounding happened
        return by
    C8, A8 = oracle.gemm(expand(a_q), a_s, expand(b_q), b_s)
    assert np.allclose(C8, C, rtol=0, atol=1e-13 * A.max()) and np.allclose(A8, A, rtol=1e-13)

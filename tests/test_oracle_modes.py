"""Pins of the oracle's ablation arms (Section 3.1 / Table 1: E5M2 elements; Section 3.3: the OCP v1
scale rule that the recipe replaces). CPU only. The recipe itself is pinned in test_oracle_pins.py."""
import math

import numpy as np
import torch

import oracle
from paper_2506_08027_amd import synth_inputs as si


def test_e5m2_table_matches_paper_constants_and_library_type():
    vals = np.array([oracle.e5m2_decode(c) for c in range(256)])
    finite = vals[np.isfinite(vals)]
    assert finite.max() == 1.75 * 2.0 ** 15 and finite[finite > 0].min() == 2.0 ** -16      # Table 1
    assert abs(math.log2(finite.max() / finite[finite > 0].min()) - 31.8) < 0.01            # binades, Table 1
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e5m2).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(vals), np.isnan(lib))
    assert np.array_equal(vals[~np.isnan(vals)], lib[~np.isnan(lib)])                       # includes +-Inf codes
    assert np.isinf(vals[0x7C]) and np.isinf(vals[0xFC]) and np.isnan(vals[[0x7D, 0x7E, 0x7F]]).all()


def test_e5m2_encoder_is_rne_and_saturates():
    enc = oracle.e5m2_encode
    rng = np.random.default_rng(0)
    grid = np.array([oracle.e5m2_decode(c) for c in range(0x7C)])
    mids = (grid[:-1] + grid[1:]) / 2                                   # every tie point
    t = np.concatenate([grid, mids, np.nextafter(mids, 0), np.nextafter(mids, np.inf),
                        rng.uniform(0, 57344, 4000), 2.0 ** rng.uniform(-18, 16, 4000)])
    t = t[t <= 57344 + 0.0]
    t = np.concatenate([t, -t])
    lib = torch.from_numpy(t.astype(np.float32)).to(torch.float8_e5m2).view(torch.uint8).numpy()
    t32 = t.astype(np.float32).astype(np.float64)
    ours = np.array([enc(x) for x in t32], np.uint8)
    assert np.array_equal(lib, ours)
    for big in (57344.0000001, 61440.0, 65536.0, 1e30, float("inf")):   # the library type overflows to Inf here
        assert enc(big) == 0x7B and enc(-big) == 0xFB
    assert enc(float("nan")) == 0x7F and enc(-0.0) == 0x80 and enc(2.0 ** -17) == 0x00


def test_ocp_rule_closed_form_and_relation_to_the_round_up_rule():
    """OCP v1: n = floor(log2 amax) - emax. The recipe's n is that plus one exactly when the significand of
    amax exceeds the format's top significand 1.75 (Section 3.3: rounding up instead of down)."""
    rng = np.random.default_rng(1)
    for fmt, emax in (("e4m3", 8), ("e5m2", 15)):
        for _ in range(3000):
            e = int(rng.integers(-100, 100))
            m = float(rng.choice([1.0, 1.25, 1.5, 1.75, np.nextafter(1.75, 2), 1.875, np.nextafter(2.0, 1),
                                  1.0 + rng.random()]))
            amax = float(np.float32(m * 2.0 ** e))
            mant, ex = math.frexp(amax)                                  # amax = mant * 2^ex, mant in [0.5, 1)
            floor_log2 = ex - 1
            ocp = oracle.scale_byte_mode(amax, fmt, "ocp") - 127
            up = oracle.scale_byte_mode(amax, fmt, "up") - 127
            assert ocp == floor_log2 - emax
            assert up == ocp + (1 if 2 * mant > 1.75 else 0)
    assert oracle.scale_byte_mode(0.0, "e4m3", "ocp") == 0 and oracle.scale_byte_mode(float("nan"), "e5m2", "ocp") == 255
    assert oracle.scale_byte_mode(2.0 ** -140, "e4m3", "ocp") == 0      # lower clamp
    assert oracle.scale_byte_mode(float("inf"), "e4m3", "ocp") == 254    # upper clamp


def test_recipe_mode_is_byte_identical_to_the_recipe_functions():
    x = si.tiny_with_specials(256, seed=3)
    q, s = oracle.quantize_rowwise(x)
    q2, s2 = oracle.quantize_rowwise_mode(x, "e4m3", "up")
    assert np.array_equal(q, q2) and np.array_equal(s, s2)
    g = np.asarray(si.gradients(64, 512, seed=4, spikes=True), np.float32)
    assert all(np.array_equal(a, b) for a, b in zip(oracle.quantize_rowwise(g), oracle.quantize_rowwise_mode(g)))
    assert np.array_equal(np.nan_to_num(oracle.dequantize_mode(q, s, "e4m3"), nan=-1.0),
                          np.nan_to_num(oracle.dequantize(q, s, "f64"), nan=-1.0))


def test_rounding_the_scale_down_overflows_exactly_where_the_paper_says():
    """Under the OCP rule the block maximum saturates whenever its significand exceeds 1.75 (V/X lands in
    (448, 512)); under the recipe's rule no element of a finite block ever saturates (Section 3.3)."""
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((256, 1024)) * np.exp(rng.standard_normal(1024))).astype(np.float32)
    blocks = np.abs(x.reshape(256, 32, 32))
    amax = blocks.max(-1)
    mant = np.frexp(amax)[0] * 2
    for rule in ("up", "ocp"):
        q, s = oracle.quantize_rowwise_mode(x, "e4m3", rule)
        scaled = np.abs(x.reshape(256, 32, 32)) / np.exp2(s.astype(np.float64) - 127)[..., None]
        over = (scaled > 448).any(-1)
        if rule == "up":
            assert not over.any()
        else:
            assert np.array_equal(over, mant > 1.75)
            assert 0.15 < over.mean() < 0.35                     # a quarter of a binade
            sat = (q.reshape(256, 32, 32) & 0x7F) == 0x7E
            assert (sat.any(-1) >= over).all()


def test_e5m2_row_quantization_end_to_end_against_the_library_cast():
    """The whole E5M2 path (block loop, E5M2 scale maximum, E5M2 encoder together): under Algorithm 1 every
    scaled element lies inside +-57344, where the conversion is the standard round-to-nearest-even cast to
    the OCP E5M2 type; PyTorch's CPU cast of x * 2^-n serves as the independent opinion. The scale byte n is
    checked against its closed form (smallest n with amax <= 57344 * 2^n) in exact rational arithmetic."""
    import torch
    from fractions import Fraction
    rng = np.random.default_rng(21)
    x = (rng.standard_normal((64, 256)) * np.exp(3 * rng.standard_normal((64, 1)))).astype(np.float32)
    x[3, 40:72] = 0.0                                    # a zero block
    x[5, 7] = 57344.0 * 2.0 ** 3                         # amax exactly max * 2^k: not bumped
    x[6, 7] = np.nextafter(np.float32(57344.0 * 2.0 ** 3), np.float32(np.inf))   # one ulp above: bumped
    q, s = oracle.quantize_rowwise_mode(x, "e5m2", "up")
    blocks = x.reshape(64, 8, 32)
    for r in range(64):
        for b in range(8):
            amax = float(np.abs(blocks[r, b]).max())
            n = int(s[r, b]) - 127
            if amax == 0.0:
                assert n == -127
                continue
            assert Fraction(amax) <= Fraction(57344) * Fraction(2) ** n                     # admissible ...
            assert n == -127 or Fraction(amax) > Fraction(57344) * Fraction(2) ** (n - 1)   # ... and the smallest
    scaled = (blocks.astype(np.float64) * np.exp2(127.0 - s.astype(np.float64))[:, :, None]).reshape(64, 256)
    assert np.all(np.abs(scaled) <= 57344.0)
    t = torch.from_numpy(scaled.astype(np.float32))      # exact: a power-of-two scaling inside the FP32 normal range
    assert np.array_equal(t.numpy().astype(np.float64), scaled)
    want = t.to(torch.float8_e5m2).view(torch.uint8).numpy()
    assert np.array_equal(q, want)
    assert int(s[5, 0]) + 1 == int(s[6, 0])


def test_mixed_format_product_against_the_recipe_product_and_brute_force():
    """gemm_mode with E4M3 x E4M3 is the recipe's product (the C triple loop); with an E5M2 operand it is the
    block-scaled double sum written out in exact rationals on a tiny case."""
    from fractions import Fraction
    rng = np.random.default_rng(21)
    a = (rng.standard_normal((5, 96)) * np.exp2(rng.integers(-5, 6, (5, 1)))).astype(np.float32)
    b = (rng.standard_normal((4, 96)) * 0.03).astype(np.float32)
    a4, b4 = oracle.quantize_rowwise(a), oracle.quantize_rowwise(b)
    C0, A0 = oracle.gemm(*a4, *b4)
    C1, A1 = oracle.gemm_mode(a4[0], a4[1], "e4m3", b4[0], b4[1], "e4m3")
    assert np.allclose(C0, C1, rtol=0, atol=1e-14 * A0.max()) and np.allclose(A0, A1, rtol=1e-14)
    a5 = oracle.quantize_rowwise_mode(a, "e5m2")
    for fa, qa, fb, qb in (("e5m2", a5, "e4m3", b4), ("e4m3", a4, "e5m2", oracle.quantize_rowwise_mode(b, "e5m2")), ("e5m2", a5, "e5m2", oracle.quantize_rowwise_mode(b, "e5m2"))):
        C, A = oracle.gemm_mode(qa[0], qa[1], fa, qb[0], qb[1], fb)
        dec = {"e4m3": oracle.e4m3_decode, "e5m2": oracle.e5m2_decode}
        for m in range(5):
            for n in range(4):
                tot = tot_abs = Fraction(0)
                for blk in range(3):
                    inner = inner_abs = Fraction(0)
                    for i in range(32):
                        p = Fraction(dec[fa](int(qa[0][m, 32 * blk + i]))) * Fraction(dec[fb](int(qb[0][n, 32 * blk + i])))
                        inner += p
                        inner_abs += abs(p)
                    sc = Fraction(2) ** (int(qa[1][m, blk]) + int(qb[1][n, blk]) - 254)
                    tot += sc * inner
                    tot_abs += sc * inner_abs
                assert abs(Fraction(C[m, n]) - tot) <= Fraction(2) ** -45 * tot_abs and Fraction(A[m, n]) == tot_abs

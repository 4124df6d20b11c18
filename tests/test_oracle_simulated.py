"""Pins of the oracle's simulated-MX path (Section 3.1: GEMM inputs are cast BF16 -> MXFP8 -> BF16 and an
ordinary BF16 GEMM follows). CPU only."""
from fractions import Fraction

import numpy as np
import torch

import oracle
from paper_2506_08027_amd import synth_inputs as si


def _bits(x):
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _f64(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()


def test_bf16_product_against_library_matmul_on_asymmetric_shapes():
    rng = np.random.default_rng(0)
    a, b = _bits(rng.standard_normal((24, 96))), _bits(rng.standard_normal((40, 96)) * 0.02)
    C, A = oracle.matmul_nt_bf16(a, b)
    ref = _f64(a) @ _f64(b).T                       # a transposed or swapped operand changes the shape or the values
    assert C.shape == (24, 40) and np.allclose(C, ref, rtol=0, atol=1e-13 * np.abs(ref).max())
    assert np.allclose(A, np.abs(_f64(a)) @ np.abs(_f64(b)).T, rtol=1e-13)
    rows = [5, 0, 23, 5]
    Cr, Ar = oracle.matmul_nt_bf16_rows(a, b, rows)
    assert np.array_equal(Cr, C[rows]) and np.array_equal(Ar, A[rows])


def test_bf16_product_exact_rational_and_small_integers():
    rng = np.random.default_rng(1)
    a, b = _bits(rng.standard_normal((3, 64)) * 8), _bits(rng.standard_normal((2, 64)))
    C, A = oracle.matmul_nt_bf16(a, b)
    av, bv = _f64(a), _f64(b)
    for m in range(3):
        for n in range(2):
            exact = sum(Fraction(float(x)) * Fraction(float(y)) for x, y in zip(av[m], bv[n]))
            assert abs(Fraction(float(C[m, n])) - exact) <= Fraction(float(A[m, n])) * Fraction(1, 2 ** 50)
    ia, ib = rng.integers(-8, 9, (16, 128)), rng.integers(-8, 9, (8, 128))
    C, A = oracle.matmul_nt_bf16(_bits(ia), _bits(ib))
    assert np.array_equal(C, (ia @ ib.T).astype(np.float64)) and np.array_equal(A, np.abs(ia) @ np.abs(ib).T)
    onehot = np.zeros((4, 128)); onehot[np.arange(4), [0, 31, 32, 127]] = 1
    C, _ = oracle.matmul_nt_bf16(_bits(onehot), _bits(ib))
    assert np.array_equal(C, ib[:, [0, 31, 32, 127]].T.astype(np.float64))


def test_round_trip_is_idempotent_exact_on_representable_values_and_bounded():
    x = si.activations(64, 256, seed=2)                      # BF16 bit patterns
    y = oracle.roundtrip_bf16(x, "row")
    assert y.shape == x.shape and np.array_equal(oracle.roundtrip_bf16(y, "row"), y)          # a fixed point after one pass
    # amax / X lies in (224, 448], where E4M3 steps by at most 32: no element moves by more than 16 X < amax / 14
    xv, yv = _f64(x).reshape(64, 8, 32), _f64(y).reshape(64, 8, 32)
    amax = np.abs(xv).max(-1, keepdims=True)
    assert (np.abs(yv - xv) <= amax / 14).all() and (np.abs(yv) <= amax * (1 + 1 / 14)).all()
    assert (np.abs(yv - xv) > amax / 64).any()                                               # and the bound is not idle
    # values that are E4M3 codes times a common power of two come back bit for bit
    codes = np.array([oracle.e4m3_decode(c) for c in range(0x7F)])
    rng = np.random.default_rng(3)
    blk = rng.choice(codes, (8, 64)) * rng.choice([-1.0, 1.0], (8, 64))
    blk[:, 0] = 448.0; blk[:, 32] = -448.0                                                   # pins the block scale to 2^0
    for e in (-20, 0, 9):
        src = _bits(blk * 2.0 ** e)
        assert np.array_equal(oracle.roundtrip_bf16(src, "row"), src)
    # column blocks: the transposed round trip of x is the row round trip of x^T
    assert np.array_equal(oracle.roundtrip_bf16(x, "col"), oracle.roundtrip_bf16(np.ascontiguousarray(x.T), "row"))


def test_simulated_product_equals_the_mxfp8_product_of_the_same_operands():
    """Decoding to BF16 loses nothing while Q_i * X stays a normal BF16 number (4 significant bits), so the
    BF16 product of the round-tripped operands is the block-scaled MXFP8 product: two routes through the
    oracle that share only the decode table."""
    xa, xb = si.activations(32, 256, seed=2), si.weights(48, 256, seed=4)
    aq, as_ = oracle.quantize_rowwise(xa)
    bq, bs = oracle.quantize_rowwise(xb)
    C1, A1 = oracle.gemm(aq, as_, bq, bs)
    C2, A2 = oracle.matmul_nt_bf16(oracle.roundtrip_bf16(xa), oracle.roundtrip_bf16(xb))
    assert np.array_equal(C1, C2) and np.array_equal(A1, A2)

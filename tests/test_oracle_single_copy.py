"""Pins of the oracle's single-copy path (Section 5 names the two stored copies per tensor as the overhead to
remove): the column copy derived from the kept row copy. CPU only."""
import numpy as np

import oracle
from paper_2506_08027_amd import synth_inputs as si


def test_values_the_row_copy_holds_exactly_give_the_direct_column_copy():
    """E4M3 codes times one power of two per 32 x 32 patch: the row copy is exact, so deriving the column copy
    from it must give what quantizing the source down its columns gives, byte for byte."""
    rng = np.random.default_rng(0)
    codes = np.array([oracle.e4m3_decode(c) for c in range(0x7F)])
    x = rng.choice(codes, (96, 128)) * rng.choice([-1.0, 1.0], (96, 128))
    x[::32, :] = 448.0                                     # every column block and ...
    x[:, ::32] = -448.0                                    # ... every row block has amax 448: scale 2^0 times the patch's
    patch = 2.0 ** rng.integers(-20, 20, (3, 4))
    x = (x * np.kron(patch, np.ones((32, 32)))).astype(np.float32)
    q, s = oracle.quantize_rowwise(x)
    assert np.array_equal(oracle.dequantize(q, s, "f64"), x.astype(np.float64))
    qT, sT = oracle.requantize_colwise(q, s)
    dT, dsT = oracle.quantize_colwise(x)
    assert np.array_equal(qT, dT) and np.array_equal(sT, dsT)


def test_derived_column_copy_is_the_column_copy_of_the_decoded_tensor_and_costs_one_more_rounding():
    x = np.asarray(si.activations(128, 256, seed=2, bf16=False), np.float32)
    q, s = oracle.quantize_rowwise(x)
    qT, sT = oracle.requantize_colwise(q, s)
    dec = oracle.dequantize(q, s, "f32")
    q2, s2 = oracle.quantize_colwise(np.asarray(dec, np.float32))
    assert np.array_equal(qT, q2) and np.array_equal(sT, s2)
    direct = oracle.dequantize(*oracle.quantize_colwise(x), "f64").T
    derived = oracle.dequantize(qT, sT, "f64").T
    xr = x.astype(np.float64)
    mse = lambda y: float(((y - xr) ** 2).sum() / (xr ** 2).sum())
    # the second rounding adds to the error, by less than a factor of 2.5 in relative MSE, and no element moves
    # by more than one column-copy step plus one row-copy step
    assert mse(direct) < mse(derived) < 2.5 * mse(direct)
    col_amax = np.abs(xr).reshape(4, 32, 256).max(1, keepdims=True).repeat(32, 1).reshape(128, 256)
    row_amax = np.abs(xr).reshape(128, 8, 32).max(2, keepdims=True).repeat(32, 2).reshape(128, 256)
    assert (np.abs(derived - xr) <= (col_amax * (1 + 1 / 14) + row_amax) / 14 + 1e-300).all()


def test_nan_blocks_of_the_row_copy_poison_the_column_blocks_they_touch():
    x = np.asarray(si.weights(64, 64, seed=4, bf16=False), np.float32)
    x[5, 40] = np.nan
    q, s = oracle.quantize_rowwise(x)
    qT, sT = oracle.requantize_colwise(q, s)
    assert (sT[32:64, 0] == 0xFF).all() and (sT[:32, :] != 0xFF).all() and (sT[32:64, 1] != 0xFF).all()
    assert (qT[32:64, :32] == 0x7F).all()

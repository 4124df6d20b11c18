"""Pins of the oracle's grouped (mixture-of-experts, Appendix A.4) products. CPU only."""
import numpy as np
import pytest

import oracle
from paper_2506_08027_amd import synth_inputs as si


def _q(x):
    return oracle.quantize_rowwise(np.asarray(x, np.float32))


def test_grouped_product_is_the_per_expert_product_of_the_decoded_operands():
    rng = np.random.default_rng(0)
    M, N, K, ends = 160, 48, 96, [40, 40, 130, 150]                    # an empty expert; rows 150.. belong to nobody
    a_q, a_s = _q(rng.standard_normal((M, K)))
    w = rng.standard_normal((4, N, K)) * 0.02 * np.array([1, 7, -3, 50]).reshape(4, 1, 1)   # experts differ a lot
    bq, bs = zip(*[_q(w[e]) for e in range(4)])
    C, A = oracle.grouped_gemm(a_q, a_s, np.stack(bq), np.stack(bs), ends)
    a = oracle.dequantize(a_q, a_s)
    start = 0
    for e, end in enumerate(ends):
        b = oracle.dequantize(bq[e], bs[e])
        ref = a[start:end] @ b.T                                        # library matmul on the decoded values
        assert np.allclose(C[start:end], ref, rtol=0, atol=1e-12 * max(np.abs(ref).max(), 1e-30) if end > start else 0)
        assert np.allclose(A[start:end], np.abs(a[start:end]) @ np.abs(b).T, rtol=1e-12)
        start = end
    assert np.isnan(C[150:]).all() and np.isnan(A[150:]).all() and not np.isnan(C[:150]).any()
    # a row moved to another expert changes: the expert index is really used
    C2, _ = oracle.grouped_gemm(a_q, a_s, np.stack(bq), np.stack(bs), [41, 41, 130, 150])
    assert not np.array_equal(C2[40], C[40]) and np.array_equal(C2[41:150], C[41:150]) and np.array_equal(C2[:40], C[:40])


def test_one_group_is_the_plain_product():
    a_q, a_s = _q(si.activations(64, 128, seed=2, bf16=False))
    b_q, b_s = _q(si.weights(32, 128, seed=4, bf16=False))
    C, A = oracle.grouped_gemm(a_q, a_s, b_q[None], b_s[None], [64])
    C1, A1 = oracle.gemm(a_q, a_s, b_q, b_s)
    assert np.array_equal(C, C1) and np.array_equal(A, A1)
    W, WA = oracle.grouped_gemm_wgrad(a_q, a_s, b_q, b_s, [128])
    assert np.array_equal(W[0], C1) and np.array_equal(WA[0], A1)


def test_grouped_weight_gradients_add_up_to_the_ungrouped_one():
    rng = np.random.default_rng(2)
    O, H, T, ends = 24, 40, 256, [64, 64, 160, 256]
    dyT_q, dyT_s = _q(rng.standard_normal((O, T)) * 1e-3)
    xT_q, xT_s = _q(rng.standard_normal((H, T)))
    W, WA = oracle.grouped_gemm_wgrad(dyT_q, dyT_s, xT_q, xT_s, ends)
    full, full_abs = oracle.gemm(dyT_q, dyT_s, xT_q, xT_s)
    assert W.shape == (4, O, H) and (W[1] == 0).all() and (WA[1] == 0).all()
    assert np.allclose(W.sum(0), full, rtol=0, atol=1e-12 * np.abs(full).max()) and np.allclose(WA.sum(0), full_abs, rtol=1e-12)
    a, b = oracle.dequantize(dyT_q, dyT_s), oracle.dequantize(xT_q, xT_s)
    assert np.allclose(W[2], a[:, 64:160] @ b[:, 64:160].T, rtol=0, atol=1e-12 * np.abs(full).max())
    with pytest.raises(ValueError):
        oracle.grouped_gemm_wgrad(dyT_q, dyT_s, xT_q, xT_s, [48, 256])   # a block would straddle two experts

"""GPU parity of the simulated MX path (Section 3.1: BF16 GEMM inputs are converted to MXFP8 and straight
back to BF16, then an ordinary BF16 GEMM with FP32 accumulation follows) against the CPU oracle, and the
cross-check it gives for the MXFP8 product: both routes compute the same sums of the same decoded values.
Calls go through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_08027_amd as mx
from mfma_model import hw_tolerance
from paper_2506_08027_amd import synth_inputs as si

pytestmark = pytest.mark.gpu

# FP32 accumulation in any order: the bound this build aims at for every product (no instruction-specific
# allowance here: the BF16 matrix instruction multiplies exactly and adds in FP32)
TARGET_ELEM = 2.0 ** -20
TARGET_FRO = 1e-5
FRO_BF16 = 3.0e-3


def _dev_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def _host(c):
    torch.cuda.synchronize()
    if c.dtype == torch.bfloat16:
        return si.bf16_bits_to_f32(c.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    return c.cpu().numpy().astype(np.float64)


def _check(got, ref, absref, label, bf16=False, fro_tol=TARGET_FRO):
    fin = np.isfinite(ref)
    assert np.array_equal(np.isnan(got), np.isnan(ref)), f"{label}: NaN pattern"
    err = np.abs(got[fin] - ref[fin])
    bound = TARGET_ELEM * absref[fin] + (np.abs(ref[fin]) * 2.0 ** -8 + 2.0 ** -133 if bf16 else 0.0)
    worst = float((err / np.maximum(absref[fin], 1e-300)).max())
    fro = float(np.linalg.norm(got[fin] - ref[fin]) / max(np.linalg.norm(ref[fin]), 1e-300))
    print(f"[simulated path] {label}: max |err|/sum|ab| = {worst:.3e} (tol {TARGET_ELEM:.3e}), rel Frobenius = {fro:.3e} (tol {fro_tol})")
    assert (err <= bound).all(), f"{label}: per-element bound exceeded, worst {worst:.3e}"
    assert fro <= fro_tol, f"{label}: Frobenius {fro:.3e}"


@pytest.mark.parametrize("shape", [(16, 16, 64), (48, 80, 128), (272, 144, 192), (256, 384, 512), (1, 1, 64), (300, 5, 64),
                                   (7, 513, 128), (512, 512, 256)])
def test_bf16_product_small_integers_bit_exact(shape):
    M, N, K = shape
    rng = np.random.default_rng(M * 1000 + N)
    a, b = rng.integers(-8, 9, (M, K)), rng.integers(-8, 9, (N, K))
    abits, bbits = si.to_bf16_bits(a.astype(np.float32)), si.to_bf16_bits(b.astype(np.float32))
    want = (a @ b.T).astype(np.float64)
    assert np.array_equal(_host(mx.gemm_bf16(_dev_bf16(abits), _dev_bf16(bbits))), want)
    want16 = si.bf16_bits_to_f32(si.to_bf16_bits(want.astype(np.float32))).astype(np.float64)
    assert np.array_equal(_host(mx.gemm_bf16(_dev_bf16(abits), _dev_bf16(bbits), torch.bfloat16)), want16)


def test_bf16_product_one_hot_rows_select_columns():
    """B = one-hot rows at every position of a 64-value step and across steps: C[:, n] must be that column
    of A exactly. Catches any mismatch between the two operands' K order."""
    rng = np.random.default_rng(5)
    K = 192
    a = si.to_bf16_bits(rng.standard_normal((40, K)).astype(np.float32))
    b = np.zeros((K, K), np.float32)
    b[np.arange(K), np.arange(K)] = 1.0
    got = _host(mx.gemm_bf16(_dev_bf16(a), _dev_bf16(si.to_bf16_bits(b))))
    assert np.array_equal(got, si.bf16_bits_to_f32(a).astype(np.float64))


@pytest.mark.parametrize("shape,dtype", [((256, 256, 256), torch.float32), ((200, 136, 192), torch.float32),
                                         ((130, 129, 64), torch.bfloat16), ((384, 256, 4096), torch.float32),
                                         ((2048, 4096, 512), torch.bfloat16), ((2048 + 72, 4096 - 100, 192), torch.float32)])
def test_bf16_product_matches_oracle(shape, dtype):
    """Round-tripped activations x weights: one-tile kernels (ragged), persistent kernels (full tiles), both
    tile configurations, long K."""
    M, N, K = shape
    a, b = oracle.roundtrip_bf16(si.activations(M, K, seed=2)), oracle.roundtrip_bf16(si.weights(N, K, seed=4))
    rows = np.arange(M) if M * N * K <= 2 ** 27 else np.unique(np.concatenate([[0, M - 1], np.random.default_rng(1).integers(0, M, 14)]))
    ref, absref = oracle.matmul_nt_bf16_rows(a, b, rows)
    got = _host(mx.gemm_bf16(_dev_bf16(a), _dev_bf16(b), dtype))[rows]
    bf16 = dtype == torch.bfloat16
    _check(got, ref, absref, f"{M}x{N}x{K} {'bf16' if bf16 else 'f32'} out", bf16, FRO_BF16 if bf16 else TARGET_FRO)


def test_bf16_product_workgroup_bound_and_padded_c_do_not_change_the_result():
    M, N, K = 1024, 1024, 256
    a, b = _dev_bf16(oracle.roundtrip_bf16(si.activations(M, K, seed=2))), _dev_bf16(oracle.roundtrip_bf16(si.weights(N, K, seed=4)))
    full = mx.gemm_bf16(a, b)
    few = mx.gemm_bf16(a, b, max_workgroups=3)
    pad = torch.full((M, N + 8), 7.0, dtype=torch.float32, device="cuda")
    mx.mxfp8_gemm_bf16(a, b, pad[:, :N])
    torch.cuda.synchronize()
    assert torch.equal(full, few) and torch.equal(full, pad[:, :N]) and bool((pad[:, N:] == 7.0).all())


def test_bf16_product_propagates_nan_and_inf():
    rng = np.random.default_rng(9)
    a = rng.standard_normal((64, 128)).astype(np.float32)
    b = rng.standard_normal((64, 128)).astype(np.float32)
    a[3, 17] = np.nan
    a[5, 100] = np.inf
    b[7, 64] = -np.inf
    abits, bbits = si.to_bf16_bits(a), si.to_bf16_bits(b)
    got = _host(mx.gemm_bf16(_dev_bf16(abits), _dev_bf16(bbits)))
    av, bv = si.bf16_bits_to_f32(abits).astype(np.float64), si.bf16_bits_to_f32(bbits).astype(np.float64)
    with np.errstate(invalid="ignore"):
        want = av @ bv.T
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want)) and np.array_equal(np.sign(got[np.isinf(want)]), np.sign(want[np.isinf(want)]))


@pytest.mark.parametrize("axis", ["row", "col"])
def test_round_trip_on_the_gpu_is_the_oracles(axis):
    """quantize -> dequantize to BF16 of the copy a pass uses = the oracle's round trip, bit for bit."""
    x = si.activations(256, 384, seed=2)
    q = mx.quantize(_dev_bf16(x), axis + "wise")
    key = "row" if axis == "row" else "colT"
    y = mx.dequantize(q["q_" + key], q["s_" + key], torch.bfloat16)
    torch.cuda.synchronize()
    assert np.array_equal(y.view(torch.int16).cpu().numpy().view(np.uint16), oracle.roundtrip_bf16(x, axis))


@pytest.mark.parametrize("pass_", ["fprop", "dgrad", "wgrad"])
def test_simulated_layer_product_cross_checks_the_mxfp8_product(pass_):
    """One linear layer (T=512, H=384, O=256) through both routes on the GPU: MXFP8 product of the quantized
    copies vs BF16 product of the same copies decoded to BF16. Both must meet their bound against the oracle
    (which gives ONE reference for both, decoding to BF16 being exact here), and they may differ from each
    other only by what the FP8 matrix instruction loses."""
    T, H, O = 512, 384, 256
    X, W, dY = si.activations(T, H, seed=2), si.weights(O, H, seed=4), si.gradients(T, O, seed=5, spikes=True)
    Xq, Wq = mx.quantize(_dev_bf16(X), "both"), mx.quantize(_dev_bf16(W), "both")
    dYq = mx.quantize(torch.from_numpy(dY).cuda(), "both")
    A, B = {"fprop": ((Xq, "row"), (Wq, "row")), "dgrad": ((dYq, "row"), (Wq, "colT")),
            "wgrad": ((dYq, "colT"), (Xq, "colT"))}[pass_]
    aq, as_, bq, bs = A[0]["q_" + A[1]], A[0]["s_" + A[1]], B[0]["q_" + B[1]], B[0]["s_" + B[1]]
    direct = _host(mx.gemm(pass_, aq, as_, bq, bs))
    a16, b16 = mx.dequantize(aq, as_, torch.bfloat16), mx.dequantize(bq, bs, torch.bfloat16)
    simulated = _host(mx.gemm_bf16(a16, b16))
    h = [t.cpu().numpy() for t in (aq, as_, bq, bs)]
    ref, absref = oracle.gemm(*h)
    ref2, absref2 = oracle.matmul_nt_bf16(a16.view(torch.int16).cpu().numpy().view(np.uint16),
                                          b16.view(torch.int16).cpu().numpy().view(np.uint16))
    assert np.array_equal(ref, ref2) and np.array_equal(absref, absref2)      # one reference for both routes
    _check(simulated, ref, absref, f"simulated {pass_}")
    allowance = hw_tolerance(*h) + 2 * TARGET_ELEM * absref
    diff = np.abs(direct - simulated)
    print(f"[simulated path] {pass_}: max |mxfp8 - simulated|/sum|ab| = {float((diff / np.maximum(absref, 1e-300)).max()):.3e}")
    assert (diff <= allowance).all()


def test_simulated_fprop_at_full_size_on_sampled_rows():
    """The benchmark's fprop shape (8192 x 14336 x 4096) in the launch configuration bench.py times."""
    T, H, O = 8192, 4096, 14336
    X, W = _dev_bf16(si.activations(T, H, seed=2)), _dev_bf16(si.weights(O, H, seed=4))
    Xq, Wq = mx.quantize(X, "rowwise", scale_layout=mx.SCALES_TILED), mx.quantize(W, "rowwise", scale_layout=mx.SCALES_TILED)
    a16 = mx.dequantize(Xq["q_row"], Xq["s_row"], torch.bfloat16, scale_layout=mx.SCALES_TILED)
    b16 = mx.dequantize(Wq["q_row"], Wq["s_row"], torch.bfloat16, scale_layout=mx.SCALES_TILED)
    y = mx.gemm_bf16(a16, b16, torch.bfloat16)
    rows = np.unique(np.concatenate([[0, 255, 256, T - 1], np.random.default_rng(3).integers(0, T, 8)]))
    torch.cuda.synchronize()
    a_host = a16[torch.from_numpy(rows).cuda()].view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(a_host, oracle.roundtrip_bf16(si.activations(T, H, seed=2)[rows]))
    full_a = np.zeros((int(rows.max()) + 1, H), np.uint16)
    full_a[rows] = a_host
    ref, absref = oracle.matmul_nt_bf16_rows(full_a, b16.view(torch.int16).cpu().numpy().view(np.uint16), rows)
    _check(_host(y)[rows], ref, absref, "full-size simulated fprop, BF16 out", bf16=True, fro_tol=FRO_BF16)

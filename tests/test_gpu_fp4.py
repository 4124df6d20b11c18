"""GPU parity of the MXFP4 conversion (Table 1: E2M1 elements; Section 3.3 / Algorithm 1 / Appendix A.1, A.2 with
the E2M1 constants): packed codes and scale bytes must equal the oracle's byte for byte, decoded values bit for
bit. Calls go through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2506_08027_amd as mx
import scale_layout as sl
from oracle import mxfp4
from paper_2506_08027_amd import synth_inputs as si

pytestmark = pytest.mark.gpu


def _dev(a, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16) if bf16 else np.ascontiguousarray(a)).cuda()
    return t.view(torch.bfloat16) if bf16 else t


def _check_quantize(x, bf16, tiled, axis="both"):
    src = si.to_bf16_bits(x) if bf16 else x
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    out = mx.fp4_quantize(_dev(src, bf16), axis, lay)
    torch.cuda.synchronize()
    for key_q, key_s, ref in (("q_row", "s_row", mxfp4.quantize_rowwise), ("q_colT", "s_colT", mxfp4.quantize_colwise)):
        if key_q in out:
            q, s = ref(src)
            assert np.array_equal(out[key_q].cpu().numpy(), q), key_q
            got = out[key_s].cpu().numpy()
            assert np.array_equal(sl.untile(got, *s.shape) if tiled else got, s), key_s


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("tiled", [False, True], ids=["rowmajor", "tiled"])
def test_fp4_quantize_ties_boundaries_and_specials(bf16, tiled):
    _check_quantize(si.fp4_hard_cases(288, 160, seed=11), bf16, tiled)
    _check_quantize(si.tiny_with_specials(256, seed=0), bf16, tiled)


@pytest.mark.parametrize("axis", ["rowwise", "colwise"])
def test_fp4_quantize_llm_shaped_tensors(axis):
    _check_quantize(np.asarray(si.activations(1024, 2048, seed=2, bf16=False), np.float32), True, True, axis)
    _check_quantize(si.gradients(768, 1536, seed=5, spikes=True), False, False, axis)


def test_fp4_quantize_padded_source_rows():
    x = si.fp4_hard_cases(160, 96, seed=12)
    buf = torch.full((160, 128), float("nan"), device="cuda")
    buf[:, :96] = _dev(x)
    out = mx.fp4_quantize(buf[:, :96], "both")
    torch.cuda.synchronize()
    q, s = mxfp4.quantize_rowwise(x)
    qT, sT = mxfp4.quantize_colwise(x)
    assert np.array_equal(out["q_row"].cpu().numpy(), q) and np.array_equal(out["s_row"].cpu().numpy(), s)
    assert np.array_equal(out["q_colT"].cpu().numpy(), qT) and np.array_equal(out["s_colT"].cpu().numpy(), sT)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("tiled", [False, True], ids=["rowmajor", "tiled"])
def test_fp4_dequantize_every_code_and_scale(dtype, tiled):
    rows, cols = 256 + 40, 64
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 16, (rows, cols)).astype(np.uint8)
    codes[:256, :16] = np.arange(16, dtype=np.uint8)[None, :]
    s = rng.integers(0, 256, (rows, cols // 32)).astype(np.uint8)
    s[:256, 0] = np.arange(256, dtype=np.uint8)
    q = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    got = mx.fp4_dequantize(_dev(q), _dev(sl.tile(s, filler=0xFF) if tiled else s), dtype, lay)
    torch.cuda.synchronize()
    want = mxfp4.dequantize(q, s)
    nan = np.isnan(want)
    with np.errstate(over="ignore", under="ignore"):
        w32 = want.astype(np.float32)
    if dtype == torch.bfloat16:
        g = got.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(g[~nan], si.to_bf16_bits(w32)[~nan])
        assert np.isnan(si.bf16_bits_to_f32(g[nan])).all()
    else:
        g = got.cpu().numpy()
        assert np.array_equal(g.view(np.uint32)[~nan], w32.view(np.uint32)[~nan])
        assert np.isnan(g[nan]).all()


def test_fp4_full_size_round_trip_properties():
    """[8192 x 4096] BF16 activations at the size the benchmark times, tiled scales: sampled rows and columns are
    compared with the oracle byte for byte; over the whole tensor every scale is tight (the block's largest
    magnitude code is 3, 4 or 6 unless the block is zero) and decoding loses at most amax / 3 per block."""
    bits = si.activations(8192, 4096, seed=2)
    x = _dev(bits, True)
    lay = mx.SCALES_TILED
    out = mx.fp4_quantize(x, "both", lay)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 63, 64, 4095, 4096, 8191])
    q, s = mxfp4.quantize_rowwise(bits[rows])
    assert np.array_equal(out["q_row"].cpu().numpy()[rows], q)
    assert np.array_equal(sl.untile(out["s_row"].cpu().numpy(), 8192, 128)[rows], s)
    cols = np.array([0, 31, 32, 2047, 4095])
    qT, sT = mxfp4.quantize_rowwise(np.ascontiguousarray(bits[:, cols].T))
    assert np.array_equal(out["q_colT"].cpu().numpy()[cols], qT)
    assert np.array_equal(sl.untile(out["s_colT"].cpu().numpy(), 4096, 256)[cols], sT)
    dec = mx.fp4_dequantize(out["q_row"], out["s_row"], torch.float32, lay)
    xf = x.float()
    amax = xf.view(8192, 128, 32).abs().amax(-1, keepdim=True)
    err = (dec.view(8192, 128, 32) - xf.view(8192, 128, 32)).abs()
    assert bool((err <= amax / 3).all())
    codes = out["q_row"].view(8192, 128, 16)
    top = torch.maximum(codes & 7, (codes >> 4) & 7).amax(-1)
    assert bool(((top >= 5) | (amax.squeeze(-1) == 0)).all())


def test_fp4_error_codes():
    x = torch.zeros((64, 64), device="cuda")
    with pytest.raises(mx.MXFP8Error):
        mx.fp4_quantize(x[:, :48], "both")
    with pytest.raises(mx.MXFP8Error):
        mx.fp4_quantize(x[:40], "both")
    out = mx.fp4_quantize(x[:0], "both")
    assert out["q_row"].numel() == 0


# ---- the MXFP4 product -----------------------------------------------------------------------------------
import os  # noqa: E402

ON_HARDWARE = "MXFP8_HOSTMODEL_LIB" not in os.environ
# Target bound of this build for the products: |err| <= 2^-20 * sum|a_k b_k| per element and relative Frobenius
# error <= 1e-5 (FP32 output) against the exact sum. Products of two E2M1 values have at most 4 significant bits and
# the products of one block pair span less than 8 binades, so the 4-bit form of the matrix instruction has nothing
# to truncate inside a block; what is left is the FP32 accumulation.
FP4_ELEM = 2.0 ** -20
FP4_FRO = 1e-5
FP4_FRO_BF16 = 3.0e-3


def _fp4_operands(M, N, K, seed, spread=8):
    rng = np.random.default_rng(seed)
    a = np.asarray(si.activations(M, K, seed=seed, bf16=False), np.float32)
    b = np.asarray(si.weights(N, K, seed=seed + 1, bf16=False), np.float32)
    if spread:
        a = (a.reshape(M, K // 32, 32) * np.exp2(rng.integers(-spread, spread + 1, (M, K // 32, 1))).astype(np.float32)).reshape(M, K)
        b = (b.reshape(N, K // 32, 32) * np.exp2(rng.integers(-spread, spread + 1, (N, K // 32, 1))).astype(np.float32)).reshape(N, K)
    return mxfp4.quantize_rowwise(a) + mxfp4.quantize_rowwise(b)


def _gpu_fp4_gemm(ops, dtype=torch.float32, tiled=False, wg=0):
    a_q, a_s, b_q, b_s = ops
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    if tiled:
        a_s, b_s = sl.tile(a_s, filler=0xFF), sl.tile(b_s, filler=0xFF)
    c = mx.fp4_gemm("fprop", _dev(a_q), _dev(a_s), _dev(b_q), _dev(b_s), dtype, lay, wg)
    torch.cuda.synchronize()
    if dtype == torch.bfloat16:
        return si.bf16_bits_to_f32(c.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    return c.cpu().numpy().astype(np.float64)


def _compare_fp4(got, ref, absum, bf16, label):
    assert not np.isnan(got).any(), label
    tol = FP4_ELEM * absum + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0) + 1e-300
    err = np.abs(got - ref)
    fro = np.linalg.norm(err) / max(np.linalg.norm(ref), 1e-300)
    print(f"{label}: max err / sum|ab| = 2^{np.log2((err / (absum + 1e-300)).max() + 1e-300):.1f}, Frobenius {fro:.2e}")
    assert (err <= tol).all(), (label, float((err / tol).max()))
    assert fro <= (FP4_FRO_BF16 if bf16 else FP4_FRO), (label, fro)


@pytest.mark.parametrize("shape", [(200, 136, 768), (72, 260, 256), (130, 40, 512), (256, 384, 768), (384, 256, 512), (1, 1, 256)])
@pytest.mark.parametrize("tiled", [False, True], ids=["rowmajor", "tiled"])
def test_fp4_gemm_matches_oracle(shape, tiled):
    """Ragged and full-tile shapes (one workgroup per tile and resident workgroups), FP32 and BF16 output; block
    magnitudes vary by up to 2^16 along every row, so a scale byte paired with the wrong block shows."""
    M, N, K = shape
    ops = _fp4_operands(M, N, K, seed=M + N)
    ref, absum = mxfp4.gemm(*ops)
    _compare_fp4(_gpu_fp4_gemm(ops, torch.float32, tiled), ref, absum, False, f"{shape} f32")
    _compare_fp4(_gpu_fp4_gemm(ops, torch.bfloat16, tiled, wg=2), ref, absum, True, f"{shape} bf16")


@pytest.mark.parametrize("shape", [(48, 80, 256), (272, 144, 512), (256, 256, 1024), (300, 5, 256)])
def test_fp4_gemm_small_integer_operands_are_bit_exact(shape):
    """Operands in {-2, ..., 2}: every code, product and partial sum is a small integer, FP32 adds them exactly."""
    M, N, K = shape
    rng = np.random.default_rng(M * 1000 + N)
    a = rng.integers(-2, 3, (M, K)).astype(np.float32)
    b = rng.integers(-2, 3, (N, K)).astype(np.float32)
    ops = mxfp4.quantize_rowwise(a) + mxfp4.quantize_rowwise(b)
    assert np.array_equal(mxfp4.dequantize(ops[0], ops[1]), a)            # the integers survive the quantization
    got = _gpu_fp4_gemm(ops)
    assert np.array_equal(got, a.astype(np.float64) @ b.astype(np.float64).T)


def test_fp4_gemm_nan_scale_poisons_its_row_only():
    ops = list(_fp4_operands(128, 128, 512, seed=7))
    ops[1] = ops[1].copy()
    ops[1][5, 3] = 0xFF
    got = _gpu_fp4_gemm(ops)
    assert np.isnan(got[5]).all() and not np.isnan(np.delete(got, 5, axis=0)).any()


@pytest.mark.parametrize("tiled", [False, True], ids=["rowmajor", "tiled"])
def test_fp4_gemm_large_tiles(tiled):
    """2048 x 4096 x 1024: the 256 x 256 configuration on resident workgroups, sampled rows against the oracle,
    and the result must not depend on the number of workgroups."""
    M, N, K = 2048, 4096, 1024
    ops = _fp4_operands(M, N, K, seed=77, spread=4)
    got = _gpu_fp4_gemm(ops, torch.float32, tiled)
    rows = np.array([0, 1, 255, 256, 1023, 1024, 2047])
    ref, absum = mxfp4.gemm(ops[0][rows], ops[1][rows], ops[2], ops[3])
    _compare_fp4(got[rows], ref, absum, False, f"large tiled={tiled}")
    assert np.array_equal(got, _gpu_fp4_gemm(ops, torch.float32, tiled, wg=96))


@pytest.mark.skipif(not ON_HARDWARE, reason="full-size problem: hardware only")
def test_fp4_gemm_full_size_end_to_end():
    """The forward product of the benchmark's layer at full size with MXFP4 operands produced by the GPU's own
    quantizer (tiled scales): sampled rows against the oracle's product of the oracle's quantization of the same
    tensors (the GPU copies are byte-exact, see above, so the operands are the same bytes)."""
    M, N, K = 8192, 14336, 4096          # the shape and scale layout the benchmark times
    xb, wb = si.activations(M, K, seed=2), si.weights(N, K, seed=4)
    lay = mx.SCALES_TILED
    xq = mx.fp4_quantize(_dev(xb, True), "rowwise", lay)
    wq = mx.fp4_quantize(_dev(wb, True), "rowwise", lay)
    c = mx.fp4_gemm("fprop", xq["q_row"], xq["s_row"], wq["q_row"], wq["s_row"], torch.float32, lay)
    torch.cuda.synchronize()
    rows = np.array([0, 77, 4095, 4096, 8191])
    a_q, a_s = mxfp4.quantize_rowwise(xb[rows])
    b_q, b_s = mxfp4.quantize_rowwise(wb)
    ref, absum = mxfp4.gemm(a_q, a_s, b_q, b_s)
    _compare_fp4(c[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64), ref, absum, False, "full size")

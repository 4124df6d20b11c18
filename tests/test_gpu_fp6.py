"""GPU parity of MXFP6 (Table 1: E2M3 and E3M2 elements; Section 3.3 / Algorithm 1 / Appendix A.1, A.2 with the 6-bit
constants): packed codes and scale bytes must equal the oracle's byte for byte, decoded values bit for bit, the
expansion to E4M3 must be exact, and the product of expanded operands must be the MXFP6 product. Calls go through
the C ABI."""
import os

import numpy as np
import pytest
import torch

import paper_2506_08027_amd as mx
import scale_layout as sl
from oracle import mxfp6
from paper_2506_08027_amd import synth_inputs as si

pytestmark = pytest.mark.gpu
ON_HARDWARE = "MXFP8_HOSTMODEL_LIB" not in os.environ
FMTS = [("e2m3", mx.E2M3), ("e3m2", mx.E3M2)]
E4M3 = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)


def _dev(a, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16) if bf16 else np.ascontiguousarray(a)).cuda()
    return t.view(torch.bfloat16) if bf16 else t


def _check_quantize(x, fmt, element, bf16, tiled, axis="both"):
    src = si.to_bf16_bits(x) if bf16 else x
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    out = mx.fp6_quantize(_dev(src, bf16), element, axis, lay)
    torch.cuda.synchronize()
    for key_q, key_s, ref in (("q_row", "s_row", mxfp6.quantize_rowwise), ("q_colT", "s_colT", mxfp6.quantize_colwise)):
        if key_q in out:
            q, s = ref(src, fmt)
            assert np.array_equal(out[key_q].cpu().numpy(), q), key_q
            got = out[key_s].cpu().numpy()
            assert np.array_equal(sl.untile(got, *s.shape) if tiled else got, s), key_s


@pytest.mark.parametrize("fmt,element", FMTS)
@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("tiled", [False, True], ids=["rowmajor", "tiled"])
def test_fp6_quantize_ties_boundaries_and_specials(fmt, element, bf16, tiled):
    _check_quantize(si.fp6_hard_cases(288, 160, seed=11, top=mxfp6.dest_max(fmt)), fmt, element, bf16, tiled)
    _check_quantize(si.tiny_with_specials(256, seed=0), fmt, element, bf16, tiled)


@pytest.mark.parametrize("fmt,element", FMTS)
@pytest.mark.parametrize("axis", ["rowwise", "colwise"])
def test_fp6_quantize_llm_shaped_tensors(fmt, element, axis):
    _check_quantize(np.asarray(si.activations(1024, 2048, seed=2, bf16=False), np.float32), fmt, element, True, True, axis)
    _check_quantize(si.gradients(768, 1536, seed=5, spikes=True), fmt, element, False, False, axis)


def _all_codes_operand(rows, cols, seed):
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, 64, (rows, cols)).astype(np.uint8)
    codes[:256, :64] = np.arange(64, dtype=np.uint8)[None, :]
    s = rng.integers(0, 256, (rows, cols // 32)).astype(np.uint8)
    s[:256, 0] = np.arange(256, dtype=np.uint8)
    return mxfp6.pack(codes), s


@pytest.mark.parametrize("fmt,element", FMTS)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("tiled", [False, True], ids=["rowmajor", "tiled"])
def test_fp6_dequantize_every_code_and_scale(fmt, element, dtype, tiled):
    q, s = _all_codes_operand(256 + 40, 96, 5)
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    got = mx.fp6_dequantize(_dev(q), _dev(sl.tile(s, filler=0xFF) if tiled else s), element, dtype, lay)
    torch.cuda.synchronize()
    want = mxfp6.dequantize(q, s, fmt)
    nan = np.isnan(want)
    with np.errstate(over="ignore", under="ignore"):
        w32 = want.astype(np.float32)
    if dtype == torch.bfloat16:
        g = got.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(g[~nan], si.to_bf16_bits(w32)[~nan]) and np.isnan(si.bf16_bits_to_f32(g[nan])).all()
    else:
        g = got.cpu().numpy()
        assert np.array_equal(g.view(np.uint32)[~nan], w32.view(np.uint32)[~nan]) and np.isnan(g[nan]).all()


@pytest.mark.parametrize("fmt,element", FMTS)
def test_fp6_expansion_to_e4m3_is_exact(fmt, element):
    q, _ = _all_codes_operand(256 + 8, 96, 6)
    by = mx.fp6_expand(_dev(q), element).cpu().numpy()
    want = mxfp6.decode(mxfp6.unpack(q), fmt)
    assert np.array_equal(E4M3[by], want) and np.array_equal(np.signbit(E4M3[by]), np.signbit(want))


def _operands(M, N, K, fa, fb, seed):
    rng = np.random.default_rng(seed)
    a = np.asarray(si.activations(M, K, seed=seed, bf16=False), np.float32)
    b = np.asarray(si.weights(N, K, seed=seed + 1, bf16=False), np.float32)
    a = (a.reshape(M, K // 32, 32) * np.exp2(rng.integers(-4, 5, (M, K // 32, 1))).astype(np.float32)).reshape(M, K)
    return mxfp6.quantize_rowwise(a, fa) + mxfp6.quantize_rowwise(b, fb)


@pytest.mark.parametrize("fa,ea,fb,eb", [("e2m3", 0, "e2m3", 0), ("e3m2", 1, "e3m2", 1), ("e2m3", 0, "e3m2", 1)])
@pytest.mark.parametrize("shape,tiled", [((200, 136, 384), False), ((256, 384, 512), True)])
def test_fp6_gemm_is_the_mxfp6_product(fa, ea, fb, eb, shape, tiled):
    """The GPU product of the GPU-expanded operands (i) equals, bit for bit, the GPU's MXFP8 product of the same
    operands expanded on the CPU by a library cast (the expansion kernel adds nothing of its own) and (ii) is the
    oracle's MXFP6 product to the accuracy of the MXFP8 matrix instruction (its in-group truncation, the bound the
    MXFP8 product tests use: Frobenius <= 1e-4)."""
    M, N, K = shape
    a_q, a_s, b_q, b_s = _operands(M, N, K, fa, fb, seed=M + N)
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    sa, sb = (sl.tile(a_s, filler=0xFF), sl.tile(b_s, filler=0xFF)) if tiled else (a_s, b_s)
    got = mx.fp6_gemm("fprop", _dev(a_q), _dev(sa), ea, _dev(b_q), _dev(sb), eb, torch.float32, lay)

    def cpu_expand(q, fmt):
        v = mxfp6.decode(mxfp6.unpack(q), fmt)
        return torch.from_numpy(v.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()

    same = mx.gemm("fprop", _dev(cpu_expand(a_q, fa)), _dev(sa), _dev(cpu_expand(b_q, fb)), _dev(sb), torch.float32, lay)
    torch.cuda.synchronize()
    assert torch.equal(got, same)
    ref, absum = mxfp6.gemm(a_q, a_s, b_q, b_s, fa, fb)
    g = got.cpu().numpy().astype(np.float64)
    err = np.abs(g - ref)
    assert (err <= 2.0 ** -10 * absum + 1e-300).all()
    assert np.linalg.norm(err) / np.linalg.norm(ref) <= 1e-4


@pytest.mark.parametrize("fmt,element", FMTS)
def test_fp6_gemm_small_integer_operands_are_bit_exact(fmt, element):
    rng = np.random.default_rng(4)
    a = rng.integers(-3, 4, (144, 256)).astype(np.float32)
    b = rng.integers(-3, 4, (80, 256)).astype(np.float32)
    (a_q, a_s), (b_q, b_s) = mxfp6.quantize_rowwise(a, fmt), mxfp6.quantize_rowwise(b, fmt)
    assert np.array_equal(mxfp6.dequantize(a_q, a_s, fmt), a)
    got = mx.fp6_gemm("fprop", _dev(a_q), _dev(a_s), element, _dev(b_q), _dev(b_s), element).cpu().numpy()
    assert np.array_equal(got.astype(np.float64), a.astype(np.float64) @ b.astype(np.float64).T)


@pytest.mark.skipif(not ON_HARDWARE, reason="full-size tensor: hardware only")
@pytest.mark.parametrize("fmt,element", FMTS)
def test_fp6_full_size_samples_and_properties(fmt, element):
    """[8192 x 4096] BF16 activations, tiled scales: sampled rows and columns byte for byte against the oracle; over
    the whole tensor decoding loses at most half a top-binade step per block."""
    bits = si.activations(8192, 4096, seed=2)
    x = _dev(bits, True)
    lay = mx.SCALES_TILED
    out = mx.fp6_quantize(x, element, "both", lay)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 63, 64, 4095, 4096, 8191])
    q, s = mxfp6.quantize_rowwise(bits[rows], fmt)
    assert np.array_equal(out["q_row"].cpu().numpy()[rows], q)
    assert np.array_equal(sl.untile(out["s_row"].cpu().numpy(), 8192, 128)[rows], s)
    cols = np.array([0, 31, 32, 2047, 4095])
    qT, sT = mxfp6.quantize_rowwise(np.ascontiguousarray(bits[:, cols].T), fmt)
    assert np.array_equal(out["q_colT"].cpu().numpy()[cols], qT)
    assert np.array_equal(sl.untile(out["s_colT"].cpu().numpy(), 4096, 256)[cols], sT)
    dec = mx.fp6_dequantize(out["q_row"], out["s_row"], element, torch.float32, lay)
    xf = x.float()
    amax = xf.view(8192, 128, 32).abs().amax(-1, keepdim=True)
    err = (dec.view(8192, 128, 32) - xf.view(8192, 128, 32)).abs()
    M = mxfp6.FORMATS[fmt][1]
    assert bool((err <= amax * 2.0 ** -M).all())        # half a step of the top binade <= X * 2^(emax - M - 1) < amax * 2^-M


@pytest.mark.skipif(not ON_HARDWARE, reason="full-size problem: hardware only")
def test_fp6_gemm_full_size_end_to_end():
    """The forward product of the benchmark's layer at full size and in its launch configuration (tiled scales): X in
    E2M3 and W in E3M2 from the GPU's own quantizer, expanded on the GPU, multiplied by the MXFP8 kernel; sampled rows
    against the oracle's MXFP6 product of the oracle's quantization of the same tensors."""
    M, N, K = 8192, 14336, 4096
    xb, wb = si.activations(M, K, seed=2), si.weights(N, K, seed=4)
    lay = mx.SCALES_TILED
    xq = mx.fp6_quantize(_dev(xb, True), mx.E2M3, "rowwise", lay)
    wq = mx.fp6_quantize(_dev(wb, True), mx.E3M2, "rowwise", lay)
    c = mx.fp6_gemm("fprop", xq["q_row"], xq["s_row"], mx.E2M3, wq["q_row"], wq["s_row"], mx.E3M2, torch.float32, lay)
    torch.cuda.synchronize()
    rows = np.array([0, 77, 4095, 4096, 8191])
    a_q, a_s = mxfp6.quantize_rowwise(xb[rows], "e2m3")
    b_q, b_s = mxfp6.quantize_rowwise(wb, "e3m2")
    assert np.array_equal(xq["q_row"].cpu().numpy()[rows], a_q)
    ref, absum = mxfp6.gemm(a_q, a_s, b_q, b_s, "e2m3", "e3m2")
    got = c[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    err = np.abs(got - ref)
    assert (err <= 2.0 ** -10 * absum + 1e-300).all() and np.linalg.norm(err) / np.linalg.norm(ref) <= 1e-4


def test_fp6_error_codes():
    x = torch.zeros((64, 64), device="cuda")
    with pytest.raises(mx.MXFP8Error):
        mx.fp6_quantize(x[:, :48], mx.E2M3, "both")
    with pytest.raises(mx.MXFP8Error):
        mx.fp6_quantize(x, 2, "both")
    assert mx.fp6_quantize(x[:0], mx.E3M2, "both")["q_row"].numel() == 0

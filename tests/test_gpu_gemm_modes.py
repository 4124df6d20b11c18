"""GPU parity of the MXFP8 product with per-operand element formats (Section 3.2.2: E4M3 or E5M2 for weights,
activations and gradients) against the oracle's product of the operands decoded with their own tables. Calls go
through the C ABI. Accuracy is that of the FP8 matrix instruction (its in-group truncation, see test_gpu_gemm.py): the
element bound here is the loose envelope 2^-10 * sum|a b|, the Frobenius bound the 1e-4 of the E4M3 product; what
these tests add is that each format field reaches the right operand."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2506_08027_amd as mx
import scale_layout as sl
from paper_2506_08027_amd import synth_inputs as si

pytestmark = pytest.mark.gpu
ON_HARDWARE = "MXFP8_HOSTMODEL_LIB" not in os.environ
FMT = {mx.E4M3: "e4m3", mx.E5M2: "e5m2"}
COMBOS = [(mx.E5M2, mx.E4M3), (mx.E4M3, mx.E5M2), (mx.E5M2, mx.E5M2), (mx.E4M3, mx.E4M3)]


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _operands(M, N, K, ea, eb, seed):
    a = np.asarray(si.activations(M, K, seed=seed, bf16=False), np.float32)
    b = np.asarray(si.weights(N, K, seed=seed + 1, bf16=False), np.float32)
    return oracle.quantize_rowwise_mode(a, FMT[ea]) + oracle.quantize_rowwise_mode(b, FMT[eb])


def _gpu(ops, ea, eb, dtype=torch.float32, tiled=False, wg=0):
    a_q, a_s, b_q, b_s = ops
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    if tiled:
        a_s, b_s = sl.tile(a_s, filler=0xFF), sl.tile(b_s, filler=0xFF)
    c = mx.gemm_mode("fprop", _dev(a_q), _dev(a_s), ea, _dev(b_q), _dev(b_s), eb, dtype, lay, wg)
    torch.cuda.synchronize()
    if dtype == torch.bfloat16:
        return si.bf16_bits_to_f32(c.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    return c.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("ea,eb", COMBOS, ids=["e5m2xe4m3", "e4m3xe5m2", "e5m2xe5m2", "e4m3xe4m3"])
@pytest.mark.parametrize("shape,tiled", [((200, 136, 384), False), ((256, 384, 512), True)])
def test_gemm_modes_match_oracle(ea, eb, shape, tiled):
    M, N, K = shape
    ops = _operands(M, N, K, ea, eb, seed=M + N)
    ref, absum = oracle.gemm_mode(ops[0], ops[1], FMT[ea], ops[2], ops[3], FMT[eb])
    got = _gpu(ops, ea, eb, torch.float32, tiled)
    err = np.abs(got - ref)
    assert (err <= 2.0 ** -10 * absum + 1e-300).all()
    assert np.linalg.norm(err) / np.linalg.norm(ref) <= 1e-4
    if ea != eb:   # the same bytes with the two format fields swapped are another product, far outside the bound
        wrong, _ = oracle.gemm_mode(ops[0], ops[1], FMT[eb], ops[2], ops[3], FMT[ea])
        with np.errstate(invalid="ignore"):
            assert (~(np.abs(got - wrong) <= 2.0 ** -10 * absum)).mean() > 0.5      # NaN (a code the other table reads as NaN) counts as different
    got16 = _gpu(ops, ea, eb, torch.bfloat16, tiled, wg=2)
    assert (np.abs(got16 - ref) <= 2.0 ** -10 * absum + 2.0 ** -8 * np.abs(ref) + 1e-300).all()
    if ea == mx.E4M3 and eb == mx.E4M3:
        same = mx.gemm("fprop", _dev(ops[0]), _dev(sl.tile(ops[1], filler=0xFF) if tiled else ops[1]), _dev(ops[2]),
                       _dev(sl.tile(ops[3], filler=0xFF) if tiled else ops[3]), torch.float32, mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR)
        assert np.array_equal(same.cpu().numpy().astype(np.float64), got)


@pytest.mark.parametrize("ea,eb", COMBOS[:3], ids=["e5m2xe4m3", "e4m3xe5m2", "e5m2xe5m2"])
def test_gemm_modes_small_integer_operands_are_bit_exact(ea, eb):
    rng = np.random.default_rng(31)
    a = rng.integers(-3, 4, (144, 256)).astype(np.float32)
    b = rng.integers(-3, 4, (80, 256)).astype(np.float32)
    ops = oracle.quantize_rowwise_mode(a, FMT[ea]) + oracle.quantize_rowwise_mode(b, FMT[eb])
    assert np.array_equal(oracle.dequantize_mode(ops[0], ops[1], FMT[ea]), a)
    assert np.array_equal(_gpu(ops, ea, eb), a.astype(np.float64) @ b.astype(np.float64).T)


def test_gemm_modes_gradient_in_e5m2_end_to_end():
    """The ablation's arm at layer size: dY quantized to E5M2 by the GPU's own quantizer, W in E4M3, the activation
    gradient dX = dY . W (dgrad operands: row copy of dY, column copy of W), sampled rows against the oracle."""
    T, H, O = (8192, 4096, 14336) if ON_HARDWARE else (256, 128, 256)
    dy = torch.from_numpy(si.gradients(T, O, seed=3, spikes=True)).cuda()
    w = torch.from_numpy(si.weights(O, H, seed=4).view(np.int16)).cuda().view(torch.bfloat16)
    lay = mx.SCALES_TILED
    dyq = mx.quantize(dy, "rowwise", lay, element=mx.E5M2)
    wq = mx.quantize(w, "colwise", lay)
    dx = mx.gemm_mode("dgrad", dyq["q_row"], dyq["s_row"], mx.E5M2, wq["q_colT"], wq["s_colT"], mx.E4M3, torch.float32, lay)
    torch.cuda.synchronize()
    rows = np.array([0, 1, T // 2, T - 1])
    a_q, a_s = oracle.quantize_rowwise_mode(dy.cpu().numpy()[rows], "e5m2")
    assert np.array_equal(dyq["q_row"].cpu().numpy()[rows], a_q)
    b_q, b_s = oracle.quantize_colwise(w.view(torch.int16).cpu().numpy().view(np.uint16))
    ref, absum = oracle.gemm_mode(a_q, a_s, "e5m2", b_q, b_s, "e4m3")
    got = dx.cpu().numpy()[rows].astype(np.float64)
    err = np.abs(got - ref)
    assert (err <= 2.0 ** -10 * absum + 1e-300).all() and np.linalg.norm(err) / np.linalg.norm(ref) <= 1e-4

"""GPU parity of the grouped (mixture-of-experts, Appendix A.4) product against the CPU oracle and against the
plain product applied expert by expert. Calls go through the C ABI."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2506_08027_amd as mx
import scale_layout as sl
from mfma_model import hw_tolerance
from paper_2506_08027_amd import synth_inputs as si

pytestmark = pytest.mark.gpu
TARGET_ELEM = 2.0 ** -20


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _operands(M, N, K, E, seed):
    a_q, a_s = oracle.quantize_rowwise(np.asarray(si.activations(M, K, seed=seed, bf16=False), np.float32))
    gains = [1.0, -6.0, 0.25, 40.0, 3.0, -0.5, 9.0, 1.5]
    b = [oracle.quantize_rowwise(np.asarray(si.weights(N, K, seed=seed + 1 + e, bf16=False) * gains[e % 8], np.float32))
         for e in range(E)]
    return a_q, a_s, np.stack([q for q, _ in b]), np.stack([s for _, s in b])


def _run(ops, ends, dtype=torch.float32, tiled=False, wg=0):
    a_q, a_s, b_q, b_s = ops
    if tiled:
        a_s = sl.tile(a_s, filler=0xFF)
        b_s = np.concatenate([sl.tile(s, filler=0xFF).ravel() for s in b_s])
    c = mx.gemm_grouped("fprop", _dev(a_q), _dev(a_s), _dev(b_q), _dev(b_s), _dev(np.asarray(ends, np.int32)), dtype,
                        mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR, wg)
    torch.cuda.synchronize()
    if dtype == torch.bfloat16:
        return si.bf16_bits_to_f32(c.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    return c.cpu().numpy().astype(np.float64)


def _check(got, ops, ends, label, bf16=False):
    ref, absref = oracle.grouped_gemm(*ops, ends)
    owned = ~np.isnan(ref)
    assert np.isnan(got[~owned]).all(), f"{label}: rows without an expert were written"
    assert not np.isnan(got[owned]).any(), f"{label}: rows of an expert were not written"
    a_q, a_s, b_q, b_s = ops
    tol = np.zeros_like(ref)
    start = 0
    for e, end in enumerate(ends):
        if end > start:
            tol[start:end] = hw_tolerance(a_q, a_s, b_q[e], b_s[e], rows=np.arange(start, end))
        start = end
    bound = tol + TARGET_ELEM * np.nan_to_num(absref) + (np.abs(np.nan_to_num(ref)) * 2.0 ** -8 + 2.0 ** -133 if bf16 else 0.0)
    err = np.abs(got - ref)
    worst = float((err[owned] / np.maximum(absref[owned], 1e-300)).max())
    print(f"[grouped] {label}: max |err|/sum|ab| = {worst:.3e}")
    assert (err[owned] <= bound[owned]).all(), f"{label}: worst {worst:.3e}"


@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_grouped_small_problem_matches_oracle(tiled, dtype):
    """Experts that end inside a tile, an empty expert, rows that belong to nobody, a last tile crossing the end of A."""
    M, N, K = (384, 256, 256) if tiled else (300, 256, 384)
    ends = [64, 192, 192, 320] if tiled else [70, 70, 200, 290]
    ops = _operands(M, N, K, len(ends), seed=40)
    for wg in (0, 2):
        _check(_run(ops, ends, dtype, tiled, wg), ops, ends, f"{M}x{N}x{K} tiled={tiled} wg={wg}", dtype == torch.bfloat16)


def test_grouped_bad_ends_are_clamped_and_no_expert_writes_nothing():
    M, N, K = 200, 128, 256
    ops = _operands(M, N, K, 3, seed=50)
    _check(_run(ops, [150, 90, 5000]), ops, [150, 150, 200], "ends clamped on the device")
    assert np.isnan(_run(ops, [0, 0, 0])).all()


@pytest.mark.parametrize("tiled", [False, True])
def test_grouped_equals_the_plain_product_expert_by_expert(tiled):
    """256x256 tiles: 8 experts over 4096 tokens. Every output element goes through the same sequence of matrix
    instructions as in the plain product of its expert's rows, so the two agree bit for bit; the oracle is
    compared on sampled rows."""
    M, N, K, E = 4096, 2048, 512, 8
    rng = np.random.default_rng(7)
    cuts = np.sort(rng.integers(0, M // 64, E - 1)) * 64 if tiled else np.sort(rng.integers(0, M - 100, E - 1))
    ends = [int(x) for x in cuts] + [M - (0 if tiled else 37)]
    ops = _operands(M, N, K, E, seed=60)
    got = _run(ops, ends, torch.float32, tiled)
    a_q, a_s, b_q, b_s = ops
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    start = 0
    for e, end in enumerate(ends):
        if end > start:
            rows = slice(start, end)
            as_e, bs_e = (sl.tile(a_s[rows], filler=0xFF), sl.tile(b_s[e], filler=0xFF)) if tiled else (a_s[rows], b_s[e])
            plain = mx.gemm("fprop", _dev(a_q[rows]), _dev(as_e), _dev(b_q[e]), _dev(bs_e), torch.float32, lay)
            torch.cuda.synchronize()
            assert np.array_equal(got[rows], plain.cpu().numpy().astype(np.float64)), f"expert {e}"
        start = end
    assert np.isnan(got[ends[-1]:]).all()
    sample = np.unique(np.concatenate([[0, ends[0] - 1 if ends[0] else 0, ends[-1] - 1], rng.integers(0, ends[-1], 6)]))
    expert_of = np.searchsorted(np.asarray(ends), sample, side="right")
    for i, m in enumerate(sample):
        e = int(expert_of[i])
        ref, absref = oracle.gemm_rows(a_q, a_s, b_q[e], b_s[e], [m])
        tol = hw_tolerance(a_q, a_s, b_q[e], b_s[e], rows=[m]) + TARGET_ELEM * absref
        assert (np.abs(got[m] - ref[0]) <= tol[0]).all(), f"row {m} of expert {e}"


def test_grouped_dgrad_roles():
    """dX = dY_row . W_e_colT^T: A = gradients quantized along rows, B_e = expert weights quantized down their
    columns and stored transposed [H x O]."""
    T, H, O, E = 256, 128, 256, 2
    dY = si.gradients(T, O, seed=5, spikes=True)
    W = [np.asarray(si.weights(O, H, seed=20 + e, bf16=False), np.float32) for e in range(E)]
    a_q, a_s = oracle.quantize_rowwise(dY)
    bT = [oracle.quantize_colwise(w) for w in W]                     # [H x O] each
    ops = (a_q, a_s, np.stack([q for q, _ in bT]), np.stack([s for _, s in bT]))
    ends = [100, 256]
    c = mx.gemm_grouped("dgrad", _dev(ops[0]), _dev(ops[1]), _dev(ops[2]), _dev(ops[3]), _dev(np.asarray(ends, np.int32)))
    torch.cuda.synchronize()
    _check(c.cpu().numpy().astype(np.float64), ops, ends, "dgrad 256x128x256")


@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_grouped_wgrad_matches_oracle_and_the_plain_product_of_each_slice(tiled, dtype):
    """dW_e = dY_colT[:, tokens of e] . X_colT[:, tokens of e]^T: experts with 0, 1, 2 and 3 K steps, ragged M and N.
    Also bit-identical to the plain product of the sliced operands."""
    M, N, K = 200, 136, 768
    ends = [128, 128, 384, 768]
    a_q, a_s = oracle.quantize_rowwise(si.gradients(M, K, seed=5, spikes=True))
    b_q, b_s = oracle.quantize_rowwise(np.asarray(si.activations(N, K, seed=2, bf16=False), np.float32))
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    t = (lambda x: sl.tile(x, filler=0xFF)) if tiled else (lambda x: x)
    c = mx.gemm_grouped("wgrad", _dev(a_q), _dev(t(a_s)), _dev(b_q), _dev(t(b_s)), _dev(np.asarray(ends, np.int32)), dtype, lay)
    torch.cuda.synchronize()
    bf16 = dtype == torch.bfloat16
    got = (si.bf16_bits_to_f32(c.view(torch.int16).cpu().numpy().view(np.uint16)) if bf16 else c.cpu().numpy()).astype(np.float64)
    ref, absref = oracle.grouped_gemm_wgrad(a_q, a_s, b_q, b_s, ends)
    start = 0
    for e, end in enumerate(ends):
        if end == start:
            assert (got[e] == 0).all()
        else:
            sl_q, sl_s = slice(start, end), slice(start // 32, end // 32)
            ops = (np.ascontiguousarray(a_q[:, sl_q]), np.ascontiguousarray(a_s[:, sl_s]),
                   np.ascontiguousarray(b_q[:, sl_q]), np.ascontiguousarray(b_s[:, sl_s]))
            tol = hw_tolerance(*ops) + TARGET_ELEM * absref[e] + (np.abs(ref[e]) * 2.0 ** -8 + 2.0 ** -133 if bf16 else 0.0)
            assert (np.abs(got[e] - ref[e]) <= tol).all(), f"expert {e}"
            plain = mx.gemm("wgrad", _dev(ops[0]), _dev(t(ops[1])), _dev(ops[2]), _dev(t(ops[3])), dtype, lay)
            torch.cuda.synchronize()
            assert torch.equal(c[e].view(torch.int16 if bf16 else torch.int32), plain.view(torch.int16 if bf16 else torch.int32)), f"expert {e}"
        start = end


@pytest.mark.skipif("MXFP8_HOSTMODEL_LIB" in os.environ, reason="full size: GPU only")
def test_grouped_wgrad_full_size_moe_layer_against_sliced_products():
    """The weight gradient of the same layer (16384 tokens, 8 experts, 14336 x 4096 each, FP32 out, tiled scales):
    bit-identical to the plain product of the sliced, re-quantized-free operands for sampled experts; oracle on
    sampled rows of one expert."""
    T, H, O, E = 16384, 4096, 14336, 8
    lay = mx.SCALES_TILED
    g = torch.Generator(device="cuda")
    g.manual_seed(9)
    x = torch.randn((T, H), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    dy = (1e-3 * torch.randn((T, O), generator=g, device="cuda", dtype=torch.float32)).to(torch.bfloat16)
    xq, dyq = mx.quantize(x, "colwise"), mx.quantize(dy, "colwise")            # row-major scales: sliceable on the host side
    ends = np.array([1536, 4096, 4096, 7808, 9984, 12032, 14976, 16384], np.int32)
    tile = lambda s: torch.from_numpy(sl.tile(s.cpu().numpy(), filler=0xFF)).cuda()
    dw = mx.gemm_grouped("wgrad", dyq["q_colT"], tile(dyq["s_colT"]), xq["q_colT"], tile(xq["s_colT"]), _dev(ends), torch.float32, lay)
    torch.cuda.synchronize()
    assert (dw[2] == 0).all()
    for e in (0, 3):
        k0, k1 = (int(ends[e - 1]) if e else 0), int(ends[e])
        a_q, b_q = dyq["q_colT"][:, k0:k1].contiguous(), xq["q_colT"][:, k0:k1].contiguous()
        a_s, b_s = dyq["s_colT"][:, k0 // 32:k1 // 32].contiguous(), xq["s_colT"][:, k0 // 32:k1 // 32].contiguous()
        plain = mx.gemm("wgrad", a_q, tile(a_s), b_q, tile(b_s), torch.float32, lay)
        torch.cuda.synchronize()
        assert torch.equal(dw[e].view(torch.int32), plain.view(torch.int32)), f"expert {e}"
        if e == 3:
            rows = [0, 255, 256, O - 1]
            h = [v.cpu().numpy() for v in (a_q, a_s, b_q, b_s)]
            ref, absref = oracle.gemm_rows(*h, rows)
            tol = hw_tolerance(*h, rows=rows) + TARGET_ELEM * absref
            assert (np.abs(dw[e][rows].cpu().numpy().astype(np.float64) - ref) <= tol).all()


@pytest.mark.skipif("MXFP8_HOSTMODEL_LIB" in os.environ, reason="full size: GPU only")
def test_grouped_full_size_moe_layer_on_sampled_rows():
    """16384 routed tokens, 8 experts, 4096 -> 14336 (the benchmark's expert shape), tiled scales, BF16 out, in the
    launch configuration bench.py times: bit-identical to the plain product per expert on sampled experts,
    oracle on sampled rows."""
    T, H, O, E = 16384, 4096, 14336, 8
    lay = mx.SCALES_TILED
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    x = torch.randn((T, H), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    xq = mx.quantize(x, "rowwise", scale_layout=lay)
    wq, ws = [], []
    for e in range(E):
        w = (0.02 * torch.randn((O, H), generator=g, device="cuda", dtype=torch.float32)).to(torch.bfloat16)
        q = mx.quantize(w, "rowwise", scale_layout=lay)
        wq.append(q["q_row"]); ws.append(q["s_row"])
    b_q, b_s = torch.stack(wq), torch.cat(ws)
    ends = np.array([1536, 4096, 4096, 7808, 9984, 12032, 14976, 16384], np.int32)
    y = mx.gemm_grouped("fprop", xq["q_row"], xq["s_row"], b_q, b_s, _dev(ends), torch.bfloat16, lay)
    torch.cuda.synchronize()
    x_rm = mx.quantize(x, "rowwise")                                  # row-major scales for slicing rows on the host side
    assert torch.equal(x_rm["q_row"], xq["q_row"])
    for e in (0, 3, 7):
        rows = slice(int(ends[e - 1]) if e else 0, int(ends[e]))
        xe = mx.quantize(x[rows].contiguous(), "rowwise", scale_layout=lay)
        plain = mx.gemm("fprop", xe["q_row"], xe["s_row"], wq[e], ws[e], torch.bfloat16, lay)
        torch.cuda.synchronize()
        assert torch.equal(y[rows].view(torch.int16), plain.view(torch.int16)), f"expert {e}"
    a_q, a_s = x_rm["q_row"].cpu().numpy(), x_rm["s_row"].cpu().numpy()
    yh = si.bf16_bits_to_f32(y.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    for m in (0, 1535, 1536, 4095, 4096, 16383):
        e = int(np.searchsorted(ends, m, side="right"))
        bq_h = wq[e].cpu().numpy()
        bs_h = sl.untile(ws[e].cpu().numpy(), O, H // 32)
        ref, absref = oracle.gemm_rows(a_q, a_s, bq_h, bs_h, [m])
        tol = hw_tolerance(a_q, a_s, bq_h, bs_h, rows=[m]) + TARGET_ELEM * absref + np.abs(ref) * 2.0 ** -8
        assert (np.abs(yh[m] - ref[0]) <= tol[0]).all(), f"row {m} of expert {e}"

"""The BF16 product of the simulated MX path (Section 3.1) on the CPU execution model of the kernels:
same kernels as the MXFP8 product with BF16 operands and no scale requests, so what needs proving before a
GPU run is that every DMA source and LDS destination stays in range with rows of 2 K bytes, that the wait
counts still fit the smaller number of requests per step, and that the fragment layout feeds the BF16 matrix
instruction consistently for both operands."""
import numpy as np
import pytest

import oracle
from paper_2506_08027_amd import synth_inputs as si
from test_host_model import MODES, hostmodel, put, run_case  # noqa: F401  (hostmodel is a fixture)


def _operands(M, N, K, seed):
    """BF16 bit patterns of round-tripped activations and weights (what the simulated path multiplies)."""
    return oracle.roundtrip_bf16(si.activations(M, K, seed=seed)), oracle.roundtrip_bf16(si.weights(N, K, seed=seed + 1))


def _case(tmp_path, M, N, K, ops, bf16=False, ldc=None, tag="", wg=0):
    ldc = ldc or N
    names = [put(tmp_path, f"{n}{tag}.bin", v) for n, v in (("a", ops[0]), ("b", ops[1]))]
    out = str(tmp_path / f"c{tag}.bin")
    return f"gemmbf16 {M} {N} {K} {'bf16' if bf16 else 'f32'} {ldc} {' '.join(names)} {out}" + (f" wg={wg}" if wg else ""), out


def _check(out, M, N, ldc, ops, bf16, expect_full=True):
    n = (M - 1) * ldc + N
    if bf16:
        raw = np.full(M * ldc, 0xA5A5, np.uint16)
        raw[:n] = np.fromfile(out, np.uint16)
        raw = raw.reshape(M, ldc)
        written, val = raw[:, :N] != 0xA5A5, si.bf16_bits_to_f32(raw[:, :N])
        assert (raw[:, N:] == 0xA5A5).all()
    else:
        raw = np.full(M * ldc, 0xA5A5A5A5, np.uint32)
        raw[:n] = np.fromfile(out, np.uint32)
        raw = raw.reshape(M, ldc)
        written, val = raw[:, :N] != 0xA5A5A5A5, raw[:, :N].view(np.float32)
        assert (raw[:, N:] == 0xA5A5A5A5).all()
    if expect_full:
        assert written.all()
    rows = np.unique(np.nonzero(written)[0])
    assert rows.size
    ref, absum = oracle.matmul_nt_bf16_rows(ops[0], ops[1], rows)
    # the modelled instruction rounds once per instruction: two per 64-value K step
    tol = max(ops[0].shape[1] // 32, 2) * 2.0 ** -24 * absum + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0) + 1e-300
    w = written[rows]
    err = np.abs(val[rows].astype(np.float64) - ref)
    assert not np.isnan(val[rows][w]).any(), "NaN in C: a tile was read before its loads were waited for"
    assert (err[w] <= tol[w]).all(), float((err[w] / tol[w]).max())
    return int(written.sum())


@pytest.mark.parametrize("mode", [MODES[0], MODES[3]], ids=["lazy-up", "eager-down"])
def test_bf16_gemm_small_tiles_ragged(hostmodel, tmp_path, mode):
    """One workgroup per tile: ragged in M and N, K of one, two and three 64-value steps, padded C."""
    lines, checks = [], []
    for i, (M, N, K, bf16, ldc) in enumerate([(200, 136, 192, False, 136), (130, 129, 64, True, 136), (64, 200, 128, False, 204)]):
        ops = _operands(M, N, K, seed=10 + i)
        line, out = _case(tmp_path, M, N, K, ops, bf16, ldc, tag=str(i))
        lines.append(line)
        checks.append((out, M, N, ldc, ops, bf16))
    _, calls = run_case(hostmodel, tmp_path, lines, **mode)
    assert [c[0] for c in calls] == [0, 0, 0]
    for c in checks:
        _check(*c)


@pytest.mark.parametrize("mode", [MODES[0], MODES[3]], ids=["lazy-up", "eager-down"])
def test_bf16_gemm_persistent_small_tiles(hostmodel, tmp_path, mode):
    """Full tiles: workgroups that walk over 3, 2 and 1 tiles of 128x128, K of 2 and 3 steps."""
    for i, (M, N, K, bf16, wgs) in enumerate([(256, 384, 192, False, 2), (256, 384, 128, True, 4), (384, 256, 192, False, 0)]):
        ops = _operands(M, N, K, seed=80 + i)
        line, out = _case(tmp_path, M, N, K, ops, bf16, tag=str(i), wg=wgs)
        _, calls = run_case(hostmodel, tmp_path, [line], **mode)
        assert calls[0] == (0, list(range(wgs or 6)))
        _check(out, M, N, N, ops, bf16)


@pytest.mark.parametrize("order", ["up", "down"])
def test_bf16_gemm_persistent_large_tiles_sampled_workgroups(hostmodel, tmp_path, order):
    """256x256 configuration: 128 tiles on 64 workgroups (2 tiles each), first and last workgroup."""
    M, N, K = 2048, 4096, 192
    ops = _operands(M, N, K, seed=90)
    line, out = _case(tmp_path, M, N, K, ops, bf16=True, wg=64)
    _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_BLOCKS=2, WAVESIM_ORDER=order)
    assert calls[0] == (0, [0, 63])
    assert _check(out, M, N, N, ops, True, expect_full=False) == 4 * 256 * 256


def test_bf16_gemm_large_tiles_ragged_sampled_workgroups(hostmodel, tmp_path):
    M, N, K = 2048 + 72, 4096 - 100, 192
    ops = _operands(M, N, K, seed=20)
    line, out = _case(tmp_path, M, N, K, ops, bf16=False)
    _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_BLOCKS=4)
    assert calls[0] == (0, [0, 47, 95, 143])
    assert 2 * 256 * 256 < _check(out, M, N, N, ops, False, expect_full=False) <= 4 * 256 * 256


def test_bf16_gemm_validation(hostmodel, tmp_path):
    ops = _operands(64, 64, 64, seed=1)
    bad_k, _ = _case(tmp_path, 64, 64, 32, (ops[0][:, :32], ops[1][:, :32]), tag="k")      # K not a multiple of 64
    small_ld, _ = _case(tmp_path, 64, 64, 64, ops, ldc=32, tag="l")
    _, calls = run_case(hostmodel, tmp_path, [bad_k, small_ld])
    assert [c[0] for c in calls] == [2, 2]                                                 # MXFP8_ERR_SHAPE

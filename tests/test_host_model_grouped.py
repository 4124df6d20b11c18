"""The grouped (mixture-of-experts, Appendix A.4) product on the CPU execution model of the kernels: the
persistent kernel finds its tiles from group ends that live in device memory, experts end in partial tiles,
and rows past the end of A are clamped. What needs proving before a GPU run: no DMA source leaves A, B or the
scale operands for any placement of the group ends (including ends the caller got wrong), every row of every
expert is written exactly once with that expert's B, and rows that belong to no expert are left alone."""
import numpy as np
import pytest

import oracle
import scale_layout as sl
from paper_2506_08027_amd import synth_inputs as si
from test_host_model import MODES, hostmodel, put, run_case  # noqa: F401  (hostmodel is a fixture)


def _operands(M, N, K, E, seed):
    a = oracle.quantize_rowwise(np.asarray(si.activations(M, K, seed=seed, bf16=False), np.float32))
    gains = [1.0, -6.0, 0.25, 40.0, 3.0, -0.5, 9.0, 1.5]
    b = [oracle.quantize_rowwise(np.asarray(si.weights(N, K, seed=seed + 1 + e, bf16=False) * gains[e % 8], np.float32))
         for e in range(E)]
    return a[0], a[1], np.stack([q for q, _ in b]), np.stack([s for _, s in b])


def _case(tmp_path, M, N, K, ops, ends, bf16=False, ldc=None, tag="", tiled=False, wg=0):
    a_q, a_s, b_q, b_s = ops
    ldc = ldc or N
    if tiled:
        a_s = sl.tile(a_s, filler=0xFF)
        b_s = np.concatenate([sl.tile(s, filler=0xFF).ravel() for s in b_s])
    names = [put(tmp_path, f"{n}{tag}.bin", v) for n, v in (("aq", a_q), ("as", a_s), ("bq", b_q), ("bs", b_s),
                                                               ("ends", np.asarray(ends, np.int32)))]
    out = str(tmp_path / f"c{tag}.bin")
    return (f"gemmgrp {M} {N} {K} {'bf16' if bf16 else 'f32'} {ldc} {len(ends)} {' '.join(names)} {out}"
            + (" tiled" if tiled else "") + (f" wg={wg}" if wg else "")), out


def _check(out, M, N, ldc, ops, ends, bf16, expect_full=True):
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
    clamped, prev = [], 0
    for e in ends:                                   # what the kernel makes of the ends: clamped to [previous, M]
        prev = min(max(int(e), prev), M)
        clamped.append(prev)
    ref, absum = oracle.grouped_gemm(*ops, clamped)
    owned = ~np.isnan(ref)
    assert not written[~owned].any(), "a row that belongs to no expert was written"
    if expect_full:
        assert written[owned].all()
    w = written & owned
    assert w.any()
    tol = max(ops[0].shape[1] // 128, 2) * 2.0 ** -24 * absum + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0) + 1e-300
    assert not np.isnan(val[w]).any(), "NaN in C: a tile was read before its loads were waited for"
    err = np.abs(val.astype(np.float64) - ref)
    assert (err[w] <= tol[w]).all(), float((err[w] / tol[w]).max())
    return int(w.sum())


@pytest.mark.parametrize("mode,tiled", [(MODES[0], False), (MODES[3], False), (MODES[0], True)], ids=["lazy-up", "eager-down", "tiled"])
def test_grouped_small_tiles_partial_and_empty_experts(hostmodel, tmp_path, mode, tiled):
    """128x128 tiles on a 3-unit device (workgroups walk over several tiles): experts that end inside a tile, an
    empty expert, a last expert whose tile crosses the end of A, rows that belong to nobody."""
    M, N, K = (384, 256, 256) if tiled else (300, 256, 384)
    ends = [64, 192, 192, 320] if tiled else [70, 70, 200, 290]
    ops = _operands(M, N, K, len(ends), seed=40)
    for i, (bf16, wg) in enumerate([(False, 0), (True, 2)]):
        line, out = _case(tmp_path, M, N, K, ops, ends, bf16, tag=str(i), tiled=tiled, wg=wg)
        _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_CUS=3, **mode)
        assert calls[0] == (0, list(range(wg or 3)))
        _check(out, M, N, N, ops, ends, bf16)


def test_grouped_more_workgroups_than_tiles_and_bad_ends(hostmodel, tmp_path):
    """The host cannot count the tiles: surplus workgroups must leave at once. Ends that decrease or exceed M are
    clamped on the device instead of sending a load out of A."""
    M, N, K = 200, 128, 256
    ops = _operands(M, N, K, 3, seed=50)
    for i, ends in enumerate([[10, 20, 30], [150, 90, 5000], [0, 0, 0]]):
        line, out = _case(tmp_path, M, N, K, ops, ends, tag=str(i))
        _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_CUS=5)
        assert calls[0][0] == 0
        if any(ends):
            _check(out, M, N, N, ops, ends, False)
        else:
            assert (np.fromfile(out, np.uint32) == 0xA5A5A5A5).all()


@pytest.mark.parametrize("tiled", [False, True])
def test_grouped_large_tiles_sampled_workgroups(hostmodel, tmp_path, tiled):
    """256x256 configuration: 8 experts over 2048 tokens, 64 workgroups, first and last one simulated."""
    M, N, K = 2048, 4096, 256
    ends = [256, 640, 640, 1024, 1216, 1600, 1984, 2048] if tiled else [250, 600, 600, 1001, 1200, 1610, 1990, 2040]
    ops = _operands(M, N, K, len(ends), seed=60)
    line, out = _case(tmp_path, M, N, K, ops, ends, bf16=True, tiled=tiled, wg=64)
    _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_BLOCKS=2)
    assert calls[0] == (0, [0, 63])
    assert _check(out, M, N, N, ops, ends, True, expect_full=False) > 2 * 128 * 256


def test_grouped_validation(hostmodel, tmp_path):
    ops = _operands(128, 128, 256, 2, seed=1)
    ok, _ = _case(tmp_path, 128, 128, 256, ops, [64, 128], tag="ok")
    bad_n = ok.replace("gemmgrp 128 128 256", "gemmgrp 128 96 256")
    _, calls = run_case(hostmodel, tmp_path, [bad_n], expect_ok=False)
    assert not calls or calls[0][0] == 2


# ---- weight-gradient form: the experts split the reduction axis ----------------------------------------------
def _wgrad_case(tmp_path, M, N, K, ops, ends, bf16=False, ldc=None, tag="", tiled=False):
    a_q, a_s, b_q, b_s = ops
    ldc = ldc or N
    if tiled:
        a_s, b_s = sl.tile(a_s, filler=0xFF), sl.tile(b_s, filler=0xFF)
    names = [put(tmp_path, f"{n}{tag}.bin", v) for n, v in (("aq", a_q), ("as", a_s), ("bq", b_q), ("bs", b_s),
                                                               ("ends", np.asarray(ends, np.int32)))]
    out = str(tmp_path / f"c{tag}.bin")
    return (f"gemmgrpk {M} {N} {K} {'bf16' if bf16 else 'f32'} {ldc} {len(ends)} {' '.join(names)} {out}"
            + (" tiled" if tiled else "")), out


def _wgrad_check(out, M, N, ldc, ops, ends, bf16):
    E = len(ends)
    n = (E * M - 1) * ldc + N
    dt, fill = (np.uint16, 0xA5A5) if bf16 else (np.uint32, 0xA5A5A5A5)
    raw = np.full(E * M * ldc, fill, dt)
    raw[:n] = np.fromfile(out, dt)
    raw = raw.reshape(E, M, ldc)
    assert (raw[:, :, N:] == fill).all(), "bytes between rows of C were written"
    val = (si.bf16_bits_to_f32(raw[:, :, :N]) if bf16 else raw[:, :, :N].view(np.float32)).astype(np.float64)
    K = ops[0].shape[1]
    clamped, prev = [], 0
    for e in ends:
        prev = min(max(int(e), prev), K)
        clamped.append(prev)
    ref, absum = oracle.grouped_gemm_wgrad(*ops, clamped)
    tol = max(K // 128, 2) * 2.0 ** -24 * absum + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0) + 1e-300
    assert not np.isnan(val).any()
    assert (np.abs(val - ref) <= tol).all(), float((np.abs(val - ref) / tol).max())
    for e in range(E):
        if clamped[e] == (clamped[e - 1] if e else 0):
            assert (val[e] == 0).all()


@pytest.mark.parametrize("mode,tiled", [(MODES[0], False), (MODES[3], True)], ids=["lazy-up-rowmajor", "eager-down-tiled"])
def test_grouped_wgrad_small_tiles(hostmodel, tmp_path, mode, tiled):
    """Experts with 0, 1, 2 and 3 K steps, ragged M and N, padded C, FP32 and BF16 output."""
    M, N, K = 200, 136, 768
    ends = [128, 128, 384, 768]
    a = oracle.quantize_rowwise(si.gradients(M, K, seed=5, spikes=True))
    b = oracle.quantize_rowwise(np.asarray(si.activations(N, K, seed=2, bf16=False), np.float32))
    ops = (a[0], a[1], b[0], b[1])
    for i, (bf16, ldc) in enumerate([(False, 136), (True, 144)]):
        line, out = _wgrad_case(tmp_path, M, N, K, ops, ends, bf16, ldc, tag=str(i), tiled=tiled)
        _, calls = run_case(hostmodel, tmp_path, [line], **mode)
        assert calls[0] == (0, list(range(4 * 2 * 2)))
        _wgrad_check(out, M, N, ldc, ops, ends, bf16)


def test_grouped_wgrad_bad_ends_are_clamped(hostmodel, tmp_path):
    M, N, K = 64, 64, 512
    a = oracle.quantize_rowwise(si.gradients(M, K, seed=6))
    b = oracle.quantize_rowwise(np.asarray(si.activations(N, K, seed=3, bf16=False), np.float32))
    ops = (a[0], a[1], b[0], b[1])
    line, out = _wgrad_case(tmp_path, M, N, K, ops, [256, 128, 9999])
    _, calls = run_case(hostmodel, tmp_path, [line])
    assert calls[0][0] == 0
    _wgrad_check(out, M, N, N, ops, [256, 128, 9999], False)

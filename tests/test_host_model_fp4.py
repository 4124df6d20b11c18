"""The MXFP4 quantizer and decoder (Table 1: E2M1 elements) on the CPU execution model of the kernels: byte-exact
against the oracle for ragged multi-tile shapes, both axes, both scale layouts, padded sources, every rounding tie
and every scale boundary, with AddressSanitizer watching the accesses."""
import numpy as np
import pytest

import scale_layout as sl
from oracle import mxfp4
from paper_2506_08027_amd import synth_inputs as si
from test_host_model import SENTINEL, _compare_scales, get, hostmodel, put, run_case  # noqa: F401  (hostmodel is a fixture)


def _check_quantize(hostmodel, tmp_path, x, bf16, axis, tiled, ld=None, **env):
    rows, cols = x.shape
    src = si.to_bf16_bits(x) if bf16 else x
    ld = ld or cols
    padded = np.full((rows, ld), 0x7FC0 if bf16 else np.nan, src.dtype)
    padded[:, :cols] = src
    flat = padded.ravel()[:(rows - 1) * ld + cols]
    line = (f"quantfp4 {'bf16' if bf16 else 'f32'} {rows} {cols} {ld} {axis} {put(tmp_path, 'src.bin', flat)} {tmp_path / 'o'}"
            + (" tiled" if tiled else ""))
    _, calls = run_case(hostmodel, tmp_path, [line], **env)
    assert calls[0][0] == 0
    if axis & 1:
        q, s = mxfp4.quantize_rowwise(src)
        assert np.array_equal(get(str(tmp_path / "o.q_row"), np.uint8, q.shape), q)
        _compare_scales(str(tmp_path / "o.s_row"), s, tiled)
    if axis & 2:
        q, s = mxfp4.quantize_colwise(src)
        assert np.array_equal(get(str(tmp_path / "o.q_colT"), np.uint8, q.shape), q)
        _compare_scales(str(tmp_path / "o.s_colT"), s, tiled)


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("tiled", [False, True], ids=["rowmajor", "tiled"])
def test_fp4_quantize_ties_boundaries_and_specials(hostmodel, tmp_path, bf16, tiled):
    x = si.fp4_hard_cases(288, 160, seed=11)                       # 3 x 2 tiles, ragged in both directions
    _check_quantize(hostmodel, tmp_path, x, bf16, 3, tiled)


@pytest.mark.parametrize("axis", [1, 2])
def test_fp4_quantize_single_axis_padded_source(hostmodel, tmp_path, axis):
    x = si.fp4_hard_cases(160, 96, seed=12)
    _check_quantize(hostmodel, tmp_path, x, False, axis, False, ld=100)
    _check_quantize(hostmodel, tmp_path, x, True, axis, True, ld=104)


def test_fp4_quantize_tiny_with_specials(hostmodel, tmp_path):
    x = si.tiny_with_specials(256, seed=0)
    _check_quantize(hostmodel, tmp_path, x, False, 3, False)


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("tiled", [False, True], ids=["rowmajor", "tiled"])
def test_fp4_dequantize_every_code_and_scale(hostmodel, tmp_path, bf16, tiled):
    """All 16 codes under all 256 scale bytes, then random operands: FP32 output is the exact value (or the
    FP32 rounding of it below 2^-126), BF16 output its RNE."""
    rows, cols, ld = 256 + 40, 64, 72
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 16, (rows, cols)).astype(np.uint8)
    codes[:256, :16] = np.arange(16, dtype=np.uint8)[None, :]
    s = rng.integers(0, 256, (rows, cols // 32)).astype(np.uint8)
    s[:256, 0] = np.arange(256, dtype=np.uint8)
    q = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    s_file = sl.tile(s, filler=0xFF) if tiled else s
    out = str(tmp_path / "d.bin")
    line = (f"dequantfp4 {rows} {cols} {'bf16' if bf16 else 'f32'} {ld} {put(tmp_path, 'q.bin', q)} {put(tmp_path, 's.bin', s_file)} {out}"
            + (" tiled" if tiled else ""))
    _, calls = run_case(hostmodel, tmp_path, [line])
    assert calls[0][0] == 0
    want = mxfp4.dequantize(q, s)
    n = (rows - 1) * ld + cols
    if bf16:
        raw = np.full(rows * ld, SENTINEL * 0x0101, np.uint16)
        raw[:n] = np.fromfile(out, np.uint16)
        raw = raw.reshape(rows, ld)
        assert (raw[:, cols:] == SENTINEL * 0x0101).all()
        with np.errstate(over="ignore", under="ignore"):
            ref = si.to_bf16_bits(want.astype(np.float32))          # FP32 holds every decoded value exactly or subnormally
        got = raw[:, :cols]
    else:
        raw = np.full(rows * ld, SENTINEL * 0x01010101, np.uint32)
        raw[:n] = np.fromfile(out, np.uint32)
        raw = raw.reshape(rows, ld)
        assert (raw[:, cols:] == SENTINEL * 0x01010101).all()
        with np.errstate(over="ignore", under="ignore"):
            ref = want.astype(np.float32).view(np.uint32)
        got = raw[:, :cols]
    nan = np.isnan(want)
    assert np.array_equal(got[~nan], ref[~nan])
    g = got[nan]
    assert ((g & (0x7F80 if bf16 else 0x7F800000)) == (0x7F80 if bf16 else 0x7F800000)).all() and \
           ((g & (0x7F if bf16 else 0x7FFFFF)) != 0).all()

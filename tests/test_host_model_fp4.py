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


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
def test_fp4_quantize_resident_grid_walks_over_several_tiles(hostmodel, tmp_path, bf16):
    """One compute unit: two workgroups, three tiles each, the next tile's loads in registers while a tile is converted."""
    x = si.fp4_hard_cases(288, 160, seed=13)
    _check_quantize(hostmodel, tmp_path, x, bf16, 3, bf16, WAVESIM_CUS=1)


@pytest.mark.parametrize("rows,cols", [(64, 96), (96, 288), (288, 96), (160, 544), (288, 320)],
                         ids=["1x1", "1x3", "3x1", "2x5", "3x3"])
def test_fp4_quantize_every_tile_of_small_and_odd_grids(hostmodel, tmp_path, rows, cols):
    """Tile grids (rows x columns of 128 x 128 tiles) of one tile, one row, one column and odd counts, on two resident
    workgroups: every tile must come out once, whatever order the workgroups take them in."""
    x = si.fp4_hard_cases(rows, cols, seed=rows + cols)
    _check_quantize(hostmodel, tmp_path, x, True, 3, True, WAVESIM_CUS=1)


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


# ---- the MXFP4 product -----------------------------------------------------------------------------------
from test_host_model import MODES  # noqa: E402


def _fp4_operands(M, N, K, seed):
    """Quantized activations x weights whose blocks differ in magnitude by up to 2^16, so that every scale byte of
    a row differs from its neighbours: a scale byte paired with the wrong block shows."""
    rng = np.random.default_rng(seed)
    a = np.asarray(si.activations(M, K, seed=seed, bf16=False), np.float32)
    b = np.asarray(si.weights(N, K, seed=seed + 1, bf16=False), np.float32)
    a = (a.reshape(M, K // 32, 32) * np.exp2(rng.integers(-8, 9, (M, K // 32, 1))).astype(np.float32)).reshape(M, K)
    b = (b.reshape(N, K // 32, 32) * np.exp2(rng.integers(-8, 9, (N, K // 32, 1))).astype(np.float32)).reshape(N, K)
    return mxfp4.quantize_rowwise(a) + mxfp4.quantize_rowwise(b)


def _fp4_gemm_case(tmp_path, M, N, K, ops, bf16=False, ldc=None, tag="", tiled=False, wg=0):
    a_q, a_s, b_q, b_s = ops
    ldc = ldc or N
    if tiled:
        a_s, b_s = sl.tile(a_s, filler=0xFF), sl.tile(b_s, filler=0xFF)
    names = [put(tmp_path, f"{n}{tag}.bin", v) for n, v in (("aq", a_q), ("as", a_s), ("bq", b_q), ("bs", b_s))]
    out = str(tmp_path / f"c{tag}.bin")
    return (f"gemmfp4 0 {M} {N} {K} {'bf16' if bf16 else 'f32'} {ldc} {' '.join(names)} {out}"
            + (" tiled" if tiled else "") + (f" wg={wg}" if wg else "")), out


def _check_fp4_gemm(out, M, N, ldc, ops, bf16, expect_full=True):
    a_q, a_s, b_q, b_s = ops
    n = (M - 1) * ldc + N
    dt, fill = (np.uint16, 0xA5A5) if bf16 else (np.uint32, 0xA5A5A5A5)
    raw = np.full(M * ldc, fill, dt)
    raw[:n] = np.fromfile(out, dt)
    raw = raw.reshape(M, ldc)
    assert (raw[:, N:] == fill).all(), "bytes between rows of C were written"
    written = raw[:, :N] != fill
    val = (si.bf16_bits_to_f32(raw[:, :N]) if bf16 else raw[:, :N].view(np.float32)).astype(np.float64)
    if expect_full:
        assert written.all()
    rows = np.unique(np.nonzero(written)[0])
    assert rows.size
    ref, absum = mxfp4.gemm(a_q[rows], a_s[rows], b_q, b_s)
    steps = max(a_q.shape[1] * 2 // 128, 2)                       # one rounding per matrix instruction
    tol = steps * 2.0 ** -24 * absum + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0) + 1e-300
    w = written[rows]
    assert not np.isnan(val[rows][w]).any(), "NaN in C: a tile was read before its loads were waited for"
    err = np.abs(val[rows] - ref)
    assert (err[w] <= tol[w]).all(), float((err[w] / tol[w]).max())
    return int(written.sum())


@pytest.mark.parametrize("mode,tiled", [(MODES[0], False), (MODES[3], True), (MODES[1], True), (MODES[2], False)],
                         ids=["lazy-up-rowmajor", "eager-down-tiled", "eager-up-tiled", "lazy-down-rowmajor"])
def test_fp4_gemm_small_tiles_ragged(hostmodel, tmp_path, mode, tiled):
    """One workgroup per tile: ragged M and N, 1, 2 and 3 K steps, FP32 and BF16 output, padded and unaligned C."""
    for i, (M, N, K, bf16, ldc) in enumerate([(200, 136, 768, False, 136), (72, 260, 256, True, 264), (130, 40, 512, True, 41)]):
        ops = _fp4_operands(M, N, K, seed=20 + i)
        line, out = _fp4_gemm_case(tmp_path, M, N, K, ops, bf16, ldc, tag=str(i), tiled=tiled)
        _, calls = run_case(hostmodel, tmp_path, [line], **mode)
        assert calls[0][0] == 0
        _check_fp4_gemm(out, M, N, ldc, ops, bf16)


@pytest.mark.parametrize("mode,tiled", [(MODES[0], False), (MODES[3], True)], ids=["lazy-up-rowmajor", "eager-down-tiled"])
def test_fp4_gemm_persistent_small_tiles(hostmodel, tmp_path, mode, tiled):
    """Workgroups that walk over 3, 2 and 1 tiles of 128 x 128 with 2 and 3 K steps of 256 elements."""
    for i, (M, N, K, bf16, wgs) in enumerate([(256, 384, 768, False, 2), (256, 384, 512, True, 4), (384, 256, 768, False, 0)]):
        ops = _fp4_operands(M, N, K, seed=30 + i)
        line, out = _fp4_gemm_case(tmp_path, M, N, K, ops, bf16, tag=str(i), tiled=tiled, wg=wgs)
        _, calls = run_case(hostmodel, tmp_path, [line], **mode)
        assert calls[0] == (0, list(range(wgs or 6)))
        _check_fp4_gemm(out, M, N, N, ops, bf16)


@pytest.mark.parametrize("tiled,order", [(True, "up"), (False, "down")])
def test_fp4_gemm_persistent_large_tiles_sampled_workgroups(hostmodel, tmp_path, tiled, order):
    """256 x 256 configuration (requests spread over the K step, two scale requests per operand): 128 tiles on 64
    workgroups, first and last workgroup."""
    M, N, K = 2048, 4096, 768
    ops = _fp4_operands(M, N, K, seed=40)
    line, out = _fp4_gemm_case(tmp_path, M, N, K, ops, bf16=True, tiled=tiled, wg=64)
    _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_BLOCKS=2, WAVESIM_ORDER=order)
    assert calls[0] == (0, [0, 63])
    assert _check_fp4_gemm(out, M, N, N, ops, True, expect_full=False) == 4 * 256 * 256


def test_fp4_gemm_large_tiles_ragged_sampled_workgroups(hostmodel, tmp_path):
    """256 x 256 configuration, one workgroup per tile, ragged last tiles in both directions."""
    M, N, K = 2040, 4100, 512
    ops = _fp4_operands(M, N, K, seed=41)
    for tiled in (False, True):
        line, out = _fp4_gemm_case(tmp_path, M, N, K, ops, tiled=tiled, tag=str(int(tiled)))
        _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_BLOCKS=2)
        assert calls[0][0] == 0
        assert _check_fp4_gemm(out, M, N, N, ops, False, expect_full=False) > 256 * 256


def test_fp4_gemm_k_zero_and_validation(hostmodel, tmp_path):
    empty = np.zeros((0,), np.uint8)
    line, out = _fp4_gemm_case(tmp_path, 70, 40, 0, (empty, empty, empty, empty))
    _, calls = run_case(hostmodel, tmp_path, [line])
    assert calls[0][0] == 0 and (np.fromfile(out, np.float32) == 0).all()
    ops = _fp4_operands(64, 64, 256, seed=1)
    good, _ = _fp4_gemm_case(tmp_path, 64, 64, 256, ops, tag="v")
    _, calls = run_case(hostmodel, tmp_path, [good.replace("gemmfp4 0 64 64 256 f32 64", "gemmfp4 0 64 64 256 f32 32")], expect_ok=False)
    assert calls and calls[0][0] == 2


def test_model_notices_a_scale_byte_paired_with_the_wrong_block(hostmodel, tmp_path):
    """Self-test of these tests: swapping the two scale dwords of every K step in the operand file (what a kernel
    that mixed up its two scale requests would compute) must not pass the check."""
    M, N, K = 128, 128, 512
    ops = _fp4_operands(M, N, K, seed=3)
    a_q, a_s, b_q, b_s = ops
    swapped = a_s.reshape(M, K // 256, 2, 4)[:, :, ::-1].reshape(M, K // 32)
    line, out = _fp4_gemm_case(tmp_path, M, N, K, (a_q, np.ascontiguousarray(swapped), b_q, b_s))
    run_case(hostmodel, tmp_path, [line])
    with pytest.raises(AssertionError):
        _check_fp4_gemm(out, M, N, N, ops, False)

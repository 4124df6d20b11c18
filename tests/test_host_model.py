"""CPU tests that run the HIP kernel sources themselves, unchanged, on a host execution model.

tests/host_model/ compiles paper_2506_08027_amd/csrc/*.hip as host C++ (AddressSanitizer and
alignment checks on) against a stand-in for the HIP runtime header that runs every workgroup as 64
cooperative fibers per wavefront: cross-lane instructions and barriers are rendezvous points,
direct-to-LDS loads complete only at the `s_waitcnt vmcnt` that retires them (their destination
holds NaN-decoding poison until then), and one wavefront always runs maximally ahead of the others.
What these tests establish before any GPU run:
  * every global and LDS access of the kernels stays inside its buffer for ragged and multi-tile
    shapes (the usual cause of a GPU memory fault), inputs are not modified, padding is not written;
  * the index arithmetic, swizzles, scale handling and the wait/barrier protocol of the software
    pipeline produce the oracle's result (bit-exact for quantize/dequantize; the modelled MFMA sums
    in double, so the GEMM matches the oracle to FP32 rounding);
  * the launchers pick grids and tile configurations that cover the output exactly once.
They say nothing about speed or about the numerics of the real matrix instruction: those are the
GPU tests' business. The instruction semantics the model relies on are the ones probed on hardware
and documented in the kernel sources."""
import os
import subprocess

import numpy as np
import pytest

import oracle
import scale_layout as sl
from paper_2506_08027_amd import synth_inputs as si

HERE = os.path.dirname(os.path.abspath(__file__))
MODEL_DIR = os.path.join(HERE, "host_model")
BINARY = os.path.join(MODEL_DIR, "_build", "hostmodel")
SENTINEL = 0xA5


_BUILT = []   # the other host-model test modules import this fixture: one build per session, not one per module


@pytest.fixture(scope="session")
def hostmodel():
    if not _BUILT:
        res = subprocess.run([os.path.join(MODEL_DIR, "build.sh"), BINARY], capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-4000:]
        _BUILT.append(BINARY)
    return BINARY


def run_case(binary, tmp_path, lines, expect_ok=True, **env):
    case = tmp_path / "case.txt"
    case.write_text("\n".join(lines) + "\n")
    res = subprocess.run([binary, str(case)], capture_output=True, text=True, timeout=600,
                         env=dict(os.environ, **{k: str(v) for k, v in env.items()}))
    if expect_ok:
        assert res.returncode == 0, (res.stdout + res.stderr)[-4000:]
    calls = []
    for line in res.stdout.splitlines():
        tok = line.split()
        if tok[:1] == ["status"]:
            calls.append((int(tok[1]), [int(t) for t in tok[3:]]))
    return res, calls


def put(tmp_path, name, arr):
    path = tmp_path / name
    np.ascontiguousarray(arr).tofile(path)
    return str(path)


def get(path, dtype, shape):
    return np.fromfile(path, dtype=dtype).reshape(shape)


# ---- quantize -------------------------------------------------------------------------------------
def _compare_scales(path, want, tiled):
    """Row-major: byte for byte. Tiled: every (row, block) byte at its tiled position; of the filler
    positions only those inside a written dword may have changed (rows past the end are never written)."""
    rows, nb = want.shape
    if not tiled:
        assert np.array_equal(get(path, np.uint8, want.shape), want)
        return
    flat = np.fromfile(path, np.uint8)
    assert flat.size == sl.tiled_bytes(rows, nb)
    assert np.array_equal(sl.untile(flat, rows, nb), want)
    dwords = flat.reshape(-1, 64, 4)                                  # [group * K step][row in group][block]
    row_of = (np.arange(dwords.shape[0]) // ((nb + 3) // 4))[:, None] * 64 + np.arange(64)[None, :]
    assert (dwords[row_of >= rows] == SENTINEL).all(), "scale dwords of rows past the end were written"


def _quantize_and_compare(hostmodel, tmp_path, x, bf16, axis, ld=None, tiled=False, groups=None, **env):
    rows, cols = x.shape
    ld = ld or cols
    stored = np.zeros((rows, ld), x.dtype)
    stored[:, :cols] = x
    flat = stored.reshape(-1)[: (rows - 1) * ld + cols]
    src = put(tmp_path, "x.bin", flat)
    prefix = str(tmp_path / "out")
    _, calls = run_case(hostmodel, tmp_path,
                        [f"quantize {'bf16' if bf16 else 'f32'} {rows} {cols} {ld} {axis} {src} {prefix}"
                         + (" tiled" if tiled else "")], **env)
    assert calls[0][0] == 0
    tiles = ((rows + 127) // 128) * ((cols + 127) // 128)
    assert calls[0][1] == list(range(groups or tiles))
    xin = np.ascontiguousarray(x)          # the oracle takes FP32 values or BF16 bit patterns (uint16)
    if axis & 1:
        q, s = oracle.quantize_rowwise(xin)
        assert np.array_equal(get(prefix + ".q_row", np.uint8, q.shape), q)
        _compare_scales(prefix + ".s_row", s, tiled)
    if axis & 2:
        q, s = oracle.quantize_colwise(xin)
        assert np.array_equal(get(prefix + ".q_colT", np.uint8, q.shape), q)
        _compare_scales(prefix + ".s_colT", s, tiled)


@pytest.mark.parametrize("axis", [1, 2, 3])
def test_quantize_fp32_with_every_special_block(hostmodel, tmp_path, axis):
    _quantize_and_compare(hostmodel, tmp_path, si.tiny_with_specials(256, seed=0), False, axis)


@pytest.mark.parametrize("axis", [1, 2, 3])
def test_quantize_bf16_with_special_blocks(hostmodel, tmp_path, axis):
    x = si.to_bf16_bits(si.tiny_with_specials(256, seed=1))
    _quantize_and_compare(hostmodel, tmp_path, x, True, axis)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape,ld", [((160, 96), 128), ((32, 288), 288), ((288, 32), 40)])
def test_quantize_ragged_tiles_and_leading_dimension(hostmodel, tmp_path, bf16, shape, ld):
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(shape) * np.exp(rng.standard_normal(shape[1]))).astype(np.float32)
    x[5, 3], x[40 % shape[0], 70 % shape[1]] = np.inf, np.nan
    if bf16:
        x = si.to_bf16_bits(x)
        ld = (ld + 7) // 8 * 8
    else:
        ld = (ld + 3) // 4 * 4
    _quantize_and_compare(hostmodel, tmp_path, x, bf16, 3, ld)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", [(256, 256), (160, 96), (32, 288), (288, 32)])
def test_quantize_tiled_scales(hostmodel, tmp_path, bf16, shape):
    """Same values, scale bytes stored in the tiled layout (both copies)."""
    x = si.tiny_with_specials(256, seed=2)[: shape[0], : shape[1]] if shape == (256, 256) else \
        (np.random.default_rng(9).standard_normal(shape) * 3).astype(np.float32)
    x = np.ascontiguousarray(x)
    if bf16:
        x = si.to_bf16_bits(x)
    _quantize_and_compare(hostmodel, tmp_path, x, bf16, 3, tiled=True)


# ---- dequantize -----------------------------------------------------------------------------------
@pytest.mark.parametrize("tiled", [False, True])
def test_quantize_resident_grid_walks_over_several_tiles(hostmodel, tmp_path, tiled):
    """The both-axes pass over a BF16 source runs on 4 workgroups per compute unit: on a one-unit device the 30
    tiles (ragged in both directions) of a 736 x 608 source go to 4 workgroups, 7 or 8 tiles each."""
    x = si.to_bf16_bits(np.random.default_rng(4).standard_normal((736, 608)).astype(np.float32) * 3)
    _quantize_and_compare(hostmodel, tmp_path, x, True, 3, tiled=tiled, groups=4, WAVESIM_CUS=1)


@pytest.mark.parametrize("bf16,axis", [(False, 3), (True, 3), (False, 2), (True, 1)])
def test_quantize_wide_tensors_walk_down_their_columns(hostmodel, tmp_path, bf16, axis):
    """More columns than rows with the column copy wanted: the tiles are handed out down the columns (3 x 5 tiles, ragged
    in both directions; BF16 with both copies on the resident grid of a one-unit device, 4 workgroups over 15 tiles).
    The row-only case keeps the row order."""
    x = (np.random.default_rng(6).standard_normal((288, 608)) * 3).astype(np.float32)
    x[7, 300], x[200, 5] = np.inf, np.nan
    env = dict(groups=4, WAVESIM_CUS=1) if bf16 and axis == 3 else {}
    _quantize_and_compare(hostmodel, tmp_path, si.to_bf16_bits(x) if bf16 else x, bf16, axis, tiled=bf16, **env)


@pytest.mark.parametrize("tiled", [False, True])
def test_requantize_column_copy_from_row_copy(hostmodel, tmp_path, tiled):
    """Single-copy storage: ragged tiles, every special block of the tiny configuration in the row copy."""
    x = np.ascontiguousarray(si.tiny_with_specials(256, seed=0)[:160, :224])
    q, s = oracle.quantize_rowwise(x)
    prefix = str(tmp_path / "rq")
    _, calls = run_case(hostmodel, tmp_path, [f"requant 160 224 {put(tmp_path, 'q.bin', q)} "
                                              f"{put(tmp_path, 's.bin', sl.tile(s) if tiled else s)} {prefix}" + (" tiled" if tiled else "")])
    assert calls[0] == (0, [0, 1, 2, 3])
    qT, sT = oracle.requantize_colwise(q, s)
    assert np.array_equal(get(prefix + ".q_colT", np.uint8, qT.shape), qT)
    _compare_scales(prefix + ".s_colT", sT, tiled)


@pytest.mark.parametrize("bf16", [False, True])
def test_dequantize_all_codes_and_padding_untouched(hostmodel, tmp_path, bf16):
    scales = np.array([0, 1, 100, 126, 127, 128, 200, 253, 254, 255], np.uint8)
    q = np.tile(np.arange(256, dtype=np.uint8), (len(scales), 1))           # [10 x 256]
    s = np.repeat(scales[:, None], 8, axis=1)
    ld = 264
    out = str(tmp_path / "d.bin")
    _, calls = run_case(hostmodel, tmp_path, [
        f"dequantize {q.shape[0]} 256 {'bf16' if bf16 else 'f32'} {ld} {put(tmp_path, 'q.bin', q)} "
        f"{put(tmp_path, 's.bin', s)} {out}"])
    assert calls[0][0] == 0
    n = (q.shape[0] - 1) * ld + 256
    ref = oracle.dequantize(q, s, "bf16" if bf16 else "f32")
    if bf16:
        got = np.zeros(q.shape[0] * ld, np.uint16)
        got[:n] = np.fromfile(out, np.uint16)
        got = got.reshape(q.shape[0], ld)
        ref = np.asarray(ref, np.uint16)
        pad = 0xA5A5
    else:
        got = np.zeros(q.shape[0] * ld, np.uint32)
        got[:n] = np.fromfile(out, np.uint32)
        got = got.reshape(q.shape[0], ld)
        ref = np.asarray(ref, np.float32).view(np.uint32)
        pad = 0xA5A5A5A5
    val, exp = got[:, :256], ref
    nan_exp = np.isnan(ref.view(np.float32)) if not bf16 else ((ref & 0x7FFF) > 0x7F80)
    nan_got = np.isnan(val.view(np.float32)) if not bf16 else ((val & 0x7FFF) > 0x7F80)
    assert np.array_equal(nan_got, nan_exp)
    assert np.array_equal(val[~nan_exp], exp[~nan_exp])
    assert (got[:-1, 256:] == pad).all()


# ---- gemm -----------------------------------------------------------------------------------------
def _operands(M, N, K, seed, spikes=False):
    a = si.gradients(M, K, seed=seed, spikes=spikes) if spikes else si.activations(M, K, seed=seed, bf16=False)
    b = si.weights(N, K, seed=seed + 1, bf16=False)
    return oracle.quantize_rowwise(np.asarray(a, np.float32)) + oracle.quantize_rowwise(np.asarray(b, np.float32))


def _gemm_case(tmp_path, M, N, K, ops, bf16=False, ldc=None, tag="", tiled=False, wg=0):
    a_q, a_s, b_q, b_s = ops
    ldc = ldc or N
    if tiled:   # filler bytes are 0xFF (a NaN scale): a kernel that read one as a scale would show it
        a_s, b_s = sl.tile(a_s, filler=0xFF), sl.tile(b_s, filler=0xFF)
    names = [put(tmp_path, f"{n}{tag}.bin", v) for n, v in (("aq", a_q), ("as", a_s), ("bq", b_q), ("bs", b_s))]
    out = str(tmp_path / f"c{tag}.bin")
    return (f"gemm 0 {M} {N} {K} {'bf16' if bf16 else 'f32'} {ldc} {' '.join(names)} {out}"
            + (" tiled" if tiled else "") + (f" wg={wg}" if wg else "")), out


def _check_gemm(out, M, N, ldc, ops, bf16, expect_full=True):
    """Compares whatever part of C the simulated workgroups wrote against the oracle. The modelled
    instruction sums in double and rounds once per K step, so the result is within K/128 FP32 roundings of
    the sum (2^-24 * sum|a b| each) plus, for BF16 output, one BF16 rounding of the value."""
    a_q, a_s, b_q, b_s = ops
    n = (M - 1) * ldc + N
    if bf16:
        raw = np.full(M * ldc, 0xA5A5, np.uint16)
        raw[:n] = np.fromfile(out, np.uint16)
        raw = raw.reshape(M, ldc)
        written = raw[:, :N] != 0xA5A5
        val = si.bf16_bits_to_f32(raw[:, :N])
        pad_ok = (raw[:, N:] == 0xA5A5).all()
    else:
        raw = np.full(M * ldc, 0xA5A5A5A5, np.uint32)
        raw[:n] = np.fromfile(out, np.uint32)
        raw = raw.reshape(M, ldc)
        written = raw[:, :N] != 0xA5A5A5A5
        val = raw[:, :N].view(np.float32)
        pad_ok = (raw[:, N:] == 0xA5A5A5A5).all()
    assert pad_ok, "bytes between rows of C were written"
    if expect_full:
        assert written.all()
    rows = np.unique(np.nonzero(written)[0])
    assert rows.size
    ref, absum = oracle.gemm_rows(a_q, a_s, b_q, b_s, rows)
    steps = max(a_q.shape[1] // 128, 2)
    tol = steps * 2.0 ** -24 * absum + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0) + 1e-300
    w = written[rows]
    err = np.abs(val[rows].astype(np.float64) - ref)
    assert not np.isnan(val[rows][w]).any(), "NaN in C: a tile was read before its loads were waited for"
    assert (err[w] <= tol[w]).all(), float((err[w] / tol[w]).max())
    return int(written.sum())


MODES = [dict(), dict(WAVESIM_DMA="eager"), dict(WAVESIM_ORDER="down"), dict(WAVESIM_DMA="eager", WAVESIM_ORDER="down")]


@pytest.mark.parametrize("mode", [MODES[0], MODES[3]], ids=["lazy-up", "eager-down"])
def test_gemm_small_tiles_ragged(hostmodel, tmp_path, mode):
    """128x128 configuration: 2x2 tiles, ragged in M and N, K = one, two and three steps (prologue
    and tail prefetch clamps), FP32 and BF16 output, padded C."""
    lines, checks = [], []
    for i, (M, N, K, bf16, ldc) in enumerate([(200, 136, 384, False, 136), (130, 129, 128, True, 136),
                                               (64, 200, 256, False, 204)]):
        ops = _operands(M, N, K, seed=10 + i)
        line, out = _gemm_case(tmp_path, M, N, K, ops, bf16, ldc, tag=str(i))
        lines.append(line)
        checks.append((out, M, N, ldc, ops, bf16))
    _, calls = run_case(hostmodel, tmp_path, lines, **mode)
    assert [c[0] for c in calls] == [0, 0, 0]
    for c in checks:
        _check_gemm(*c)


@pytest.mark.parametrize("mode", [MODES[0], MODES[3]], ids=["lazy-up", "eager-down"])
def test_gemm_large_tiles_sampled_workgroups(hostmodel, tmp_path, mode):
    """256x256 configuration (taken when there are at least 128 such tiles): first, last (ragged in
    both directions) and two interior workgroups of a 9 x 16 tile grid."""
    M, N, K = 2048 + 72, 4096 - 100, 384
    ops = _operands(M, N, K, seed=20, spikes=True)
    line, out = _gemm_case(tmp_path, M, N, K, ops, bf16=True)
    _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_BLOCKS=4, **mode)
    assert calls[0] == (0, [0, 47, 95, 143])
    n_written = _check_gemm(out, M, N, N, ops, True, expect_full=False)
    # two interior tiles, plus the two corner tiles of the XCD-aware order, whatever their raggedness:
    # every simulated workgroup wrote a disjoint tile
    assert 2 * 256 * 256 < n_written <= 4 * 256 * 256


@pytest.mark.parametrize("mode", [MODES[0], MODES[3]], ids=["lazy-up", "eager-down"])
def test_gemm_tiled_scales_small_tiles(hostmodel, tmp_path, mode):
    """Tiled scale operands, 128x128 configuration, ragged shapes whose last 64-row group is partial."""
    lines, checks = [], []
    for i, (M, N, K, bf16, ldc) in enumerate([(200, 136, 384, False, 136), (130, 129, 128, True, 136),
                                               (30, 250, 256, False, 252)]):
        ops = _operands(M, N, K, seed=60 + i)
        line, out = _gemm_case(tmp_path, M, N, K, ops, bf16, ldc, tag=str(i), tiled=True)
        lines.append(line)
        checks.append((out, M, N, ldc, ops, bf16))
    _, calls = run_case(hostmodel, tmp_path, lines, **mode)
    assert [c[0] for c in calls] == [0, 0, 0]
    for c in checks:
        _check_gemm(*c)


def test_gemm_tiled_scales_large_tiles_sampled_workgroups(hostmodel, tmp_path):
    M, N, K = 2048 + 72, 4096 - 100, 384
    ops = _operands(M, N, K, seed=21, spikes=True)
    line, out = _gemm_case(tmp_path, M, N, K, ops, bf16=False, tiled=True)
    _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_BLOCKS=4)
    assert calls[0] == (0, [0, 47, 95, 143])
    n_written = _check_gemm(out, M, N, N, ops, False, expect_full=False)
    assert 2 * 256 * 256 < n_written <= 4 * 256 * 256


def test_dequantize_tiled_scales(hostmodel, tmp_path):
    rng = np.random.default_rng(3)
    rows, cols = 100, 96                                   # partial last group, blocks not a multiple of 4
    q = rng.integers(0, 256, (rows, cols), dtype=np.uint8)
    s = rng.integers(100, 150, (rows, cols // 32), dtype=np.uint8)
    out = str(tmp_path / "d.bin")
    _, calls = run_case(hostmodel, tmp_path, [
        f"dequantize {rows} {cols} f32 {cols} {put(tmp_path, 'q.bin', q)} {put(tmp_path, 's.bin', sl.tile(s))} {out} tiled"])
    assert calls[0][0] == 0
    got = np.fromfile(out, np.float32).reshape(rows, cols)
    want = np.asarray(oracle.dequantize(q, s, "f32"), np.float32)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[~np.isnan(want)], want[~np.isnan(want)])


@pytest.mark.parametrize("bf16,tiled,rows,cols,cus", [(False, True, 100, 96, 1), (True, False, 300, 160, 1),
                                                       (True, True, 515, 64, 1), (False, False, 257, 224, 2)])
def test_dequantize_resident_grid_unrolled_loop_and_tail(hostmodel, tmp_path, bf16, tiled, rows, cols, cus):
    """On a device shrunk to 1 or 2 compute units the grid is smaller than the work: work-items take several rounds
    with four loads in flight, then single items, and some take none; padded output rows stay untouched."""
    rng = np.random.default_rng(rows + cols)
    q = rng.integers(0, 256, (rows, cols), dtype=np.uint8)
    s = rng.integers(90, 160, (rows, cols // 32), dtype=np.uint8)
    s[rows // 2, 0] = 255                                  # a NaN block
    ld = cols + 8
    out = str(tmp_path / "d.bin")
    _, calls = run_case(hostmodel, tmp_path, [
        f"dequantize {rows} {cols} {'bf16' if bf16 else 'f32'} {ld} {put(tmp_path, 'q.bin', q)} "
        f"{put(tmp_path, 's.bin', sl.tile(s) if tiled else s)} {out}" + (" tiled" if tiled else "")], WAVESIM_CUS=cus)
    assert calls[0][0] == 0
    dt = np.uint16 if bf16 else np.uint32
    n = (rows - 1) * ld + cols
    got = np.zeros(rows * ld, dt)
    got[:n] = np.fromfile(out, dt)
    got = got.reshape(rows, ld)
    want = oracle.dequantize(q, s, "bf16" if bf16 else "f32")
    want = np.asarray(want, np.uint16) if bf16 else np.asarray(want, np.float32).view(np.uint32)
    nan = ((want & 0x7FFF) > 0x7F80) if bf16 else np.isnan(want.view(np.float32))
    val = got[:, :cols]
    assert nan[rows // 2, :32].all()
    assert np.array_equal(((val & 0x7FFF) > 0x7F80) if bf16 else np.isnan(val.view(np.float32)), nan)
    assert np.array_equal(val[~nan], want[~nan])
    assert (got[:-1, cols:] == (0xA5A5 if bf16 else 0xA5A5A5A5)).all()


# ---- persistent GEMM kernel (every problem made of full tiles; max_workgroups bounds its grid) ------------
@pytest.mark.parametrize("mode,tiled", [(MODES[0], False), (MODES[3], True)], ids=["lazy-up-rowmajor", "eager-down-tiled"])
def test_gemm_persistent_small_tiles(hostmodel, tmp_path, mode, tiled):
    """Workgroups that walk over 3, 2 and 1 tiles (6 tiles of 128x128 on 2, 4 and 6 workgroups), K of
    2 and 3 steps: the K pipeline runs across tile boundaries, each tile is stored once."""
    for i, (M, N, K, bf16, wgs) in enumerate([(256, 384, 384, False, 2), (256, 384, 256, True, 4),
                                               (384, 256, 384, False, 0)]):
        ops = _operands(M, N, K, seed=80 + i)
        line, out = _gemm_case(tmp_path, M, N, K, ops, bf16, tag=str(i), tiled=tiled, wg=wgs)
        _, calls = run_case(hostmodel, tmp_path, [line], **mode)
        assert calls[0] == (0, list(range(wgs or 6)))
        _check_gemm(out, M, N, N, ops, bf16)


@pytest.mark.parametrize("tiled,order", [(True, "up"), (False, "down")])
def test_gemm_persistent_large_tiles_sampled_workgroups(hostmodel, tmp_path, tiled, order):
    """256x256 configuration (requests spread over the K step): 128 tiles on 64 workgroups (2 tiles each),
    first and last workgroup."""
    M, N, K = 2048, 4096, 384
    ops = _operands(M, N, K, seed=90, spikes=True)
    line, out = _gemm_case(tmp_path, M, N, K, ops, bf16=True, tiled=tiled, wg=64)
    _, calls = run_case(hostmodel, tmp_path, [line], WAVESIM_BLOCKS=2, WAVESIM_ORDER=order)
    assert calls[0] == (0, [0, 63])
    assert _check_gemm(out, M, N, N, ops, True, expect_full=False) == 4 * 256 * 256


def test_gemm_ragged_shapes_take_one_workgroup_per_tile(hostmodel, tmp_path):
    M, N, K = 200, 136, 384
    ops = _operands(M, N, K, seed=91)
    line, out = _gemm_case(tmp_path, M, N, K, ops, wg=2)
    _, calls = run_case(hostmodel, tmp_path, [line])
    assert calls[0] == (0, [0, 1, 2, 3])                 # the bound only applies to the persistent kernel
    _check_gemm(out, M, N, N, ops, False)


def test_gemm_unaligned_c_takes_element_stores(hostmodel, tmp_path):
    M, N, K = 40, 37, 128
    ops = _operands(M, N, K, seed=30)
    line, out = _gemm_case(tmp_path, M, N, K, ops, bf16=True, ldc=37)
    _, calls = run_case(hostmodel, tmp_path, [line])
    assert calls[0][0] == 0
    _check_gemm(out, M, N, 37, ops, True)


def test_gemm_k_zero_stores_zeros(hostmodel, tmp_path):
    M, N = 70, 40
    empty = np.zeros((0,), np.uint8)
    line, out = _gemm_case(tmp_path, M, N, 0, (empty, empty, empty, empty))
    _, calls = run_case(hostmodel, tmp_path, [line])
    assert calls[0][0] == 0
    assert (np.fromfile(out, np.float32) == 0).all()


def test_model_notices_a_missing_wait(hostmodel, tmp_path):
    """Self-test of the model: with every partial `s_waitcnt vmcnt(n > 0)` of the K loop ignored the
    fragments are read before their tiles have landed, and the result must come out as NaN."""
    M, N, K = 128, 128, 384
    ops = _operands(M, N, K, seed=40)
    line, out = _gemm_case(tmp_path, M, N, K, ops)
    run_case(hostmodel, tmp_path, [line], WAVESIM_DROP_PARTIAL_WAITS=1)
    assert np.isnan(np.fromfile(out, np.float32)).all()


def test_validation_errors_reach_the_caller(hostmodel, tmp_path):
    ops = _operands(32, 32, 128, seed=50)
    good, _ = _gemm_case(tmp_path, 32, 32, 128, ops)
    bad_k = good.replace("gemm 0 32 32 128 f32 32", "gemm 0 32 32 128 f32 16")      # ldc < N
    res, calls = run_case(hostmodel, tmp_path, [bad_k], expect_ok=False)
    assert calls and calls[0][0] == 2


# ---- GEMM that also emits the MXFP8 copies of its BF16 output -------------------------------------------
def _fused_case(hostmodel, tmp_path, M, N, K, axis, tiled, seed, wg=0, **env):
    """Runs mxfp8_gemm_quantize_ex with exact-size buffers under AddressSanitizer and checks, for every
    output tile the simulated workgroups wrote, that c is the BF16 product and that the copies are the
    oracle's quantization of exactly those BF16 values."""
    a_q, a_s, b_q, b_s = _operands(M, N, K, seed=seed)
    a_s = a_s.copy()
    a_s[3, 1] = 0xFF                     # a NaN row of C
    a_s[5, :] = 250                      # a row whose products overflow to +-Inf in BF16
    ops = (a_q, a_s, b_q, b_s)
    sa, sb = (sl.tile(a_s, filler=0xFF), sl.tile(b_s, filler=0xFF)) if tiled else (a_s, b_s)
    names = [put(tmp_path, f"{n}.bin", v) for n, v in (("aq", a_q), ("as", sa), ("bq", b_q), ("bs", sb))]
    prefix = str(tmp_path / "f")
    _, calls = run_case(hostmodel, tmp_path,
                        [f"gemmq 0 {M} {N} {K} {N} {axis} {' '.join(names)} {prefix}" + (" tiled" if tiled else "")
                         + (f" wg={wg}" if wg else "")], **env)
    assert calls[0][0] == 0
    bits = np.fromfile(prefix + ".c", np.uint16).reshape(M, N)
    written = bits != 0xA5A5
    rows = np.unique(np.nonzero(written)[0])
    cols = np.unique(np.nonzero(written)[1])
    assert rows.size and rows.size % 32 == 0 and cols.size % 32 == 0
    # the product itself, on the written part (one FP32 rounding of the modelled sum, one BF16 rounding)
    ref, absum = oracle.gemm_rows(*ops, rows)
    val = si.bf16_bits_to_f32(bits[rows]).astype(np.float64)
    w = written[rows]
    fin = w & np.isfinite(ref) & (absum < 3e38)
    assert (np.abs(val - ref)[fin] <= (2.0 ** -23 * absum + 2.0 ** -8 * np.abs(ref) + 1e-300)[fin]).all()
    # the copies: whole 32-blocks of written rows / columns, quantized from the stored BF16 bits
    if axis & 1:
        q = np.fromfile(prefix + ".q_row", np.uint8).reshape(M, N)
        s = np.fromfile(prefix + ".s_row", np.uint8)
        s = sl.untile(s, M, N // 32) if tiled else s.reshape(M, N // 32)
        for r in rows:
            c = np.nonzero(written[r])[0]
            wq, ws = oracle.quantize_rowwise(np.ascontiguousarray(bits[r:r + 1, c]))
            assert np.array_equal(q[r, c], wq[0]) and np.array_equal(s[r, c[::32] // 32], ws[0])
    if axis & 2:
        q = np.fromfile(prefix + ".q_colT", np.uint8).reshape(N, M)
        s = np.fromfile(prefix + ".s_colT", np.uint8)
        s = sl.untile(s, N, M // 32) if tiled else s.reshape(N, M // 32)
        for c in cols:
            r = np.nonzero(written[:, c])[0]
            wq, ws = oracle.quantize_colwise(np.ascontiguousarray(bits[r, c:c + 1]))
            assert np.array_equal(q[c, r], wq[0]) and np.array_equal(s[c, r[::32] // 32], ws[0])
    return int(written.sum())


@pytest.mark.parametrize("axis,tiled,mode", [(1, False, MODES[0]), (2, True, MODES[3]), (3, False, MODES[3]),
                                             (3, True, MODES[0])])
def test_fused_output_quantization_small_tiles(hostmodel, tmp_path, axis, tiled, mode):
    """128x128 configuration, 6 tiles on 2 workgroups and one tile on the default grid."""
    assert _fused_case(hostmodel, tmp_path, 256, 384, 384, axis, tiled, seed=300 + axis, wg=2, **mode) == 256 * 384
    assert _fused_case(hostmodel, tmp_path, 128, 128, 256, axis, tiled, seed=310 + axis, **mode) == 128 * 128


@pytest.mark.parametrize("axis,tiled", [(3, True), (3, False)])
def test_fused_output_quantization_large_tiles_sampled_workgroups(hostmodel, tmp_path, axis, tiled):
    """256x256 configuration, 128 tiles on 64 workgroups: the first and the last workgroup, two tiles each."""
    n = _fused_case(hostmodel, tmp_path, 2048, 4096, 384, axis, tiled, seed=320, wg=64, WAVESIM_BLOCKS=2)
    assert n == 4 * 256 * 256


# ---- measurement aids ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_copy_rate_probe_copies_exactly_its_bytes(hostmodel, tmp_path, mode):
    """Sizes that leave a tail for the unrolled loop, fewer units than work-items, and a single unit."""
    rng = np.random.default_rng(mode)
    lines, want = [], []
    for i, (units, wgs) in enumerate([(3 * 256 * 4 * 3 + 777, 3), (100, 2), (1, 5)]):
        data = rng.integers(0, 256, units * 16, dtype=np.uint8)
        out = str(tmp_path / f"d{i}.bin")
        lines.append(f"copy {units * 16} {wgs} {mode} {put(tmp_path, f's{i}.bin', data)} {out}")
        want.append((out, data))
    _, calls = run_case(hostmodel, tmp_path, lines)
    assert [c[0] for c in calls] == [0, 0, 0]
    for out, data in want:
        assert np.array_equal(np.fromfile(out, np.uint8), data)


@pytest.mark.parametrize("mode,run", [(3, 128), (4, 256)])
def test_copy_rate_probe_scattered_runs_permute_the_bytes(hostmodel, tmp_path, mode, run):
    rng = np.random.default_rng(mode)
    nruns = 64 * 5
    data = rng.integers(0, 256, nruns * run, dtype=np.uint8)
    out = str(tmp_path / "d.bin")
    _, calls = run_case(hostmodel, tmp_path, [f"copy {data.size} 3 {mode} {put(tmp_path, 's.bin', data)} {out}"])
    assert calls[0][0] == 0
    r = np.arange(nruns)
    where = (r % 64) * (nruns // 64) + r // 64
    want = np.empty_like(data).reshape(nruns, run)
    want[where] = data.reshape(nruns, run)
    assert np.array_equal(np.fromfile(out, np.uint8), want.ravel())

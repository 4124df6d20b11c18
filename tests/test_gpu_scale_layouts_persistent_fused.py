"""GPU parity of the tiled scale layout (MXFP8_SCALES_TILED), of the persistent GEMM kernel with a bounded
number of workgroups, and of the GEMM that also emits the MXFP8 copies of its BF16 output, through the C
ABI against the CPU oracle. The layout only moves scale bytes, so every value must equal what the
row-major entry points are held to: quantized bytes bit-exact, products within the tolerance of
test_gpu_gemm, and, on identical operands, identical to the row-major product bit for bit (the same
instructions add the same numbers in the same order). The persistent kernel runs the same K steps in the
same order as the one-tile-per-workgroup kernel, so the two agree bit for bit, whatever the number of
workgroups."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_08027_amd as mx
import scale_layout as sl
from paper_2506_08027_amd import synth_inputs as si
from mfma_model import hw_tolerance
from test_gpu_gemm import FRO_HW, TARGET_ELEM, _compare

pytestmark = pytest.mark.gpu
TILED = mx.SCALES_TILED


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _src(host, bf16):
    if bf16:
        return _dev(si.to_bf16_bits(host).view(np.int16)).view(torch.bfloat16), si.to_bf16_bits(host)
    return _dev(host), host


def _check_tiled_scales(flat, want):
    rows, nb = want.shape
    flat = flat.cpu().numpy()
    assert flat.size == sl.tiled_bytes(rows, nb)
    assert np.array_equal(sl.untile(flat, rows, nb), want)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", [(256, 256), (160, 96), (32, 288), (288, 32), (1024, 4096)])
def test_quantize_tiled_matches_oracle(shape, bf16):
    host = si.tiny_with_specials(256, seed=2) if shape == (256, 256) else \
        np.asarray(si.gradients(shape[0], shape[1], seed=shape[0] + shape[1], spikes=True), np.float32)
    src, oracle_in = _src(host, bf16)
    out = mx.quantize(src, "both", scale_layout=TILED)
    torch.cuda.synchronize()
    q, s = oracle.quantize_rowwise(np.ascontiguousarray(oracle_in))
    assert np.array_equal(out["q_row"].cpu().numpy(), q)
    _check_tiled_scales(out["s_row"], s)
    q, s = oracle.quantize_colwise(np.ascontiguousarray(oracle_in))
    assert np.array_equal(out["q_colT"].cpu().numpy(), q)
    _check_tiled_scales(out["s_colT"], s)


@pytest.mark.parametrize("axis", ["rowwise", "colwise"])
def test_quantize_tiled_single_axis_and_untouched_filler(axis):
    host = np.asarray(si.activations(160, 96, seed=5, bf16=False), np.float32)
    src = _dev(host)
    u8 = dict(dtype=torch.uint8, device="cuda")
    rows, cols = host.shape
    q = torch.empty((rows, cols) if axis == "rowwise" else (cols, rows), **u8)
    r, nb = (rows, cols // 32) if axis == "rowwise" else (cols, rows // 32)
    s = torch.full((sl.tiled_bytes(r, nb),), 0xA5, **u8)
    if axis == "rowwise":
        mx.mxfp8_quantize_ex(src, axis, q_row=q, s_row=s, scale_layout=TILED)
        wq, ws = oracle.quantize_rowwise(host)
    else:
        mx.mxfp8_quantize_ex(src, axis, q_colT=q, s_colT=s, scale_layout=TILED)
        wq, ws = oracle.quantize_colwise(host)
    torch.cuda.synchronize()
    assert np.array_equal(q.cpu().numpy(), wq)
    flat = s.cpu().numpy()
    assert np.array_equal(sl.untile(flat, r, nb), ws)
    dwords = flat.reshape(-1, 64, 4)
    row_of = (np.arange(dwords.shape[0]) // ((nb + 3) // 4))[:, None] * 64 + np.arange(64)[None, :]
    assert (dwords[row_of >= r] == 0xA5).all()          # rows past the end are never written


def _operands(M, N, K, seed):
    a = np.asarray(si.activations(M, K, seed=seed, bf16=False), np.float32)
    b = np.asarray(si.weights(N, K, seed=seed + 1, bf16=False), np.float32)
    return oracle.quantize_rowwise(a) + oracle.quantize_rowwise(b)


def _gemm_both_layouts(ops, dtype):
    a_q, a_s, b_q, b_s = ops
    flat = lambda s: _dev(sl.tile(s, filler=0xFF))       # a filler byte read as a scale would give NaN
    c_t = mx.gemm("fprop", _dev(a_q), flat(a_s), _dev(b_q), flat(b_s), dtype, scale_layout=TILED)
    c_r = mx.gemm("fprop", _dev(a_q), _dev(a_s), _dev(b_q), _dev(b_s), dtype)
    torch.cuda.synchronize()
    return c_t, c_r


@pytest.mark.parametrize("shape", [(200, 136, 384), (130, 129, 128), (30, 250, 256), (2120, 3996, 512)])
def test_gemm_tiled_matches_oracle_and_row_major(shape):
    M, N, K = shape
    ops = _operands(M, N, K, seed=70 + M)
    c_t, c_r = _gemm_both_layouts(ops, torch.float32)
    assert torch.equal(c_t, c_r)
    rows = np.unique(np.linspace(0, M - 1, min(M, 48)).astype(int))
    ref, absref = oracle.gemm_rows(*ops, rows)
    _compare(c_t.cpu().numpy().astype(np.float64)[rows], ref, absref, TARGET_ELEM, FRO_HW, f"tiled {shape}",
             extra=hw_tolerance(*ops, rows=rows))


def test_gemm_tiled_full_size_bf16_equals_row_major():
    """The benchmark's forward product (8192 x 14336 x 4096) from operands quantized on the GPU in
    both layouts: same element bytes, same scale values, identical BF16 result."""
    T, H, O = 8192, 4096, 14336
    X = _dev(si.activations(T, H, seed=2).view(np.int16)).view(torch.bfloat16)
    W = _dev(si.weights(O, H, seed=4).view(np.int16)).view(torch.bfloat16)
    xt, wt = mx.quantize(X, "rowwise", scale_layout=TILED), mx.quantize(W, "rowwise", scale_layout=TILED)
    xr, wr = mx.quantize(X, "rowwise"), mx.quantize(W, "rowwise")
    assert torch.equal(xt["q_row"], xr["q_row"]) and torch.equal(wt["q_row"], wr["q_row"])
    assert np.array_equal(sl.untile(xt["s_row"].cpu().numpy(), T, H // 32), xr["s_row"].cpu().numpy())
    assert np.array_equal(sl.untile(wt["s_row"].cpu().numpy(), O, H // 32), wr["s_row"].cpu().numpy())
    y_t = mx.gemm("fprop", xt["q_row"], xt["s_row"], wt["q_row"], wt["s_row"], torch.bfloat16, scale_layout=TILED)
    y_r = mx.gemm("fprop", xr["q_row"], xr["s_row"], wr["q_row"], wr["s_row"], torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(y_t.view(torch.int16), y_r.view(torch.int16))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_dequantize_tiled_matches_oracle(dtype):
    rng = np.random.default_rng(3)
    rows, cols = 100, 96
    q = rng.integers(0, 256, (rows, cols), dtype=np.uint8)
    s = rng.integers(90, 160, (rows, cols // 32), dtype=np.uint8)
    got = mx.dequantize(_dev(q), _dev(sl.tile(s)), dtype, scale_layout=TILED)
    torch.cuda.synchronize()
    if dtype == torch.float32:
        got = got.cpu().numpy()
        want = np.asarray(oracle.dequantize(q, s, "f32"), np.float32)
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], want[~nan])
    else:
        got = got.view(torch.int16).cpu().numpy().view(np.uint16)
        want = np.asarray(oracle.dequantize(q, s, "bf16"), np.uint16)
        nan = (want & 0x7FFF) > 0x7F80
        assert np.array_equal((got & 0x7FFF) > 0x7F80, nan) and np.array_equal(got[~nan], want[~nan])


def test_tiled_error_codes():
    u8 = dict(dtype=torch.uint8, device="cuda")
    src = torch.zeros((64, 64), dtype=torch.float32, device="cuda")
    q = torch.empty((64, 64), **u8)
    with pytest.raises(ValueError):                      # the binding checks the tiled buffer size
        mx.mxfp8_quantize_ex(src, "rowwise", q_row=q, s_row=torch.empty(255, **u8), scale_layout=TILED)
    with pytest.raises(mx.MXFP8Error) as e:              # unknown layout
        mx.mxfp8_quantize_ex(src, "rowwise", q_row=q, s_row=torch.empty((64, 2), **u8), scale_layout=7)
    assert e.value.code == 5
    base = torch.empty(512, **u8)
    off = (-base.data_ptr()) % 16 + 4
    with pytest.raises(mx.MXFP8Error) as e:              # tiled scale buffers must be 16-byte aligned
        mx.mxfp8_quantize_ex(src, "rowwise", q_row=q, s_row=base[off:off + 256], scale_layout=TILED)
    assert e.value.code == 3
    assert mx.mxfp8_scale_bytes(8192, 4096, TILED) == 8192 * 128
    assert mx.mxfp8_scale_bytes(100, 96, TILED) == 2 * 1 * 256


# ---- persistent GEMM kernel ---------------------------------------------------------------------------
def _one_tile_per_workgroup(args, dtype, lay):
    """The same product on the one-tile-per-workgroup kernel: an output whose rows are not 16-byte aligned
    cannot take the persistent kernel's vector stores."""
    M, N = args[1].shape[0], args[3].shape[0]
    pad = torch.empty((M, N + 1), dtype=dtype, device="cuda")
    mx.mxfp8_gemm_ex(*args, pad[:, :N], lay)
    return pad[:, :N].contiguous()


@pytest.mark.parametrize("shape,workgroups", [((256, 384, 384), 2), ((384, 256, 256), 0), ((2048, 4096, 512), 64),
                                              ((2048, 4096, 512), 0), ((4352, 4096, 256), 0)])
@pytest.mark.parametrize("tiled", [False, True])
def test_persistent_gemm_matches_oracle_and_one_tile_kernel(shape, workgroups, tiled):
    """Full-tile shapes run on the persistent kernel; 2 and 64 workgroups walk over 3 and 2 tiles each, the
    last shape has 272 tiles of 256 x 256 for 256 compute units (16 workgroups take a second tile)."""
    M, N, K = shape
    ops = _operands(M, N, K, seed=100 + M + K)
    a_q, a_s, b_q, b_s = ops
    lay = TILED if tiled else mx.SCALES_ROWMAJOR
    sc = (lambda s: _dev(sl.tile(s, filler=0xFF))) if tiled else _dev
    args = ("fprop", _dev(a_q), sc(a_s), _dev(b_q), sc(b_s))
    for dtype in (torch.float32, torch.bfloat16):
        bits = torch.int32 if dtype == torch.float32 else torch.int16
        pers = mx.gemm(*args, dtype, scale_layout=lay, max_workgroups=workgroups)
        plain = _one_tile_per_workgroup(args, dtype, lay)
        torch.cuda.synchronize()
        assert torch.equal(plain.view(bits), pers.view(bits))
    rows = np.unique(np.linspace(0, M - 1, min(M, 32)).astype(int))
    ref, absref = oracle.gemm_rows(*ops, rows)
    got = mx.gemm(*args, torch.float32, scale_layout=lay, max_workgroups=workgroups)
    torch.cuda.synchronize()
    _compare(got.cpu().numpy().astype(np.float64)[rows], ref, absref, TARGET_ELEM, FRO_HW,
             f"persistent {shape} x{workgroups}", extra=hw_tolerance(*ops, rows=rows))


def test_persistent_gemm_full_size_equals_one_tile_kernel_and_ignores_the_bound():
    """The benchmark's forward product (1792 tiles: 7 per workgroup on 256 compute units), both layouts; a
    bound of 100 workgroups changes nothing in the result."""
    T, H, O = 8192, 4096, 14336
    X = _dev(si.activations(T, H, seed=2).view(np.int16)).view(torch.bfloat16)
    W = _dev(si.weights(O, H, seed=4).view(np.int16)).view(torch.bfloat16)
    for lay in (mx.SCALES_ROWMAJOR, TILED):
        x, w = mx.quantize(X, "rowwise", scale_layout=lay), mx.quantize(W, "rowwise", scale_layout=lay)
        args = ("fprop", x["q_row"], x["s_row"], w["q_row"], w["s_row"])
        pers = mx.gemm(*args, torch.bfloat16, scale_layout=lay)
        bounded = mx.gemm(*args, torch.bfloat16, scale_layout=lay, max_workgroups=100)
        plain = _one_tile_per_workgroup(args, torch.bfloat16, lay)
        torch.cuda.synchronize()
        assert torch.equal(plain.view(torch.int16), pers.view(torch.int16))
        assert torch.equal(bounded.view(torch.int16), pers.view(torch.int16))


def test_negative_workgroup_bound_is_rejected():
    a_q, a_s, b_q, b_s = (_dev(t) for t in _operands(128, 128, 256, seed=8))
    with pytest.raises(mx.MXFP8Error) as e:
        mx.gemm("fprop", a_q, a_s, b_q, b_s, max_workgroups=-1)
    assert e.value.code == 5


# ---- GEMM with the MXFP8 copies of its BF16 output from the same epilogue -------------------------------
@pytest.mark.parametrize("shape,workgroups", [((256, 384, 384), 2), ((128, 128, 256), 0), ((2048, 4096, 512), 0),
                                              ((2048, 4096, 512), 50)])
@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("axis", ["rowwise", "colwise", "both"])
def test_fused_output_quantization_matches_gemm_then_quantize(shape, workgroups, tiled, axis):
    """c must equal the plain BF16 product bit for bit, and the copies must be the oracle's quantization of
    those BF16 values: NaN rows (a NaN scale), rows with entries that overflow to Inf and ordinary rows."""
    M, N, K = shape
    a_q, a_s, b_q, b_s = _operands(M, N, K, seed=200 + M)
    a_s = a_s.copy()
    a_s[3, 1] = 0xFF                     # row 3 of C becomes NaN
    a_s[5, :] = 250                      # row 5: many products overflow FP32, +-Inf in BF16
    lay = TILED if tiled else mx.SCALES_ROWMAJOR
    sc = (lambda s: _dev(sl.tile(s, filler=0xFF))) if tiled else _dev
    args = ("fprop", _dev(a_q), sc(a_s), _dev(b_q), sc(b_s))
    out = mx.gemm_quantize(*args, axis=axis, scale_layout=lay, max_workgroups=workgroups)
    plain = mx.gemm(*args, torch.bfloat16, scale_layout=lay)
    torch.cuda.synchronize()
    assert torch.equal(out["c"].view(torch.int16), plain.view(torch.int16))
    bits = np.ascontiguousarray(out["c"].view(torch.int16).cpu().numpy().view(np.uint16))
    assert ((bits[3] & 0x7FFF) > 0x7F80).all() and ((bits[5] & 0x7FFF) == 0x7F80).any()   # NaN row, Inf entries
    for ax, fn, qk, sk, shp in (("rowwise", oracle.quantize_rowwise, "q_row", "s_row", (M, N // 32)),
                                ("colwise", oracle.quantize_colwise, "q_colT", "s_colT", (N, M // 32))):
        if axis in (ax, "both"):
            q, s = fn(bits)
            assert np.array_equal(out[qk].cpu().numpy(), q), ax
            got = out[sk].cpu().numpy()
            assert np.array_equal(sl.untile(got, *shp) if tiled else got, s), ax
        else:
            assert qk not in out


def test_fused_output_quantization_rejects_partial_tiles():
    a_q, a_s, b_q, b_s = _operands(200, 128, 256, seed=7)
    with pytest.raises(mx.MXFP8Error) as e:
        mx.gemm_quantize("fprop", _dev(a_q), _dev(a_s), _dev(b_q), _dev(b_s))
    assert e.value.code == 2

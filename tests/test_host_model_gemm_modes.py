"""The MXFP8 product with the element format of each operand chosen by the caller (Section 3.2.2: E4M3 or E5M2 per
tensor type) on the CPU execution model of the kernels: the format fields of the matrix instruction must reach the
right operand (the kernels feed B fragments as the instruction's first operand, A as its second)."""
import numpy as np
import pytest

import oracle
import scale_layout as sl
from paper_2506_08027_amd import synth_inputs as si
from test_host_model import MODES, hostmodel, put, run_case  # noqa: F401  (hostmodel is a fixture)

FMT = {0: "e4m3", 1: "e5m2"}


def _operands(M, N, K, ea, eb, seed):
    a = np.asarray(si.activations(M, K, seed=seed, bf16=False), np.float32)
    b = np.asarray(si.weights(N, K, seed=seed + 1, bf16=False), np.float32)
    return oracle.quantize_rowwise_mode(a, FMT[ea]) + oracle.quantize_rowwise_mode(b, FMT[eb])


def _run(hostmodel, tmp_path, M, N, K, ea, eb, ops, bf16=False, tiled=False, wg=0, tag="", **env):
    a_q, a_s, b_q, b_s = ops
    if tiled:
        a_s, b_s = sl.tile(a_s, filler=0xFF), sl.tile(b_s, filler=0xFF)
    names = [put(tmp_path, f"{n}{tag}.bin", v) for n, v in (("aq", a_q), ("as", a_s), ("bq", b_q), ("bs", b_s))]
    out = str(tmp_path / f"c{tag}.bin")
    line = (f"gemmmode 0 {M} {N} {K} {ea} {eb} {'bf16' if bf16 else 'f32'} {N} {' '.join(names)} {out}"
            + (" tiled" if tiled else "") + (f" wg={wg}" if wg else ""))
    _, calls = run_case(hostmodel, tmp_path, [line], **env)
    assert calls[0][0] == 0
    raw = np.fromfile(out, np.uint16 if bf16 else np.uint32).reshape(M, N)
    written = raw != (0xA5A5 if bf16 else 0xA5A5A5A5)
    val = (si.bf16_bits_to_f32(raw) if bf16 else raw.view(np.float32)).astype(np.float64)
    return val, written


@pytest.mark.parametrize("ea,eb", [(1, 0), (0, 1), (1, 1)], ids=["e5m2xe4m3", "e4m3xe5m2", "e5m2xe5m2"])
def test_gemm_modes_small_tiles(hostmodel, tmp_path, ea, eb):
    """Ragged one-tile-per-workgroup case and a resident case; FP32 and BF16 output; both scale layouts."""
    for i, (M, N, K, bf16, tiled, wg) in enumerate([(200, 136, 384, False, False, 0), (256, 384, 256, True, True, 2)]):
        ops = _operands(M, N, K, ea, eb, seed=60 + i)
        val, written = _run(hostmodel, tmp_path, M, N, K, ea, eb, ops, bf16, tiled, wg, tag=str(i), **MODES[3 * i])
        assert written.all()
        ref, absum = oracle.gemm_mode(ops[0], ops[1], FMT[ea], ops[2], ops[3], FMT[eb])
        tol = max(K // 128, 2) * 2.0 ** -24 * absum + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0) + 1e-300
        assert (np.abs(val - ref) <= tol).all()
        if ea != eb:   # the same bytes read with the formats swapped give another product: the fields are not symmetric
            wrong, _ = oracle.gemm_mode(ops[0], ops[1], FMT[eb], ops[2], ops[3], FMT[ea])
            with np.errstate(invalid="ignore"):
                assert (~(np.abs(val - wrong) <= tol)).mean() > 0.5   # NaN (a code the other table reads as NaN) counts as different


def test_gemm_modes_large_tiles_sampled_workgroups(hostmodel, tmp_path):
    M, N, K = 2048, 4096, 384
    ops = _operands(M, N, K, 1, 0, seed=70)
    val, written = _run(hostmodel, tmp_path, M, N, K, 1, 0, ops, bf16=True, tiled=True, wg=64, WAVESIM_BLOCKS=2)
    rows = np.unique(np.nonzero(written)[0])
    assert written.sum() == 4 * 256 * 256
    ref, absum = oracle.gemm_mode(ops[0][rows], ops[1][rows], "e5m2", ops[2], ops[3], "e4m3")
    w = written[rows]
    tol = 3 * 2.0 ** -24 * absum + 2.0 ** -8 * np.abs(ref) + 1e-300
    assert (np.abs(val[rows] - ref)[w] <= tol[w]).all()

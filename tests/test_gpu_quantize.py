"""GPU parity of mxfp8_quantize / mxfp8_dequantize against the CPU oracle: every byte must match.
All calls go through the C ABI (ctypes binding); inputs are the seeded synthetic tensors."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_08027_amd as mx
from paper_2506_08027_amd import synth_inputs as si

pytestmark = pytest.mark.gpu


def _to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def _check_quantize(host: np.ndarray, axis: str, dev=None):
    dev = _to_dev(host) if dev is None else dev
    out = mx.quantize(dev, axis)
    torch.cuda.synchronize()
    if axis in ("rowwise", "both"):
        q, s = oracle.quantize_rowwise(host)
        gs, gq = out["s_row"].cpu().numpy(), out["q_row"].cpu().numpy()
        assert np.array_equal(gs, s), f"row scales differ at {np.argwhere(gs != s)[:5]}"
        assert np.array_equal(gq, q), f"row elements differ at {np.argwhere(gq != q)[:5]}"
    if axis in ("colwise", "both"):
        qT, sT = oracle.quantize_colwise(host)
        gs, gq = out["s_colT"].cpu().numpy(), out["q_colT"].cpu().numpy()
        assert np.array_equal(gs, sT), f"col scales differ at {np.argwhere(gs != sT)[:5]}"
        assert np.array_equal(gq, qT), f"col elements differ at {np.argwhere(gq != qT)[:5]}"
    return out


@pytest.mark.parametrize("axis", ["rowwise", "colwise", "both"])
def test_tiny_config_with_special_blocks(axis):
    _check_quantize(si.tiny_with_specials(256, 0), axis)


@pytest.mark.parametrize("axis", ["rowwise", "colwise", "both"])
@pytest.mark.parametrize("shape", [(32, 32), (96, 160), (352, 416), (128, 2048), (1056, 96)])
def test_bf16_activations_ragged_tiles(shape, axis):
    _check_quantize(si.activations(*shape, seed=2), axis)


@pytest.mark.parametrize("axis", ["rowwise", "colwise", "both"])
@pytest.mark.parametrize("shape", [(32, 32), (224, 96), (160, 352), (64, 1024)])
def test_fp32_gradients_ragged_tiles(shape, axis):
    _check_quantize(si.gradients(*shape, seed=3, spikes=True), axis)
    _check_quantize(si.activations(*shape, seed=4, bf16=False), axis)


def test_leading_dimension():
    host = si.activations(64, 256, seed=5)
    dev = _to_dev(host)
    view_h = host[:, 64:192]
    _check_quantize(np.ascontiguousarray(view_h), "both", dev=dev[:, 64:192])
    hostf = si.gradients(96, 160, seed=6)
    devf = _to_dev(hostf)
    _check_quantize(np.ascontiguousarray(hostf[:, 32:96]), "both", dev=devf[:, 32:96])


def test_every_bf16_pattern_under_several_scales():
    """All 65536 BF16 patterns (NaN and Inf included) as block elements. Patterns are grouped by
    magnitude, and a pivot element 2^d times larger than the group puts the same values into the
    top binade, the middle and the subnormal range of E4M3 in turn."""
    bits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    order = bits[np.argsort(bits & 0x7FFF, kind="stable")]
    pad = (-len(order)) % 31
    blk = np.concatenate([order, np.zeros(pad, np.uint16)]).reshape(-1, 31)
    top = (blk & 0x7FFF).max(axis=1).astype(np.uint32)
    for d in (0, 1, 3, 6, 9, 13, 40):
        pivot = np.where(top >= 0x7F80, top, np.minimum(top + (d << 7), 0x7F7F)).astype(np.uint16)
        src = np.concatenate([blk, pivot[:, None]], axis=1)
        rows = (-src.shape[0]) % 32
        src = np.ascontiguousarray(np.concatenate([src, np.zeros((rows, 32), np.uint16)], axis=0))
        _check_quantize(src, "both")


def test_fp32_scale_boundaries_and_rounding_ties():
    """FP32 blocks whose amax walks across 448*2^k (every mantissa near 1.75, several exponents,
    the lower clamp and the largest finite values), and elements on every E4M3 tie point."""
    blocks = []
    rng = np.random.default_rng(1)
    for e in (1, 7, 8, 9, 60, 127, 135, 200, 254):
        for m in list(range(0x600000 - 40, 0x600000 + 40)) + [0, 1, 0x7FFFFF, 0x400000]:
            amax = np.array([(e << 23) | m], np.uint32).view(np.float32)[0]
            v = (rng.uniform(-1, 1, 32).astype(np.float32) * amax).astype(np.float32)
            v[rng.integers(32)] = amax
            blocks.append(v)
    vals = np.array([oracle.e4m3_decode(c) for c in range(0x7F)])
    mids = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)
    ties = np.concatenate([mids, np.nextafter(mids, np.float32(1e9)), np.nextafter(mids, np.float32(0))])
    ties = np.concatenate([ties, -ties])
    for k in (-100, -1, 0, 30, 118):
        t = (ties.astype(np.float64) * 2.0 ** k).astype(np.float32)
        pad = (-len(t)) % 31
        t = np.concatenate([t, np.zeros(pad, np.float32)]).reshape(-1, 31)
        piv = np.full((t.shape[0], 1), np.float32(448.0 * 2.0 ** k), np.float32)
        for row in np.concatenate([t, piv], axis=1):
            blocks.append(row)
    sub = (rng.integers(0, 1 << 23, (64, 32)).astype(np.uint32) | (rng.integers(0, 2, (64, 32)).astype(np.uint32) << 31))
    blocks.extend(list(sub.view(np.float32)))
    src = np.stack(blocks).astype(np.float32)
    src = np.concatenate([src, np.zeros(((-len(src)) % 32, 32), np.float32)])
    _check_quantize(np.ascontiguousarray(src), "both")


def test_empty_and_error_codes():
    dev = torch.zeros((64, 64), dtype=torch.float32, device="cuda")
    mx.quantize(dev[:0], "both")
    mx.quantize(dev[:, :0], "rowwise")
    with pytest.raises(mx.MXFP8Error) as e:
        mx.quantize(dev[:33], "rowwise")
    assert e.value.code == 2
    with pytest.raises(mx.MXFP8Error) as e:
        mx.quantize(dev[:, :48], "colwise")
    assert e.value.code == 2
    q = torch.empty((64, 64), dtype=torch.uint8, device="cuda")
    s = torch.empty((64, 2), dtype=torch.uint8, device="cuda")
    with pytest.raises(mx.MXFP8Error) as e:
        mx.mxfp8_quantize(dev, "both", q, s, None, None)
    assert e.value.code == 1
    with pytest.raises(mx.MXFP8Error) as e:          # misaligned source (offset by one float)
        mx.mxfp8_quantize(dev.view(-1)[1:1 + 32 * 32].view(32, 32), "rowwise", q[:32, :32].contiguous(), s[:32, :1].contiguous())
    assert e.value.code == 3
    with pytest.raises(KeyError):
        mx.quantize(dev, "diagonal")
    torch.cuda.synchronize()


# ---- dequantize ---------------------------------------------------------------------------------

def _check_dequantize(q: np.ndarray, s: np.ndarray):
    dq, ds = torch.from_numpy(q).cuda(), torch.from_numpy(s).cuda()
    want32 = oracle.dequantize(q, s, "f32")
    got32 = mx.dequantize(dq, ds, torch.float32).cpu().numpy()
    nan = np.isnan(want32)
    assert np.array_equal(np.isnan(got32), nan)
    assert np.array_equal(got32.view(np.uint32)[~nan], want32.view(np.uint32)[~nan])
    want16 = oracle.dequantize(q, s, "bf16")
    got16 = mx.dequantize(dq, ds, torch.bfloat16).view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal((got16 & 0x7FFF) > 0x7F80, nan)
    assert np.array_equal(got16[~nan], want16[~nan])


def test_dequantize_every_code_under_every_scale():
    codes = np.tile(np.arange(256, dtype=np.uint8).reshape(8, 32), (256, 1))      # [2048 x 32]
    scales = np.repeat(np.arange(256, dtype=np.uint8), 8).reshape(-1, 1)
    _check_dequantize(np.ascontiguousarray(codes), np.ascontiguousarray(scales))


def test_dequantize_round_trip_of_quantized_tensors():
    for host in (si.activations(96, 160, seed=2), si.gradients(64, 224, seed=3, spikes=True),
                 si.tiny_with_specials(256, 0)):
        out = mx.quantize(_to_dev(host), "both")
        q, s = oracle.quantize_rowwise(host)
        _check_dequantize(q, s)
        qT, sT = oracle.quantize_colwise(host)
        _check_dequantize(qT, sT)
        # device round trip through the device's own bytes, with a padded destination
        dst = torch.full((q.shape[0], q.shape[1] + 32), -7.0, dtype=torch.float32, device="cuda")
        mx.mxfp8_dequantize(out["q_row"], out["s_row"], dst[:, :q.shape[1]])
        want = oracle.dequantize(q, s, "f32")
        got = dst.cpu().numpy()
        nan = np.isnan(want)
        assert np.array_equal(got[:, :q.shape[1]][~nan], want[~nan]) and np.all(got[:, q.shape[1]:] == -7.0)


@pytest.mark.parametrize("which", ["act_bf16", "grad_fp32"])
def test_full_size_quantize_sweep_config(which):
    """The 8B-class quantize configuration at full size, in the launch shape the benchmark times:
    every byte of both copies against the oracle."""
    if which == "act_bf16":
        host = si.activations(8192, 4096, seed=2)
    else:
        host = si.gradients(8192, 14336, seed=3)
    _check_quantize(host, "both")

"""GPU parity of the single-copy path (Section 5 names the two stored copies per tensor as the overhead to
remove): the column copy derived from a kept row copy must equal the oracle's byte for byte. Calls go through
the C ABI."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2506_08027_amd as mx
import scale_layout as sl
from paper_2506_08027_amd import synth_inputs as si

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _check(x, tiled):
    q, s = oracle.quantize_rowwise(x)
    lay = mx.SCALES_TILED if tiled else mx.SCALES_ROWMAJOR
    out = mx.requantize_colwise(_dev(q), _dev(sl.tile(s) if tiled else s), lay)
    torch.cuda.synchronize()
    qT, sT = oracle.requantize_colwise(q, s)
    assert np.array_equal(out["q_colT"].cpu().numpy(), qT)
    got_s = out["s_colT"].cpu().numpy()
    assert np.array_equal(sl.untile(got_s, *sT.shape) if tiled else got_s, sT)


@pytest.mark.parametrize("tiled", [False, True])
def test_requantize_tiny_configuration_with_every_special_block(tiled):
    _check(si.tiny_with_specials(256, seed=0), tiled)
    _check(np.ascontiguousarray(si.tiny_with_specials(256, seed=1)[:160, :224]), tiled)      # ragged tiles


@pytest.mark.parametrize("tiled", [False, True])
def test_requantize_llm_shaped_tensors(tiled):
    _check(np.asarray(si.activations(512, 1024, seed=2, bf16=False), np.float32), tiled)
    _check(si.gradients(384, 768, seed=5, spikes=True), tiled)


def test_requantize_equals_gpu_quantize_of_the_decoded_tensor_at_full_size():
    """[8192 x 4096] activations, tiled scales: the derived column copy is the GPU's own column quantization of
    the GPU's own FP32 decode of the row copy (each of which is byte-exact against the oracle at this size)."""
    lay = mx.SCALES_TILED
    x = torch.from_numpy(si.activations(8192, 4096, seed=2).view(np.int16)).cuda().view(torch.bfloat16)
    row = mx.quantize(x, "rowwise", scale_layout=lay)
    derived = mx.requantize_colwise(row["q_row"], row["s_row"], lay)
    decoded = mx.dequantize(row["q_row"], row["s_row"], torch.float32, scale_layout=lay)
    direct = mx.quantize(decoded, "colwise", scale_layout=lay)
    torch.cuda.synchronize()
    assert torch.equal(derived["q_colT"], direct["q_colT"]) and torch.equal(derived["s_colT"], direct["s_colT"])


def test_requantize_error_codes():
    q = torch.zeros((64, 64), dtype=torch.uint8, device="cuda")
    s = torch.zeros((64, 2), dtype=torch.uint8, device="cuda")
    with pytest.raises(mx.MXFP8Error):
        mx.mxfp8_requantize_colwise_ex(q[:48], s[:48], torch.empty((64, 48), dtype=torch.uint8, device="cuda"),
                                       torch.empty((64, 1), dtype=torch.uint8, device="cuda"))   # 48 rows: no whole column block

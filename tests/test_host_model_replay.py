"""Replays the GPU parity tests on the CPU execution model (see tests/host_model/replay_plugin.py): the
test files of the `gpu` marker run unchanged, in a child pytest process whose binding loads the
host-model build of the library. Everything that fits the model's speed is selected: the exactness,
special-value, ragged-shape, all-BF16-pattern, error-code and tolerance tests; the full-size cases are
left to the GPU. A failure here means the GPU run would fail
for a reason that has nothing to do with the hardware (a bug in a test or in a kernel's logic)."""
import os
import re
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
MODEL_DIR = os.path.join(HERE, "host_model")
LIB = os.path.join(MODEL_DIR, "_build", "libmxfp8_hostmodel.so")


@pytest.fixture(scope="module")
def hostmodel_lib():
    res = subprocess.run([os.path.join(MODEL_DIR, "build.sh"), "--shared", LIB], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-4000:]
    return LIB


def replay(lib, files, select, extra_env=None):
    env = dict(os.environ, MXFP8_HOSTMODEL_LIB=lib,
               PYTHONPATH=os.pathsep.join([MODEL_DIR, ROOT, os.environ.get("PYTHONPATH", "")]))
    env.update(extra_env or {})
    res = subprocess.run([sys.executable, "-m", "pytest", "-p", "no:cacheprovider", "-p", "replay_plugin", "-q", "-x",
                          "-m", "gpu", "-k", select] + [os.path.join(HERE, f) for f in files],
                         capture_output=True, text=True, cwd=ROOT, env=env, timeout=1500)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    m = re.search(r"(\d+) passed", res.stdout)
    assert m, tail
    return int(m.group(1))


def test_gpu_parity_tests_pass_on_the_host_model(hostmodel_lib):
    n = replay(hostmodel_lib, ["test_gpu_quantize.py", "test_gpu_quantize_modes.py", "test_gpu_gemm.py"],
               "not full_size and not transformer_layer")
    assert n >= 50


def test_layout_persistent_and_fused_gpu_tests_pass_on_the_host_model(hostmodel_lib):
    """The parity tests of the tiled scale layout, the persistent kernel and the fused output quantization:
    everything but the cases whose size the model cannot run in minutes (the full-size layer and the
    2048 x 4096 / 4352 x 4096 problems, which were replayed once by hand)."""
    n = replay(hostmodel_lib, ["test_gpu_scale_layouts_persistent_fused.py"],
               "not full_size and not (quantize_tiled_matches and shape4) and not (gemm_tiled_matches and shape3) "
               "and not (persistent_gemm_matches and (shape2 or shape3 or shape4)) "
               "and not (fused_output and (shape2 or shape3))")
    assert n >= 34


def test_simulated_path_gpu_tests_pass_on_the_host_model(hostmodel_lib):
    """The BF16 product and the round trip of the simulated path; the long-K, 2048 x 4096 and full-size cases
    are left to the GPU."""
    n = replay(hostmodel_lib, ["test_gpu_simulated.py"],
               "not full_size and not (matches_oracle and (shape3 or shape4 or shape5)) and not (small_integers and shape7)")
    assert n >= 18


def test_grouped_gpu_tests_pass_on_the_host_model(hostmodel_lib):
    """The grouped (mixture-of-experts) product; the 4096-token and full-size cases are left to the GPU."""
    n = replay(hostmodel_lib, ["test_gpu_grouped.py"], "not full_size and not equals_the_plain_product")
    assert n >= 6


def test_single_copy_gpu_tests_pass_on_the_host_model(hostmodel_lib):
    n = replay(hostmodel_lib, ["test_gpu_single_copy.py"], "not full_size")
    assert n >= 5


def test_fp4_gpu_tests_pass_on_the_host_model(hostmodel_lib):
    """MXFP4 conversion and product; the full-size and 2048 x 4096 cases are left to the GPU."""
    n = replay(hostmodel_lib, ["test_gpu_fp4.py"], "not full_size and not large_tiles")
    assert n >= 28


def test_matrix_instruction_layout_tests_pass_on_the_host_model(hostmodel_lib):
    """The facts about the scaled matrix instruction that the GPU test pins on the hardware hold for the CPU
    model of the instruction as well: the two cannot drift apart."""
    n = replay(hostmodel_lib, ["test_gpu_mfma_layout.py"], "layout or scale or operand")
    assert n >= 7


def test_fp6_gpu_tests_pass_on_the_host_model(hostmodel_lib):
    """MXFP6 conversion, expansion and product; the full-size case is left to the GPU."""
    n = replay(hostmodel_lib, ["test_gpu_fp6.py"], "not full_size")
    assert n >= 31


def test_gemm_mode_gpu_tests_pass_on_the_host_model(hostmodel_lib):
    n = replay(hostmodel_lib, ["test_gpu_gemm_modes.py"], "not nothing")
    assert n >= 12

"""Replays the GPU parity tests on the CPU execution model (see tests/host_model/replay_plugin.py): the
test files of the `gpu` marker run unchanged, in a child pytest process whose binding loads the
host-model build of the library. Everything that fits the model's speed is selected: the exactness,
special-value, ragged-shape, all-BF16-pattern, error-code and tolerance tests; the full-size cases are
left to the GPU. A failure here means the GPU run would fail
for a reason that has nothing to do with the hardware (a bug in a test or in a kernel's logic).
The child processes are independent of one another, so all of them are started when the first replay test runs
and each test then waits for its own: the module takes as long as its longest replay, not the sum."""
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
def hostmodel_lib(request):
    proc = getattr(request.config, "_hostmodel_shared_build", None)   # started by conftest.py when collection ended
    if proc is not None:
        out, _ = proc.communicate()
        assert proc.returncode == 0, out[-4000:]
    else:
        res = subprocess.run([os.path.join(MODEL_DIR, "build.sh"), "--shared", LIB], capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-4000:]
    return LIB


# name -> (test files, -k selection, least number of tests that must have run)
PLAN = {
    "core": (("test_gpu_quantize.py", "test_gpu_quantize_modes.py", "test_gpu_gemm.py"),
             "not full_size and not transformer_layer", 50),
    # everything but the cases whose size the model cannot run in minutes (the full-size layer and the
    # 2048 x 4096 / 4352 x 4096 problems, which were replayed once by hand)
    "layouts": (("test_gpu_scale_layouts_persistent_fused.py",),
                "not full_size and not (quantize_tiled_matches and shape4) and not (gemm_tiled_matches and shape3) "
                "and not (persistent_gemm_matches and (shape2 or shape3 or shape4)) "
                "and not (fused_output and (shape2 or shape3))", 34),
    # the long-K, 2048 x 4096 and full-size cases are left to the GPU
    "simulated": (("test_gpu_simulated.py",),
                  "not full_size and not (matches_oracle and (shape3 or shape4 or shape5)) and not (small_integers and shape7)", 18),
    "grouped": (("test_gpu_grouped.py",), "not full_size and not equals_the_plain_product", 6),
    "single_copy": (("test_gpu_single_copy.py",), "not full_size", 5),
    "fp4": (("test_gpu_fp4.py",), "not full_size and not large_tiles", 28),
    "mfma_layout": (("test_gpu_mfma_layout.py",), "layout or scale or operand", 7),
    "fp6": (("test_gpu_fp6.py",), "not full_size", 31),
    "gemm_modes": (("test_gpu_gemm_modes.py",), "not nothing", 12),
}
_RUNNING = {}   # name -> child process; all of them are started by the first call of replay()


def _start(lib, files, select):
    env = dict(os.environ, MXFP8_HOSTMODEL_LIB=lib,
               PYTHONPATH=os.pathsep.join([MODEL_DIR, ROOT, os.environ.get("PYTHONPATH", "")]))
    for var in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS"):
        env[var] = "2"   # nine children side by side: the oracle's and numpy's thread pools must not each take every core
    return subprocess.Popen([sys.executable, "-m", "pytest", "-p", "no:cacheprovider", "-p", "replay_plugin", "-q", "-x",
                             "-m", "gpu", "-k", select] + [os.path.join(HERE, f) for f in files],
                            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, cwd=ROOT, env=env)


@pytest.fixture(scope="module", autouse=True)
def _reap_children():
    yield
    for proc in _RUNNING.values():   # a failure with -x leaves the other replays running
        if proc.poll() is None:
            proc.kill()


def replay(lib, name):
    if not _RUNNING:
        for key, (files, select, _) in PLAN.items():
            _RUNNING[key] = _start(lib, files, select)
    proc = _RUNNING[name]
    try:
        out, _ = proc.communicate(timeout=2400)
    except subprocess.TimeoutExpired:
        proc.kill()
        raise
    tail = out[-3000:]
    assert proc.returncode == 0, tail
    m = re.search(r"(\d+) passed", out)
    assert m, tail
    assert int(m.group(1)) >= PLAN[name][2], tail


@pytest.mark.parametrize("name", list(PLAN))
def test_gpu_parity_tests_pass_on_the_host_model(hostmodel_lib, name):
    """core: quantize / dequantize / GEMM parity; layouts: tiled scales, resident kernel, fused output quantization;
    simulated: the BF16 product and round trip of the simulated path; grouped: mixture-of-experts products;
    single_copy: the derived column copy; fp4 / fp6: the narrow formats; mfma_layout: the facts about the scaled matrix
    instruction that the GPU test pins on the hardware hold for the CPU model of the instruction as well (the two
    cannot drift apart); gemm_modes: per-operand element formats."""
    replay(hostmodel_lib, name)

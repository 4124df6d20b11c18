import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--runslow", action="store_true", default=False,
                     help="also run the tests marked slow (the full mutation checks, the long cases of the kernels' CPU execution model)")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")
    config.addinivalue_line("markers", "slow: long-running (minutes); runs only with --runslow")


# Cases of the CPU execution model of the kernels (tests/test_host_model*.py) that run only with --runslow: the
# second execution-order / scale-layout variant of a case whose first variant stays in the default run, and the
# sampled-workgroup cases of the 256 x 256 configuration but one. They take 5 .. 20 s each (six minutes together);
# the default run keeps one case per kernel family, and the GPU parity tests replayed on the model
# (tests/test_host_model_replay.py) walk the same kernels again. Before a changed kernel goes to a GPU: --runslow.
SLOW_HOST_MODEL_CASES = (
    "test_fp4_gemm_persistent_small_tiles[eager-down-tiled]", "test_fp4_gemm_persistent_large_tiles", "test_fp4_gemm_large_tiles_ragged",
    "test_fp4_gemm_small_tiles_ragged[lazy-up-rowmajor]", "test_fp4_gemm_small_tiles_ragged[lazy-down-rowmajor]",
    "test_fp4_gemm_small_tiles_ragged[eager-up-tiled]",
    "test_fused_output_quantization_large_tiles", "test_gemm_large_tiles_sampled_workgroups",
    "test_gemm_persistent_large_tiles_sampled_workgroups[False-down]", "test_gemm_tiled_scales_large_tiles",
    "test_gemm_persistent_small_tiles[eager-down-tiled]", "test_gemm_small_tiles_ragged[eager-down]",
    "test_fused_output_quantization_small_tiles[3-", "test_gemm_tiled_scales_small_tiles[eager-down]",
    "test_grouped_wgrad_small_tiles[eager-down-tiled]", "test_grouped_large_tiles",
    "test_grouped_small_tiles_partial_and_empty_experts[eager-down]", "test_grouped_small_tiles_partial_and_empty_experts[lazy-up]",
    "test_bf16_gemm_persistent_small_tiles[eager-down]", "test_bf16_gemm_persistent_large_tiles", "test_bf16_gemm_large_tiles_ragged",
    "test_bf16_gemm_small_tiles_ragged[eager-down]",
    "test_gemm_modes_large_tiles", "test_gemm_modes_small_tiles[e5m2xe5m2]", "test_gemm_modes_small_tiles[e4m3xe5m2]",
)


def pytest_collection_modifyitems(config, items):
    for item in items:
        if "test_host_model" in item.nodeid and any(case in item.nodeid for case in SLOW_HOST_MODEL_CASES):
            item.add_marker(pytest.mark.slow)
    if config.getoption("--runslow"):
        return
    skip = pytest.mark.skip(reason="slow: run with --runslow")
    for item in items:
        if "slow" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


def pytest_collection_finish(session):
    """The replayed GPU tests need the optimised shared build of the kernels' CPU model (a minute of compilation):
    started here, in the background, as soon as it is known that they will run; their fixture waits for it."""
    if session.config.option.collectonly or not any("test_host_model_replay" in item.nodeid for item in session.items):
        return
    model = os.path.join(ROOT, "tests", "host_model")
    session.config._hostmodel_shared_build = subprocess.Popen(
        [os.path.join(model, "build.sh"), "--shared", os.path.join(model, "_build", "libmxfp8_hostmodel.so")],
        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


def pytest_sessionfinish(session, exitstatus):
    proc = getattr(session.config, "_hostmodel_shared_build", None)
    if proc is not None and proc.poll() is None:   # the session ended before the replay tests asked for it
        proc.kill()

"""The C ABI used without Python: paper_2506_08027_amd/examples/linear_layer_step.cpp quantizes X, W and dY, runs the
three products of a linear layer and the decode through libmxfp8.so alone and checks samples of every result on the
host against the block-scaled sums computed from the library's own bytes (its exit code says whether they agree)."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BINARY = os.path.join(ROOT, "paper_2506_08027_amd", "examples", "linear_layer_step")


@pytest.mark.skipif("MXFP8_HOSTMODEL_LIB" in os.environ, reason="a compiled GPU program: hardware only")
@pytest.mark.parametrize("sizes", [(), ("2048", "1024", "1536")])
def test_linear_layer_step_through_the_c_abi(sizes):
    assert os.path.exists(BINARY), "build it first: python -c 'import __graft_entry__ as g; g.build()'"
    res = subprocess.run([BINARY, *sizes], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "linear layer step ok" in res.stdout

"""Runs the two mutation checks as tests, so that "every planted mistake is caught" can be reproduced:
oracle/mutation_check.py plants single plausible mistakes in the oracle's C source and expects the pins
(tests/test_oracle_pins.py, tests/test_oracle_modes.py) to fail; tests/host_model/mutation_check.py does the
same to the GEMM kernels on the CPU execution model. The full sets take tens of minutes and run only with
`--runslow` (`python -m pytest tests/test_mutation_checks.py --runslow`); a three-mutant sample of the oracle
check runs every time."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(script, *select, timeout):
    res = subprocess.run([sys.executable, os.path.join(ROOT, script), *select], cwd=ROOT, capture_output=True,
                         text=True, timeout=timeout)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "SURVIVED" not in res.stdout, tail
    return res.stdout


def test_oracle_pins_catch_a_sample_of_planted_mistakes():
    out = _run("oracle/mutation_check.py", "encode: ties toward zero", "scale: round down (OCP", "gemm: abs-sum",
               timeout=600)
    assert "3 of 3 killed" in out


@pytest.mark.slow
def test_oracle_pins_catch_every_planted_mistake():
    out = _run("oracle/mutation_check.py", timeout=3000)
    assert " of 52 killed" in out and "52 of 52" in out


@pytest.mark.slow
def test_host_model_catches_every_planted_kernel_mistake():
    _run("tests/host_model/mutation_check.py", timeout=3400)

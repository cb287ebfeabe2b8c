"""The C ABI from a plain host program: hipMalloc'd buffers, its own stream, no Python in the
process.  The program (paper_2205_00119_amd/examples/step_from_c.cpp, built by build()) checks every
result against a closed form itself; here it only has to run and say so."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROGRAM = os.path.join(ROOT, "paper_2205_00119_amd", "examples", "step_from_c")


def test_a_step_through_the_c_abi_without_python():
    if not os.path.exists(PROGRAM):
        pytest.skip("the example program is not built (build() compiles it)")
    res = subprocess.run([PROGRAM], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    for step in ("gather-reorder", "reduce-scatter-accumulate", "replica-average", "adam-shard", "error path"):
        assert f"ok {step}" in res.stdout, res.stdout
    assert "all checks passed" in res.stdout

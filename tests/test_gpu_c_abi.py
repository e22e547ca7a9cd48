"""The C ABI used from a plain C program (tests/c_abi_check.c, built by __graft_entry__.build()):
no Python binding and no torch between the caller and the library."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def test_c_program_runs_the_outer_step_and_matches_the_oracle():
    exe = os.path.join(HERE, "c_abi_check")
    if not os.path.exists(exe):
        pytest.skip("tests/c_abi_check is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "agree" in out.stdout

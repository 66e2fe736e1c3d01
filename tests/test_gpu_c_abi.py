"""The C ABI driven by a plain HIP host program (tests/c_abi/round.cpp, built by
__graft_entry__.build()): no Python and no torch between the caller and the library."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "round")


def test_c_program_round_matches_oracle():
    assert os.path.exists(EXE), "tests/c_abi/round is not built - run __graft_entry__.build()"
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "c-abi round ok" in r.stdout

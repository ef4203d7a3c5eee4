"""Runs the torch-free C++ caller of the C ABI (tests/c_abi/c_abi_check.cpp): attention and accept through
plain HIP allocations, compared in the program itself with the float64 C oracle."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "c_abi_check")


def test_c_program_matches_oracle():
    assert os.path.exists(EXE), "tests/c_abi/c_abi_check is not built: run __graft_entry__.build() (or tests/c_abi/build.py)"
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(r.stdout)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "PASSED" in r.stdout

"""Runs the plain C program tests/c_abi_roundtrip (no Python, no PyTorch in
the process): the C ABI works for a caller that only has the HIP runtime."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))


def test_c_program_round_trip():
    exe = os.path.join(HERE, "c_abi_roundtrip")
    if not os.path.exists(exe):
        pytest.skip("tests/c_abi_roundtrip has not been built (python -m tests.build_c_check)")
    out = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert out.returncode == 0, out.stdout
    assert "C ABI round trip OK" in out.stdout

"""The C ABI used from a plain C++ program (tests/c_abi_client.cpp): HIP runtime + granq.h only."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def test_c_client_runs_the_worked_examples():
    exe = os.path.join(HERE, "c_abi_client.bin")
    assert os.path.exists(exe), "build it first: python -c 'import __graft_entry__ as g; g.build()'"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "c_abi_client ok" in r.stdout

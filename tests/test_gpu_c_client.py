"""The C ABI used from a plain C++ program (tests/c_abi_client.cpp): HIP runtime + granq.h only."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def test_c_client_runs_the_worked_examples():
    exe = os.path.join(HERE, "c_abi_client.bin")
    if not os.path.exists(exe):                  # normally built beforehand by __graft_entry__.build()
        import sys
        sys.path.insert(0, os.path.dirname(HERE))
        import __graft_entry__
        __graft_entry__.build_c_client()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "c_abi_client ok" in r.stdout

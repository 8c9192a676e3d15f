"""The library's five-operation quotient, compiled for the host from the
product's own header, against the correctly rounded division (tests/quotient_check.cpp)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_fast_quotient_matches_true_division(tmp_path):
    exe = str(tmp_path / "quotient_check")
    subprocess.run(["g++", "-O2", "-ffp-contract=off", "-I", os.path.join(ROOT, "paper_2503_18339_amd", "csrc"),
                    os.path.join(ROOT, "tests", "quotient_check.cpp"), "-o", exe, "-lm"], check=True)
    out = subprocess.run([exe, "4000000"], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout[-2000:]
    assert "0 quotient mismatches, 0 code mismatches" in out.stdout

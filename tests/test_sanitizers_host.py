"""Address- and undefined-behaviour-sanitizer builds of everything that runs on the host
(no GPU): the CPU oracle under its pins, the library's exact quotient against true
division, and a replay of every index the library's launch plans produce."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2503_18339_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


def _env():
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    return env


def test_launch_plans_stay_inside_tensor_and_workspace(tmp_path):
    exe = str(tmp_path / "plan_check")
    subprocess.run(["g++", "-O1", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                    os.path.join(ROOT, "tests", "plan_check.cpp"), "-o", exe], check=True)
    out = subprocess.run([exe], capture_output=True, text=True, env=_env())
    assert out.returncode == 0, (out.stdout[-3000:], out.stderr[-3000:])
    assert ", 0 failures" in out.stdout


def test_fast_quotient_under_sanitizers(tmp_path):
    exe = str(tmp_path / "quotient_check")
    subprocess.run(["g++", "-O1", "-ffp-contract=off", *SAN, "-I", CSRC,
                    os.path.join(ROOT, "tests", "quotient_check.cpp"), "-o", exe, "-lm"], check=True)
    out = subprocess.run([exe, "300000"], capture_output=True, text=True, env=_env())
    assert out.returncode == 0, (out.stdout[-2000:], out.stderr[-3000:])
    assert "0 quotient mismatches, 0 code mismatches" in out.stdout


def test_oracle_pins_through_the_sanitized_oracle(tmp_path):
    """The oracle, instrumented, runs every pin in a child interpreter (the sanitizer's runtime
    has to be loaded before the interpreter starts)."""
    import oracle
    lib = str(tmp_path / "libgranq_oracle_san.so")
    oracle.build(out=lib, extra_flags=SAN)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc has no libasan"
    env = _env()
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["PYTHONPATH"] = os.pathsep.join([ROOT, os.path.join(ROOT, "tests"), env.get("PYTHONPATH", "")])
    code = ("import sys, oracle, oracle_pins\n"
            "lib = oracle.load(sys.argv[1])\n"
            "for check in oracle_pins.ALL_CHECKS:\n"
            "    check(lib)\n"
            "    print('ok', check.__name__, flush=True)\n"
            "print('ALL PINS PASSED')\n")
    out = subprocess.run([sys.executable, "-c", code, lib], capture_output=True, text=True, env=env)
    assert out.returncode == 0 and "ALL PINS PASSED" in out.stdout, (out.stdout[-2000:], out.stderr[-4000:])
    assert "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr, out.stderr[-4000:]

"""bench.py's command line on a machine without a GPU: refusals are explicit."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""


def test_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        return
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode != 0 and "no CPU fallback" in r.stderr


def test_trace_summary_lists_kernels_and_filters_by_name(tmp_path):
    """The rocprofv3 --stats summariser: every kernel above 0.05 % by default, only the matching ones
    (however small) with a filter."""
    from paper_2503_18339_amd import profiling
    csv_text = ('"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n'
                '"void granq::fq_bwd_cols<granq::F32, 1, 1, false, 0>(int)",4,528000,132000,90.0,1,2,0\n'
                '"naive_conv_search_kernel",2,58000,29000,9.97,1,2,0\n'
                '"void granq::prescale_kernel(float const*)",5,200,40,0.03,1,2,0\n')
    p = tmp_path / "stats.csv"
    p.write_text(csv_text)
    plain = profiling.summarise_trace(str(p))
    assert "fq_bwd_cols<F32, 1, 1, false, 0>" in plain and "naive_conv_search_kernel" in plain
    assert "prescale_kernel" not in plain                      # below 0.05 %
    only = profiling.summarise_trace(str(p), "granq")
    assert "fq_bwd_cols" in only and "prescale_kernel" in only and "naive_conv" not in only

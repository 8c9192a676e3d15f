"""Build the GranQ HIP library for gfx950 with hipcc (in-tree, no JIT cache)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libgranq.so")
SOURCES = [os.path.join(CSRC, "granq_kernels.hip"), os.path.join(CSRC, "granq_compare.hip"),
           os.path.join(CSRC, "granq_rowwise.hip"),
           os.path.join(CSRC, "granq_metrics.hip"),
           os.path.join(CSRC, "granq_conv.hip"),
           os.path.join(CSRC, "granq_fconv.hip"),
           os.path.join(CSRC, "granq_fused.hip")]
HEADERS = [os.path.join(CSRC, "granq_device.h"), os.path.join(CSRC, "granq_plan.h"),
           os.path.join(CSRC, "granq_block.h"), os.path.join(CSRC, "granq_pixels.h"), os.path.join(CSRC, "granq_launch.h"), os.path.join(CSRC, "granq_internal.h"), os.path.join(CSRC, "granq_tiling.h"),
           os.path.join(CSRC, "granq_quotient.h"), os.path.join(INCLUDE, "granq.h"),
           os.path.join(INCLUDE, "granq_compare.h")]

# -ffp-contract=off: one rounding per source operation (no FMA contraction);
# correctly rounded float division is HIP's default and is stated explicitly;
# packed-FP32 instructions are switched off for the device code.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(out: str = LIB, defines=(), verbose: bool = False) -> str:
    """Compile the library.  ``defines`` are extra -D options (tuning builds)."""
    cmd = [hipcc(), *HIPCC_FLAGS, "-I", INCLUDE, "-I", CSRC,
           *["-D" + d for d in defines], "-o", out, *SOURCES]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    res = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    # the host pass does not know the device-only target feature and says so once per
    # translation unit; everything else the compiler prints is passed on
    noise = "'-packed-fp32-ops' is not a recognized feature for this target"
    rest = [ln for ln in res.stderr.splitlines() if noise not in ln]
    if rest:
        print("\n".join(rest), file=sys.stderr)
    if res.returncode != 0:
        raise subprocess.CalledProcessError(res.returncode, cmd)
    return out


def is_stale(lib: str = LIB) -> bool:
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True))

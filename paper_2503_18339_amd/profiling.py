"""Turn rocprofv3 output of `bench.py` into the short summaries kept under
profiles/ and into the measured-traffic record that bench.py reports.

    python -m paper_2503_18339_amd.profiling trace  <bench_kernel_stats.csv>
    python -m paper_2503_18339_amd.profiling counters <fetch_counter_collection.csv> \
            <write_counter_collection.csv> --copy-bytes N [--write-record]

`counters` expects two `rocprofv3 --pmc` runs of `bench.py --pmc-calibration`
(FETCH_SIZE in one, WRITE_SIZE in the other; both counters are in KiB per
dispatch).  The calibration launches are plain device copies of N bytes; what
the counters read for them gives the factor that converts counter units into
bytes.  `--write-record` stores the per-launch traffic of the dominant kernel,
together with a hash of the kernel sources, in traffic_record.json next to this
file; bench.py reports it as `roofline.traffic` only while that hash still
matches the sources it runs.
"""
from __future__ import annotations

import argparse
import collections
import csv
import hashlib
import json
import os
import sys

from . import build as _build

RECORD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "traffic_record.json")
COPY_KERNEL = "__amd_rocclr_copyBuffer"


def source_hash() -> str:
    """Hash of everything that determines the code of the four-call kernels: their source,
    the device headers it includes and the compiler flags."""
    h = hashlib.sha256()
    names = ("granq_kernels.hip", "granq_device.h", "granq_plan.h", "granq_quotient.h", "granq_launch.h",
             "granq_internal.h")
    paths = [os.path.join(_build.CSRC, n) for n in names]
    for path in sorted(paths):
        with open(path, "rb") as fh:
            h.update(os.path.basename(path).encode())
            h.update(fh.read())
    h.update(" ".join(_build.HIPCC_FLAGS).encode())
    return h.hexdigest()[:16]


def _short(name: str) -> str:
    name = name.replace("granq::", "").replace("void ", "")
    cut = name.find("(")
    return name[:cut] if cut > 0 else name


def summarise_trace(stats_csv: str, match: str = "") -> str:
    """One line per kernel of a rocprofv3 --stats file.  `match`: a regular expression; only kernels
    whose name matches are listed (a run that also holds a framework's search or warm-up kernels),
    however small their share."""
    import re
    rows = list(csv.DictReader(open(stats_csv)))
    out = ["%-58s %7s %12s %10s %7s" % ("kernel", "calls", "avg_us", "total_ms", "%")]
    for r in rows:
        if match:
            if not re.search(match, r["Name"]):
                continue
        elif float(r["Percentage"]) < 0.05:
            continue
        out.append("%-58s %7d %12.2f %10.2f %7.2f" % (
            _short(r["Name"])[:58], int(r["Calls"]), float(r["AverageNs"]) / 1e3,
            float(r["TotalDurationNs"]) / 1e6, float(r["Percentage"])))
    return "\n".join(out)


def _per_kernel(counter_csv: str):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(counter_csv)):
        agg[(r["Kernel_Name"], int(r["Grid_Size"]))].append(float(r["Counter_Value"]))
    return agg


def summarise_counters(fetch_csv: str, write_csv: str, copy_bytes: int, dominant: str = "fq_bwd_cols"):
    fetch, write = _per_kernel(fetch_csv), _per_kernel(write_csv)

    def copy_reading(agg):
        vals = [max(v) for (k, _), v in agg.items() if k.startswith(COPY_KERNEL)]
        if not vals:
            raise SystemExit("no calibration copy kernel in the counter file")
        return max(vals)

    f_scale = copy_bytes / 1024.0 / copy_reading(fetch)
    w_scale = copy_bytes / 1024.0 / copy_reading(write)
    lines = ["calibration: plain device copy of %d bytes reads FETCH_SIZE %.1f KiB, WRITE_SIZE %.1f KiB"
             % (copy_bytes, copy_reading(fetch), copy_reading(write)),
             "             -> bytes = FETCH_SIZE * 1024 * %.4f,  bytes = WRITE_SIZE * 1024 * %.4f" % (f_scale, w_scale),
             "", "%-50s %12s %14s %14s" % ("kernel", "grid", "fetched MB", "written MB")]
    per_kernel = collections.defaultdict(lambda: [0.0, 0.0, 0])
    for (k, g), v in sorted(fetch.items(), key=lambda kv: -max(kv[1])):
        if "granq::" not in k:
            continue
        fb = sum(v) / len(v) * 1024 * f_scale
        wv = write.get((k, g), [0.0])
        wb = sum(wv) / len(wv) * 1024 * w_scale
        lines.append("%-50s %12d %14.2f %14.2f" % (_short(k)[:50], g, fb / 1e6, wb / 1e6))
        rec = per_kernel[_short(k)]
        rec[0] += fb
        rec[1] += wb
        rec[2] += 1
    # the instance whose last template argument is 0: one channel per 16-byte vector
    dom = [(k, r) for k, r in per_kernel.items() if dominant in k and k.rstrip(">").rstrip().endswith(", 0")]
    if not dom:
        raise SystemExit("dominant kernel %r not found" % dominant)
    name, (fb, wb, shapes) = max(dom, key=lambda kr: kr[1][0] + kr[1][1])
    record = {"kernel": name, "launch_shapes": shapes, "fetch_bytes_per_launch": fb / shapes,
              "write_bytes_per_launch": wb / shapes, "traffic_bytes_per_launch": (fb + wb) / shapes,
              "fetch_scale": f_scale, "write_scale": w_scale, "source_hash": source_hash(),
              "workload": "config3", "dtype": "f32"}
    lines += ["", "dominant kernel %s: %.2f MB fetched + %.2f MB written per launch (mean over its %d launch shapes)"
              % (name, fb / shapes / 1e6, wb / shapes / 1e6, shapes)]
    return "\n".join(lines), record


def load_record(workload: str = "config3", dtype: str = "f32"):
    """The stored traffic figure, or None when it was taken from other kernel sources, on
    another workload or with another storage type than the launch it is to describe."""
    try:
        rec = json.load(open(RECORD))
    except (OSError, ValueError):
        return None
    same = (rec.get("source_hash") == source_hash() and rec.get("workload", "config3") == workload
            and rec.get("dtype", "f32") == dtype)
    return rec if same else None


TRACE_HEADER = """Kernel times of the default benchmark run (ResNet-18 ImageNet activation set, batch 256, float32,
4-bit: granq_calibrate_fakequant_fwd per tensor, then backward in reverse; 20 warm-up + 200 timed steps)

command (from /tmp with TMPDIR=/tmp, repository at $R, output under $OUT):
  rocprofv3 --kernel-trace --stats --output-format csv -d $OUT/trace -o bench -- \\
      python3 $R/bench.py --no-extras --cpu-sample-batch 0
summary made with:
  python -m paper_2503_18339_amd.profiling trace $OUT/trace/bench_kernel_stats.csv
(avg_us of the dominant kernel is to be compared with roofline.avg_launch_us of bench.py's JSON line)
"""

COUNTER_HEADER = """HBM traffic of the GranQ kernels on the default benchmark workload, from two rocprofv3 counter runs
(ResNet-18 ImageNet activation set, batch 256, float32, 4-bit, granq_calibrate_fakequant_fwd per tensor then
backward in reverse; FETCH_SIZE and WRITE_SIZE in KiB per dispatch)

commands (from /tmp with TMPDIR=/tmp, repository at $R, output under $OUT), one counter per run:
  rocprofv3 --pmc FETCH_SIZE --output-format csv -d $OUT/fetch -o bench -- \\
      python3 $R/bench.py --no-extras --cpu-sample-batch 0 --steps 3 --warmup 1 --pmc-calibration
  rocprofv3 --pmc WRITE_SIZE --output-format csv -d $OUT/write -o bench -- \\
      python3 $R/bench.py --no-extras --cpu-sample-batch 0 --steps 3 --warmup 1 --pmc-calibration
summary made with:
  python -m paper_2503_18339_amd.profiling counters $OUT/fetch/bench_counter_collection.csv \\
      $OUT/write/bench_counter_collection.csv --copy-bytes 822083584 --write-record
(--pmc-calibration adds three plain device copies of the 822 MB tensor: what the two counters read for
a known number of bytes gives the scale factors below)
"""


def summarise_pmc(counter_csv: str, only: str = "granq") -> str:
    """Per kernel and counter: mean of the counter over the kernel's dispatches."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(counter_csv)):
        if only and only not in r["Kernel_Name"]:
            continue
        agg[_short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    names = sorted({c for k in agg.values() for c in k})
    out = ["%-58s %9s " % ("kernel", "launches") + " ".join("%16s" % n for n in names)]
    for k, cs in sorted(agg.items()):
        n = max(len(v) for v in cs.values())
        out.append("%-58s %9d " % (k[:58], n) + " ".join(
            "%16.2f" % (sum(cs[c]) / len(cs[c])) if c in cs else "%16s" % "-" for c in names))
    return "\n".join(out)


def _header(title: str, command: str, made_with: str) -> str:
    return "%s\n\ncommand (from /tmp with TMPDIR=/tmp, repository at $R, output under $OUT):\n  %s\nsummary made with:\n  %s\n" % (
        title, command.replace("\\n", "\n  "), made_with)


def main(argv=None):
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("stats_csv")
    t.add_argument("--title", help="what was run (default: the default benchmark run)")
    t.add_argument("--command", help="the rocprofv3 command that made the file")
    t.add_argument("--match", default="", help="regular expression a kernel name must match to be listed")
    c = sub.add_parser("counters")
    c.add_argument("fetch_csv")
    c.add_argument("write_csv")
    c.add_argument("--copy-bytes", type=int, required=True)
    c.add_argument("--write-record", action="store_true")
    m = sub.add_parser("pmc")
    m.add_argument("counter_csv")
    m.add_argument("--title", required=True)
    m.add_argument("--command", required=True)
    m.add_argument("--only", default="granq", help="substring a kernel name must contain")
    args = ap.parse_args(argv)
    if args.cmd == "trace":
        if args.title:
            print(_header(args.title, args.command or "", "python -m paper_2503_18339_amd.profiling trace "
                          "<stats csv> --title ... --command ..." + (" --match '%s'" % args.match if args.match else "")))
        else:
            print(TRACE_HEADER)
        print(summarise_trace(args.stats_csv, args.match))
    elif args.cmd == "pmc":
        print(_header(args.title, args.command, "python -m paper_2503_18339_amd.profiling pmc "
                      "<counter_collection csv> --title ... --command ..."))
        print(summarise_pmc(args.counter_csv, args.only))
    else:
        text, record = summarise_counters(args.fetch_csv, args.write_csv, args.copy_bytes)
        print(COUNTER_HEADER)
        print(text)
        if args.write_record:
            json.dump(record, open(RECORD, "w"), indent=1)
            print("\nwrote", RECORD, file=sys.stderr)


if __name__ == "__main__":
    main()

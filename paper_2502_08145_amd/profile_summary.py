"""Turn rocprofv3 CSV output into a short text summary (per kernel: calls, mean duration,
counter means, HBM bytes scaled by the copy probe).

    python -m paper_2502_08145_amd.profile_summary <dir> [<dir> ...]

Each <dir> is the -d directory of one rocprofv3 run (--kernel-trace, with --stats and/or --pmc).
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import re
import sys


def short(name: str) -> str:
    m = re.search(r"gemm_tile_kernel<(\d+), (\d+), (true|false), (true|false)>", name)
    if m:
        bm, bn, akc, bkc = m.groups()
        lay = {("true", "false"): "NN", ("true", "true"): "NT", ("false", "false"): "TN"}.get((akc, bkc), "??")
        return f"mfma_{bm}x{bn}/{lay}"
    if "copy_probe_kernel" in name:
        return "copy_probe"
    if "gemm_naive_kernel" in name:
        return "naive"
    return re.sub(r"\(.*", "", name)[:60]


def summarize(d: str, out=sys.stdout):
    traces = glob.glob(os.path.join(d, "**", "*kernel_trace.csv"), recursive=True)
    counters = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    dur = collections.defaultdict(list)
    for f in traces:
        for r in csv.DictReader(open(f)):
            dur[short(r["Kernel_Name"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    ctr = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in counters:
        for r in csv.DictReader(open(f)):
            ctr[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    print(f"== {d}", file=out)
    keys = [k for k in dur if k.startswith(("mfma_", "copy_probe", "naive"))]
    for k in sorted(keys, key=lambda k: -sum(dur[k])):
        v = dur[k]
        print(f"{k:<22s} calls {len(v):5d}  mean {sum(v) / len(v) / 1e3:9.2f} us  min {min(v) / 1e3:9.2f}  "
              f"max {max(v) / 1e3:9.2f}  total {sum(v) / 1e6:9.3f} ms", file=out)
        for c, vals in sorted(ctr.get(k, {}).items()):
            print(f"    {c:<28s} mean per dispatch {sum(vals) / len(vals):.6g}  (n={len(vals)})", file=out)
    return dur, ctr


def main(argv):
    if len(argv) < 2:
        sys.exit(__doc__)
    for d in argv[1:]:
        summarize(d)


if __name__ == "__main__":
    main(sys.argv)

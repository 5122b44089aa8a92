"""Turn rocprofv3 CSV output into a short text summary (per kernel: calls, mean duration,
counter means) and, on request, into the HBM bytes per launch that bench.py reports.

    python -m paper_2502_08145_amd.profile_summary <dir> [<dir> ...]
    python -m paper_2502_08145_amd.profile_summary --traffic <workload> <copy MiB> <FETCH dir> <WRITE dir>

Each <dir> is the -d directory of one rocprofv3 run (--kernel-trace, with --stats and/or --pmc).
--traffic prints a JSON object {workload: {kernel: bytes per launch}}: FETCH_SIZE and WRITE_SIZE
(KiB per dispatch) of every GEMM kernel, each scaled by what the same counter read for a kernel of
exactly known traffic that ran in the same process: the tiled transpose of a <copy MiB> MiB matrix
(bench.py --calibrate-copy; every element read once and written once).  The object also carries
the hash of the kernel sources it was measured with ("_source", build.source_id()).
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import re
import sys


def short(name: str) -> str:
    m = re.search(r"gemm_tile_kernel(16)?<(\d+), (\d+), (\d+), (\d+), (true|false), (true|false), (true|false)>", name)
    if m:
        k16, bm, bn, wm, wn, akc, bkc, split = m.groups()
        lay = {("true", "false"): "NN", ("true", "true"): "NT", ("false", "false"): "TN"}.get((akc, bkc), "??")
        waves = "_w8" if int(wm) * int(wn) == 8 else ""
        return f"mfma{k16 or ''}_{bm}x{bn}{waves}{'_sk' if split == 'true' else ''}/{lay}"
    m = re.search(r"gemm_tile_kernel_k64<(\d+), (\d+), (\d+), (true|false), (true|false), (true|false), \d+>", name)
    if m:
        bm, bn, wn, akc, bkc, split = m.groups()
        lay = {("true", "false"): "NN", ("true", "true"): "NT", ("false", "false"): "TN"}.get((akc, bkc), "??")
        return f"mfma16k64_{bm}x{bn}{'_w8' if wn == '4' else ''}{'_sk' if split == 'true' else ''}/{lay}"
    m = re.search(r"gemm_tile_kernel_k64p<(true|false), (true|false)>", name)
    if m:
        lay = {("true", "false"): "NN", ("true", "true"): "NT", ("false", "false"): "TN"}.get(m.groups(), "??")
        return f"mfma16k64p_256x256_w8/{lay}"
    if "transpose_tile_kernel" in name:
        return "transpose_tile"
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
    keys = [k for k in dur if k.startswith(("mfma", "transpose_tile", "naive"))]
    for k in sorted(keys, key=lambda k: -sum(dur[k])):
        v = dur[k]
        print(f"{k:<22s} calls {len(v):5d}  mean {sum(v) / len(v) / 1e3:9.2f} us  min {min(v) / 1e3:9.2f}  "
              f"max {max(v) / 1e3:9.2f}  total {sum(v) / 1e6:9.3f} ms", file=out)
        means = {c: sum(vals) / len(vals) for c, vals in ctr.get(k, {}).items()}
        for c in sorted(means):
            print(f"    {c:<28s} mean per dispatch {means[c]:.6g}  (n={len(ctr[k][c])})", file=out)
        # derived: GRBM_GUI_ACTIVE is summed over the 8 XCDs, SQ_VALU_MFMA_BUSY_CYCLES over 256 CUs x 4 SIMDs
        if "SQ_VALU_MFMA_BUSY_CYCLES" in means and means.get("GRBM_GUI_ACTIVE"):
            print(f"    -> MFMA busy {means['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024.0 / (means['GRBM_GUI_ACTIVE'] / 8.0) * 100:.1f} % of "
                  f"the kernel's cycles", file=out)
        if "SQ_LDS_BANK_CONFLICT" in means and means.get("SQ_LDS_IDX_ACTIVE"):
            print(f"    -> LDS bank-conflict cycles / LDS-active cycles {means['SQ_LDS_BANK_CONFLICT'] / means['SQ_LDS_IDX_ACTIVE'] * 100:.1f} %",
                  file=out)
    return dur, ctr


def kernel_key(variant: str, layout: str) -> str:
    """The name this module gives the kernel behind a library variant (split-K variants of 2 and
    4 K ranges are one kernel)."""
    return re.sub(r"_sk\d+$", "_sk", variant) + "/" + layout


def traffic(workload: str, copy_mib: float, fetch_dir: str, write_dir: str) -> dict:
    import io
    _, fetch = summarize(fetch_dir, io.StringIO())
    _, write = summarize(write_dir, io.StringIO())
    mean = lambda v: sum(v) / len(v)
    kib = copy_mib * 1024.0
    f_scale = kib / mean(fetch["transpose_tile"]["FETCH_SIZE"])
    w_scale = kib / mean(write["transpose_tile"]["WRITE_SIZE"])
    out = {}
    for k in fetch:
        if k.startswith("mfma") and k in write:
            out[k] = int(round(1024.0 * (mean(fetch[k]["FETCH_SIZE"]) * f_scale + mean(write[k]["WRITE_SIZE"]) * w_scale)))
    from .build import source_id
    return {workload: out, "_scale": {"FETCH_SIZE": round(f_scale, 4), "WRITE_SIZE": round(w_scale, 4)},
            "_source": source_id(),
            "_note": "bytes per launch = FETCH_SIZE x scale + WRITE_SIZE x scale (KiB -> bytes), scales from a tiled "
                     "transpose of known size in the same process; _source = hash of the kernel sources measured"}


def main(argv):
    if len(argv) < 2:
        sys.exit(__doc__)
    if argv[1] == "--traffic":
        import json
        if len(argv) != 6:
            sys.exit(__doc__)
        print(json.dumps(traffic(argv[2], float(argv[3]), argv[4], argv[5]), indent=1))
        return
    for d in argv[1:]:
        summarize(d)


if __name__ == "__main__":
    main(sys.argv)

"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python profsum.py kernels <dir with *_kernel_stats.csv>
    python profsum.py traffic <FETCH_SIZE counter csv> <WRITE_SIZE counter csv> \
        --copy-bytes N --workload NAME [--json profiles/traffic.json]

`traffic` scales the FETCH_SIZE / WRITE_SIZE readings (KiB per dispatch) by what the same counter
shows for the library's plain copy kernel (stream_copy_kernel, N bytes read and N bytes written per
dispatch), and reports HBM bytes per launch for every kernel of the library, plus the totals per
C-ABI call (monarch_fwd = the forward kernel, monarch_fwd_ws = the pack kernel + the packed-weight
forward, monarch_bwd = every other kernel of the library; the m = 64 pack kernel serves both
monarch_fwd_ws and monarch_bwd and is counted with the latter).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

COPY_KERNEL = "stream_copy_kernel"


def short(name: str) -> str:
    name = name.replace("monarch::(anonymous namespace)::", "").replace("monarch::", "")
    name = re.sub(r"^void ", "", name)
    return re.sub(r"\(.*$", "", name)


def is_ours(name: str) -> bool:
    return "monarch::" in name


def cmd_kernels(args):
    files = glob.glob(os.path.join(args.dir, "**", "*kernel_stats.csv"), recursive=True)
    if not files:
        sys.exit("no *kernel_stats.csv under " + args.dir)
    rows = list(csv.DictReader(open(files[0])))
    print("%-78s %6s %12s %12s %12s %7s" % ("kernel", "calls", "avg_ns", "min_ns", "max_ns", "pct"))
    for r in rows:
        if float(r["Percentage"]) < 0.05 and not is_ours(r["Name"]):
            continue
        print("%-78s %6s %12.0f %12s %12s %6.2f%%" % (short(r["Name"])[:78], r["Calls"], float(r["AverageNs"]),
                                                     r["MinNs"], r["MaxNs"], float(r["Percentage"])))


def read_counter(path: str, counter: str):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            agg[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in agg.items()}, {k: len(v) for k, v in agg.items()}


def cmd_traffic(args):
    fetch, nf = read_counter(args.fetch_csv, "FETCH_SIZE")
    write, _ = read_counter(args.write_csv, "WRITE_SIZE")
    if COPY_KERNEL not in fetch or COPY_KERNEL not in write:
        sys.exit("the copy kernel was not profiled: run bench.py (it times monarch_stream_copy)")
    kib = args.copy_bytes / 1024.0
    f_scale, w_scale = kib / fetch[COPY_KERNEL], kib / write[COPY_KERNEL]
    print("calibration: %s moves %.0f KiB each way; FETCH_SIZE reads %.0f (factor %.3f), WRITE_SIZE reads %.0f (factor %.3f)"
          % (COPY_KERNEL, kib, fetch[COPY_KERNEL], f_scale, write[COPY_KERNEL], w_scale))
    print("%-60s %6s %14s %14s" % ("kernel", "calls", "fetch_MB", "write_MB"))
    calls = {"monarch_fwd": [0.0, 0.0], "monarch_fwd_ws": [0.0, 0.0], "monarch_bwd": [0.0, 0.0]}
    per_kernel = {}
    for k in sorted(fetch):
        if k == COPY_KERNEL or not any(t in k for t in ("fwd_", "bwd_", "wgrad_", "prep_", "y1_gemm", "pack64", "transpose64", "transpose_blocks", "reduce_sq16", "generic_", "fill_zero", "f32_to_bf16")):
            continue
        fb, wb = fetch[k] * f_scale * 1024.0, write.get(k, 0.0) * w_scale * 1024.0
        per_kernel[k] = {"fetch_bytes": fb, "write_bytes": wb}
        print("%-60s %6d %14.2f %14.2f" % (k[:60], nf[k], fb / 1e6, wb / 1e6))
        if k.startswith("fwd_frag") or k.startswith("pack_fwd") or k.startswith("fwd_sq64_kernel<true>"):
            call = "monarch_fwd_ws"
        elif k.startswith("fwd_") or k.startswith("generic_fwd") or k.startswith("tiled_fwd"):
            call = "monarch_fwd"
        else:
            call = "monarch_bwd"
        calls[call][0] += fb
        calls[call][1] += wb
    for c, (fb, wb) in calls.items():
        print("%-60s %6s %14.2f %14.2f   total %.2f MB per call" % (c, "", fb / 1e6, wb / 1e6, (fb + wb) / 1e6))
    if args.json:
        data = json.load(open(args.json)) if os.path.exists(args.json) else {}
        data[args.workload] = {c: {"fetch_bytes": v[0], "write_bytes": v[1]} for c, v in calls.items()}
        data[args.workload]["kernels"] = per_kernel
        data[args.workload]["calibration"] = {"fetch_factor": f_scale, "write_factor": w_scale}
        json.dump(data, open(args.json, "w"), indent=1, sort_keys=True)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    k = sub.add_parser("kernels")
    k.add_argument("dir")
    k.set_defaults(fn=cmd_kernels)
    t = sub.add_parser("traffic")
    t.add_argument("fetch_csv")
    t.add_argument("write_csv")
    t.add_argument("--copy-bytes", type=float, required=True)
    t.add_argument("--workload", required=True)
    t.add_argument("--json", default=None)
    t.set_defaults(fn=cmd_traffic)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()

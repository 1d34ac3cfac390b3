#!/usr/bin/env python3
"""Condenses rocprofv3 CSV output of a bench.py run into a short text summary and a JSON
of measured HBM traffic per kernel launch.

Inputs (any subset):
  --stats  <..._kernel_stats.csv>        from  rocprofv3 --kernel-trace --stats --output-format csv
  --fetch  <..._counter_collection.csv>  from  rocprofv3 --pmc FETCH_SIZE --output-format csv
  --write  <..._counter_collection.csv>  from  rocprofv3 --pmc WRITE_SIZE --output-format csv
  --pmc    <..._counter_collection.csv>  (repeatable) any other counter run: every counter in
                                         it is averaged per dispatch and per kernel
The two counter runs must come from `bench.py --calibrate-copy`, which also launches the
library's plain copy kernel on a 256 MiB buffer: what the counters read for that known
traffic gives the scale factor applied to every other kernel.

All tile-shape instantiations of one __global__ template are summed under the template's
name, as bench.py does for its roofline object.
"""
from __future__ import annotations

import argparse
import csv
import json
import re
import sys
from collections import defaultdict

COPY_BYTES = 256 << 20


def kernel_of(symbol: str) -> str:
    m = re.search(r"(\w+_kernel)\b", symbol)
    if m:
        return m.group(1)
    if symbol.startswith("_Z"):
        # (rocprofv3 leaves the instantiations on _Float16 mangled: <length><name> pieces)
        i = 3 if symbol.startswith("_ZN") else 2
        while True:
            d = re.match(r"\d+", symbol[i:])
            if not d:
                break
            i += d.end()
            name = symbol[i:i + int(d.group())]
            if name.endswith("_kernel"):
                return name
            i += int(d.group())
    return symbol.split("(")[0].split("<")[0]


def read_stats(path):
    agg = defaultdict(lambda: [0, 0.0])
    with open(path) as f:
        for r in csv.DictReader(f):
            k = kernel_of(r["Name"])
            agg[k][0] += int(r["Calls"])
            agg[k][1] += float(r["TotalDurationNs"])
    return {k: {"calls": c, "total_ns": t, "avg_ns": t / c} for k, (c, t) in agg.items()}


def read_counter(path, counter):
    """Average counter value (KiB) per dispatch, per kernel."""
    per = defaultdict(lambda: defaultdict(float))      # kernel -> dispatch -> sum over rows
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter:
                continue
            per[kernel_of(r["Kernel_Name"])][r["Dispatch_Id"]] += float(r["Counter_Value"])
    return {k: {"dispatches": len(d), "avg_kib": sum(d.values()) / len(d)} for k, d in per.items()}


def read_all_counters(path):
    """{kernel: {counter: average value per dispatch}} for every counter in the file."""
    per = defaultdict(lambda: defaultdict(lambda: defaultdict(float)))
    with open(path) as f:
        for r in csv.DictReader(f):
            per[kernel_of(r["Kernel_Name"])][r["Counter_Name"]][r["Dispatch_Id"]] += float(r["Counter_Value"])
    return {k: {c: sum(d.values()) / len(d) for c, d in cs.items()} for k, cs in per.items()}


# (label, numerator, denominator): plain ratios of the raw per-dispatch averages above.  The
# SQ "cycles" counters are sums over all SIMDs / CUs / dies in the tool's own units, so the
# ratios are for comparing kernels with each other, not absolute utilisations.
RATIOS = [
    ("FMA share of VALU instructions", "SQ_INSTS_VALU_FMA_F32", "SQ_INSTS_VALU"),
    ("VALU instructions per vector memory read", "SQ_INSTS_VALU", "SQ_INSTS_VMEM_RD"),
    ("VALU active / busy-CU cycles", "SQ_ACTIVE_INST_VALU", "SQ_BUSY_CU_CYCLES"),
    ("LDS bank-conflict / LDS active cycles", "SQ_LDS_BANK_CONFLICT", "SQ_ACTIVE_INST_LDS"),
    ("MFMA busy / busy-CU cycles", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES"),
    ("L2 hit rate", "TCC_HIT_sum", None),
    ("vector-cache line accesses per buffer-load wave instruction", "TCP_TOTAL_CACHE_ACCESSES_sum", "TA_BUFFER_LOAD_WAVEFRONTS_sum"),
    ("address unit busy / vector-cache clocked cycles", "TA_TA_BUSY_sum", "TCP_GATE_EN1_sum"),
    ("vector cache waiting on misses / clocked cycles", "TCP_PENDING_STALL_CYCLES_sum", "TCP_GATE_EN1_sum"),
]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--stats")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--pmc", action="append", default=[])
    ap.add_argument("--command", action="append", default=[], help="command line(s) to record in the summary")
    ap.add_argument("--title", default="rocprofv3 summary")
    ap.add_argument("--out-txt", required=True)
    ap.add_argument("--out-json", default="")
    args = ap.parse_args()

    lines = [args.title, "=" * len(args.title), ""]
    for c in args.command:
        lines.append("command: " + c)
    lines.append("")
    stats = read_stats(args.stats) if args.stats else {}
    if stats:
        tot = sum(v["total_ns"] for v in stats.values())
        lines.append("kernel time (rocprofv3 --kernel-trace --stats; instantiations of one template summed)")
        lines.append("%-28s %8s %14s %12s %7s" % ("kernel", "calls", "total_us", "avg_us", "share"))
        for k, v in sorted(stats.items(), key=lambda kv: -kv[1]["total_ns"]):
            lines.append("%-28s %8d %14.1f %12.3f %6.1f%%" % (k, v["calls"], v["total_ns"] / 1e3, v["avg_ns"] / 1e3,
                                                              100.0 * v["total_ns"] / tot))
        lines.append("")
    traffic = {}
    factors = {}
    for label, path, counter in (("fetch", args.fetch, "FETCH_SIZE"), ("write", args.write, "WRITE_SIZE")):
        if not path:
            continue
        c = read_counter(path, counter)
        if "copy_kernel" not in c:
            print("no copy_kernel dispatches in %s: run bench.py with --calibrate-copy" % path, file=sys.stderr)
            return 1
        factor = (COPY_BYTES / 1024.0) / c["copy_kernel"]["avg_kib"]
        factors[label] = factor
        lines.append("%s per dispatch (rocprofv3 --pmc %s, KiB); plain copy of %d KiB reads %.0f KiB "
                     "=> scale factor %.3f" % (counter, counter, COPY_BYTES // 1024, c["copy_kernel"]["avg_kib"], factor))
        lines.append("%-28s %10s %14s %14s" % ("kernel", "dispatches", "raw_avg_KiB", "scaled_KiB"))
        for k, v in sorted(c.items(), key=lambda kv: -kv[1]["avg_kib"] * kv[1]["dispatches"]):
            lines.append("%-28s %10d %14.1f %14.1f" % (k, v["dispatches"], v["avg_kib"], v["avg_kib"] * factor))
            traffic.setdefault(k, {})[label + "_bytes_per_launch"] = v["avg_kib"] * factor * 1024.0
        lines.append("")
    merged = defaultdict(dict)
    for path in args.pmc:
        for k, cs in read_all_counters(path).items():
            merged[k].update(cs)
    if merged:
        names = sorted({c for cs in merged.values() for c in cs})
        lines.append("other counters, average per dispatch (rocprofv3 --pmc, one run per counter group)")
        for k in sorted(merged, key=lambda k: -merged[k].get("SQ_BUSY_CYCLES", merged[k].get("SQ_WAVES", 0.0))):
            if not k.endswith("_kernel"):
                continue
            lines.append("  " + k)
            for c in names:
                if c in merged[k]:
                    lines.append("    %-34s %16.1f" % (c, merged[k][c]))
            for label, num, den in RATIOS:
                if num in merged[k]:
                    if den is None:
                        tot = merged[k][num] + merged[k].get("TCC_MISS_sum", 0.0)
                        if tot > 0:
                            lines.append("    %-50s %8.3f" % (label, merged[k][num] / tot))
                    elif merged[k].get(den, 0.0) > 0:
                        lines.append("    %-50s %8.3f" % (label, merged[k][num] / merged[k][den]))
        lines.append("")
    for k, v in traffic.items():
        v["hbm_bytes_per_launch"] = v.get("fetch_bytes_per_launch", 0.0) + v.get("write_bytes_per_launch", 0.0)
    with open(args.out_txt, "w") as f:
        f.write("\n".join(lines) + "\n")
    if args.out_json:
        with open(args.out_json, "w") as f:
            json.dump({"scale_factors": factors, "kernels": traffic}, f, indent=1, sort_keys=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

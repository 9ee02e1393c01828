#!/usr/bin/env python3
"""Condense rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under profiles/.

Runs on the CPU over directories a profiling run left behind; it launches nothing.

    python -m paper_2506_15545_amd.profile_summary stats   <rocprofv3 -d dir> <out.txt> "<command>"
    python -m paper_2506_15545_amd.profile_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir> <out.txt> \
           <workload> "<fetch command>" "<write command>"

`stats` lists calls / average / min / max duration per kernel from the `--kernel-trace --stats` run.
`traffic` averages the FETCH_SIZE and WRITE_SIZE readings per dispatch of every kernel and scales them by
what the same counters read for the calibration pass of `bench.py --calibrate-copy` (an out-of-place
elementwise kernel that reads and writes 256 MiB); the result is HBM-side bytes per launch.  The table is
followed by the same rows as JSON after a `---JSON---` line, which `bench.py` reads for `roofline.traffic`.
"""
import collections
import csv
import glob
import json
import os
import re
import sys

CAL_BYTES = 256 * 2 ** 20
ALIASES = {"decode_kernel_2pass": "decode_kernel"}   # the name bench.py reports the decode launch under
WORKLOAD_KERNELS = {"decode_b128_w512": ("decode_kernel",)}


def short_name(full):
    full = full.replace("(anonymous namespace)::", "")
    m = re.search(r"(?:rattn::)?([A-Za-z_][A-Za-z_0-9]*)\s*(?:<|\()", full.replace("void ", ""))
    name = m.group(1) if m else full[:48]
    if "elementwise" in full:      # torch kernels: only the out-of-place add is the calibration pass
        name = "calibration_elementwise" if "add" in full else "torch_elementwise_other"
    return ALIASES.get(name, name)


def find(d, suffix):
    return sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))


def stats(d, out, command):
    rows = collections.OrderedDict()
    for f in find(d, "kernel_stats.csv"):
        for r in csv.DictReader(open(f)):
            rows[short_name(r["Name"])] = r
    with open(out, "w") as fo:
        fo.write(f"command: {command}\n")
        fo.write("source: rocprofv3 kernel_stats.csv (durations in microseconds)\n\n")
        fo.write(f"{'kernel':34s} {'calls':>7s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'share_%':>8s}\n")
        for n, r in rows.items():
            fo.write(f"{n:34s} {int(r['Calls']):7d} {float(r['AverageNs']) / 1e3:10.1f} {float(r['MinNs']) / 1e3:10.1f} "
                     f"{float(r['MaxNs']) / 1e3:10.1f} {float(r['Percentage']):8.2f}\n")


def counter_means(d, counter):
    tot, cnt = collections.defaultdict(float), collections.Counter()
    for f in find(d, "counter_collection.csv"):
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] != counter:
                continue
            n = short_name(r["Kernel_Name"])
            tot[n] += float(r["Counter_Value"]); cnt[n] += 1
    return {n: tot[n] / cnt[n] for n in tot}, cnt


def traffic(dfetch, dwrite, out, workload, cmd_fetch, cmd_write):
    fetch, nf = counter_means(dfetch, "FETCH_SIZE")
    write, nw = counter_means(dwrite, "WRITE_SIZE")
    cal = "calibration_elementwise"
    if cal not in fetch or cal not in write:
        raise SystemExit("calibration kernel not found: run bench.py with --calibrate-copy under the counters")
    kf, kw = CAL_BYTES / fetch[cal], CAL_BYTES / write[cal]
    only = WORKLOAD_KERNELS.get(workload)
    table = {}
    for n in fetch:
        if n == cal or n == "torch_elementwise_other" or (only and n not in only) or (not only and n in sum(WORKLOAD_KERNELS.values(), ())):
            continue
        rd, wr = fetch[n] * kf, write.get(n, 0.0) * kw
        table[n] = {"dispatches": nf[n], "fetch_bytes": rd, "write_bytes": wr, "hbm_bytes_per_launch": rd + wr}
    with open(out, "w") as fo:
        fo.write(f"workload: {workload}\ncommand (FETCH_SIZE): {cmd_fetch}\ncommand (WRITE_SIZE): {cmd_write}\n")
        fo.write(f"calibration: the 256 MiB out-of-place elementwise pass read FETCH_SIZE={fetch[cal]:.0f} and "
                 f"WRITE_SIZE={write[cal]:.0f}; bytes per count = {kf:.1f} (fetch), {kw:.1f} (write)\n\n")
        fo.write(f"{'kernel':28s} {'dispatches':>10s} {'fetch_MB':>10s} {'write_MB':>10s} {'total_MB':>10s}\n")
        for n, r in table.items():
            fo.write(f"{n:28s} {r['dispatches']:10d} {r['fetch_bytes'] / 1e6:10.2f} {r['write_bytes'] / 1e6:10.2f} "
                     f"{r['hbm_bytes_per_launch'] / 1e6:10.2f}\n")
        fo.write("\n---JSON---\n" + json.dumps(table, indent=1) + "\n")


if __name__ == "__main__":
    if len(sys.argv) >= 5 and sys.argv[1] == "stats":
        stats(sys.argv[2], sys.argv[3], sys.argv[4])
    elif len(sys.argv) >= 8 and sys.argv[1] == "traffic":
        traffic(*sys.argv[2:8])
    else:
        raise SystemExit(__doc__)

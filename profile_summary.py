#!/usr/bin/env python3
"""Condense rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under profiles/.

Runs on the CPU over directories a profiling run left behind; it launches nothing.

    python profile_summary.py stats   <rocprofv3 -d dir> <out.txt> "<command>"
    python profile_summary.py traffic <FETCH_SIZE dir> <WRITE_SIZE dir> <out.txt> \
           <workload> "<fetch command>" "<write command>"
    python profile_summary.py mfma    <SQ counters dir> <out.txt> "<command>"

`stats` lists calls / average / min / max duration per kernel from the `--kernel-trace --stats` run.
`traffic` averages the FETCH_SIZE and WRITE_SIZE readings per dispatch of every kernel and scales them by
what the same counters read for the calibration pass of `bench.py --calibrate-copy` (an out-of-place
elementwise kernel that reads and writes 256 MiB); the result is HBM-side bytes per launch.  The table is
followed by the same rows as JSON after a `---JSON---` line, which `bench.py` reads for `roofline.traffic`.
`mfma` reads one `--pmc` run with SQ_BUSY_CYCLES, SQ_VALU_MFMA_BUSY_CYCLES, SQ_INSTS_MFMA and, if present,
SQ_INSTS_VALU, SQ_INSTS_LDS, SQ_INSTS_SALU, and lists per kernel how busy the
matrix pipes were: MFMA busy cycles per SIMD (1024 SIMDs) over the kernel's busy cycles (SQ_BUSY_CYCLES is summed
over the 32 shader engines), the matrix FLOP/s actually executed (32x32x16 MFMAs, 32768 FLOP each), and the other
instruction classes per MFMA.  Kernels run serialised under the counters, so durations are a little longer than
in the timing runs.
"""
import collections
import csv
import glob
import json
import os
import re
import sys

import hashlib

CAL_BYTES = 256 * 2 ** 20


def kernel_sources_digest():
    """sha256 over the library's kernel sources (csrc/*, sorted by name): written into every summary, so that a
    reader (and bench.py) can tell whether a summary was taken from the kernels that are in the tree now."""
    d = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2506_15545_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".hpp")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


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
        fo.write(f"kernel sources (sha256 of csrc/*.hip, *.hpp): {kernel_sources_digest()}\n")
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
        fo.write(f"kernel sources (sha256 of csrc/*.hip, *.hpp): {kernel_sources_digest()}\n")
        fo.write(f"calibration: the 256 MiB out-of-place elementwise pass read FETCH_SIZE={fetch[cal]:.0f} and "
                 f"WRITE_SIZE={write[cal]:.0f}; bytes per count = {kf:.1f} (fetch), {kw:.1f} (write)\n\n")
        fo.write(f"{'kernel':28s} {'dispatches':>10s} {'fetch_MB':>10s} {'write_MB':>10s} {'total_MB':>10s}\n")
        for n, r in table.items():
            fo.write(f"{n:28s} {r['dispatches']:10d} {r['fetch_bytes'] / 1e6:10.2f} {r['write_bytes'] / 1e6:10.2f} "
                     f"{r['hbm_bytes_per_launch'] / 1e6:10.2f}\n")
        table["_kernel_sources"] = kernel_sources_digest()
        fo.write("\n---JSON---\n" + json.dumps(table, indent=1) + "\n")


def mfma(d, out, command):
    names = ("SQ_BUSY_CYCLES", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_MFMA", "SQ_INSTS_VALU", "SQ_INSTS_LDS",
             "SQ_INSTS_SALU")
    means = {c: counter_means(d, c)[0] for c in names}
    dur, nd = collections.defaultdict(float), collections.Counter()
    for f in find(d, "counter_collection.csv"):
        seen = set()
        for r in csv.DictReader(open(f)):
            if r["Dispatch_Id"] in seen:
                continue
            seen.add(r["Dispatch_Id"])
            n = short_name(r["Kernel_Name"])
            dur[n] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"]); nd[n] += 1
    SIMDS, SES, FLOP = 1024, 32, 2 * 32 * 32 * 16
    with open(out, "w") as fo:
        fo.write(f"command: {command}\nkernel sources (sha256 of csrc/*.hip, *.hpp): {kernel_sources_digest()}\n")
        fo.write("source: rocprofv3 counter_collection.csv, means per dispatch; busy = SQ_VALU_MFMA_BUSY_CYCLES / 1024 SIMDs "
                 "over SQ_BUSY_CYCLES / 32 shader engines\n\n")
        fo.write(f"{'kernel':24s} {'disp':>5s} {'avg_us':>8s} {'MFMA_insts':>11s} {'MFMA_TFLOPs':>11s} {'pipe_busy':>9s} "
                 f"{'VALU/MFMA':>9s} {'LDS/MFMA':>8s} {'SALU/MFMA':>9s}\n")
        for n in means["SQ_INSTS_MFMA"]:
            m = means["SQ_INSTS_MFMA"][n]
            if m <= 0 or n not in means["SQ_BUSY_CYCLES"]:
                continue
            us = dur[n] / nd[n] / 1e3
            busy = means["SQ_BUSY_CYCLES"][n] / SES
            frac = means["SQ_VALU_MFMA_BUSY_CYCLES"].get(n, 0.0) / SIMDS / busy
            per = lambda c: (f"{means[c][n] / m:.2f}" if n in means[c] else "-")
            # vector instructions other than MFMAs (the MFMA count is part of SQ_INSTS_VALU)
            valu = f"{(means['SQ_INSTS_VALU'][n] - m) / m:.2f}" if n in means["SQ_INSTS_VALU"] else "-"
            fo.write(f"{n:24s} {nd[n]:5d} {us:8.1f} {m:11.0f} {m * FLOP / (us * 1e-6) / 1e12:11.0f} {frac:9.3f} "
                     f"{valu:>9s} {per('SQ_INSTS_LDS'):>8s} {per('SQ_INSTS_SALU'):>9s}\n")


if __name__ == "__main__":
    if len(sys.argv) >= 5 and sys.argv[1] == "stats":
        stats(sys.argv[2], sys.argv[3], sys.argv[4])
    elif len(sys.argv) >= 8 and sys.argv[1] == "traffic":
        traffic(*sys.argv[2:8])
    elif len(sys.argv) >= 5 and sys.argv[1] == "mfma":
        mfma(sys.argv[2], sys.argv[3], sys.argv[4])
    else:
        raise SystemExit(__doc__)

"""Turns rocprofv3 CSV output of a bench.py run into the short text summaries kept under profiles/.

    python -m paper_2604_17701_amd.profile_summary kernels <kernel_stats.csv> <out.txt> "<command>"
    python -m paper_2604_17701_amd.profile_summary traffic <fetch counter_collection.csv> <write counter_collection.csv> <out.txt> "<commands>"

The traffic summary scales FETCH_SIZE / WRITE_SIZE by what the same counters read for the library's plain
1 GiB copy kernel in the same run, and records a hash of the kernel sources so that bench.py can tell whether
the figures still describe the kernels it runs.
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import os
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
COPY_BYTES = float(1 << 30)


def source_hash() -> str:
    h = hashlib.sha256()
    for p in sorted(glob.glob(os.path.join(PKG, "csrc", "*"))):
        with open(p, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def short(name: str) -> str:
    return name.replace("void ", "").replace("wisv::", "").split("(")[0]


def kernels(stats_csv: str, out: str, command: str):
    rows = list(csv.DictReader(open(stats_csv)))
    seen, lines = set(), []
    total = sum(float(r["TotalDurationNs"]) for r in rows if "wisv" in r["Name"] and r["Name"] not in seen and not seen.add(r["Name"]))
    seen.clear()
    for r in rows:
        if "wisv" not in r["Name"] or r["Name"] in seen:
            continue
        seen.add(r["Name"])
        lines.append(f"{short(r['Name']):44s} calls {int(r['Calls']):7d}  avg {float(r['AverageNs']) / 1e3:9.2f} us  "
                     f"min {float(r['MinNs']) / 1e3:8.2f}  max {float(r['MaxNs']) / 1e3:8.2f}  "
                     f"{100 * float(r['TotalDurationNs']) / total:5.1f} % of library kernel time")
    with open(out, "w") as f:
        f.write(f"# rocprofv3 --kernel-trace --stats summary (library kernels only)\n# command: {command}\n")
        f.write("\n".join(lines) + "\n")


def traffic(fetch_csv: str, write_csv: str, out: str, command: str):
    def per_kernel(path):
        agg = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            agg[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
        return {k: sum(v) / len(v) for k, v in agg.items()}, {k: len(v) for k, v in agg.items()}
    fe, nf = per_kernel(fetch_csv)
    wr, _ = per_kernel(write_csv)
    cf = COPY_BYTES / fe["k_calibration_copy"]          # bytes per FETCH_SIZE count
    cw = COPY_BYTES / wr["k_calibration_copy"]
    with open(out, "w") as f:
        f.write("# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (two runs)\n")
        f.write(f"# commands: {command}\n")
        f.write(f"# calibration: the plain 1 GiB copy kernel reads FETCH_SIZE {fe['k_calibration_copy']:.1f} and WRITE_SIZE "
                f"{wr['k_calibration_copy']:.1f} per dispatch -> {cf:.1f} / {cw:.1f} bytes per count\n")
        f.write(f"source_sha256 {source_hash()}\n")
        for k in sorted(fe, key=lambda k: -fe[k] * nf[k]):
            if k.startswith("k_") and k != "k_calibration_copy" and k != "k_retile":
                f.write(f"kernel {k:40s} launches {nf[k]:6d} fetch_bytes_per_launch {fe[k] * cf:14.0f} "
                        f"write_bytes_per_launch {wr.get(k, 0.0) * cw:12.0f}\n")


def read_traffic(path: str):
    """Parses a traffic summary: (source hash, {kernel: (launches, fetch bytes, write bytes per launch)})."""
    sha, table = None, {}
    with open(path) as f:
        for line in f:
            if line.startswith("source_sha256"):
                sha = line.split()[1]
            elif line.startswith("kernel "):
                body = line[len("kernel "):]
                name = body[:body.index(" launches ")].strip()
                nums = body[body.index(" launches "):].split()
                table[name] = (int(nums[1]), float(nums[3]), float(nums[5]))
    return sha, table


def template_args(kernel: str):
    """'k_gemm_ws<1, 1, 8, 1, 8, 1>' -> ('k_gemm_ws', ['1', '1', '8', '1', '8', '1'])"""
    if "<" not in kernel:
        return kernel, []
    base, rest = kernel.split("<", 1)
    return base, [a.strip() for a in rest.rstrip(">").split(",")]


if __name__ == "__main__":
    if sys.argv[1] == "kernels":
        kernels(*sys.argv[2:5])
    else:
        traffic(*sys.argv[2:6])

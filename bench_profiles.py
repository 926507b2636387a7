"""The rocprofv3 side of bench.py: turns rocprofv3 CSV output of a bench.py run into the short text summaries kept
under profiles/, and reads those summaries back for bench.py's roofline line.

    python bench_profiles.py kernels <kernel_stats.csv> <out.txt> "<command>"
    python bench_profiles.py traffic <fetch counter_collection.csv> <write counter_collection.csv> <out.txt> "<commands>"
    python bench_profiles.py counters <counter_collection.csv> <out.txt> "<command>"

The traffic summary scales FETCH_SIZE / WRITE_SIZE by what the same counters read for the library's plain
1 GiB copy kernel in the same run, and every summary records a hash of the kernel sources so that bench.py can tell
whether the figures still describe the kernels it runs.
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(ROOT, "paper_2604_17701_amd", "csrc")
COPY_BYTES = float(1 << 30)


def source_hash() -> str:
    h = hashlib.sha256()
    for p in sorted(glob.glob(os.path.join(CSRC, "*"))):
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
        f.write(f"source_sha256 {source_hash()}\n")
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


def counters(csv_path: str, out: str, command: str):
    """Per-kernel averages of whatever counters one --pmc run collected, plus the matrix-core figures they give:
    executed bf16 / f16 MFMA flop per launch (SQ_INSTS_VALU_MFMA_MOPS_* count units of 512 flop) and the share of
    the chip's SIMD cycles in which the MFMA unit was busy."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(csv_path)):
        agg[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    names = sorted({c for k in agg.values() for c in k})
    with open(out, "w") as f:
        f.write("# per-launch averages of rocprofv3 --pmc counters (summed over the chip by the profiler)\n")
        f.write(f"# command: {command}\n")
        f.write(f"source_sha256 {source_hash()}\n")
        for k in sorted(agg, key=lambda k: -sum(agg[k].get("SQ_BUSY_CU_CYCLES", agg[k][names[0]]))):
            if not k.startswith("k_") or k in ("k_calibration_copy", "k_retile"):
                continue
            avg = {c: sum(v) / len(v) for c, v in agg[k].items()}
            n = len(next(iter(agg[k].values())))
            f.write(f"kernel {k}  launches {n}\n")
            for c in names:
                if c in avg:
                    f.write(f"    {c:34s} {avg[c]:16.1f}\n")
            if "SQ_INSTS_VALU_MFMA_MOPS_BF16" in avg:
                f.write(f"    {'executed_bf16_mfma_flop':34s} {avg['SQ_INSTS_VALU_MFMA_MOPS_BF16'] * 512:16.4g}\n")
            if "SQ_INSTS_VALU_MFMA_MOPS_F16" in avg:
                f.write(f"    {'executed_f16_mfma_flop':34s} {avg['SQ_INSTS_VALU_MFMA_MOPS_F16'] * 512:16.4g}\n")
            if avg.get("GRBM_GUI_ACTIVE") and "SQ_VALU_MFMA_BUSY_CYCLES" in avg:
                # GRBM_GUI_ACTIVE comes summed over the 8 XCDs, the MFMA busy cycles over the 1024 SIMDs
                share = avg["SQ_VALU_MFMA_BUSY_CYCLES"] / (avg["GRBM_GUI_ACTIVE"] / 8 * 1024)
                f.write(f"    {'mfma_busy_share_of_simd_cycles':34s} {share:16.3f}\n")


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


def read_kernels(path: str):
    """Parses a kernel-stats summary: {kernel: (calls, average microseconds)}."""
    table = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or " calls " not in line:
                continue
            name = line[:line.index(" calls ")].strip()
            nums = line[line.index(" calls "):].split()
            table[name] = (int(nums[1]), float(nums[3]))
    return table


def template_args(kernel: str):
    """'k_gemm_ws<1, 1, 8, 1, 8, 1>' -> ('k_gemm_ws', ['1', '1', '8', '1', '8', '1'])"""
    if "<" not in kernel:
        return kernel, []
    base, rest = kernel.split("<", 1)
    return base, [a.strip() for a in rest.rstrip(">").split(",")]


def read_hash(path: str):
    """The source hash a summary was taken at (None for a summary without one)."""
    with open(path) as f:
        for line in f:
            if line.startswith("source_sha256"):
                return line.split()[1]
    return None


# position of the epilogue in the template arguments of the two GEMM kernels, and which class an epilogue means
_EPI_ARG = {"k_gemm_ws": 6, "k_gemm_mm": 7}
_EPI_CLASS = {"0": "gemm_qkv_o_down", "1": "gemm_gate_up", "2": "lm_head", "3": "gemm_qkv_o_down"}


def kernel_class(kernel: str):
    """bench.py's kernel class of a (shortened) kernel name, or None.  The three k-split products of a layer (QKV, O,
    down) share kernel templates: a trace cannot tell them apart, so they map to one class that bench.py's per-launch
    event timing splits further."""
    base, args = template_args(kernel)
    if base == "k_attn_mfma":
        return "attention"
    if base in _EPI_ARG and len(args) > _EPI_ARG[base]:
        return _EPI_CLASS.get(args[_EPI_ARG[base]])
    return None


if __name__ == "__main__":
    if sys.argv[1] == "kernels":
        kernels(*sys.argv[2:5])
    elif sys.argv[1] == "counters":
        counters(*sys.argv[2:5])
    else:
        traffic(*sys.argv[2:6])

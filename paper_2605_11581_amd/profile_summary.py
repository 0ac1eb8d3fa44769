"""Condense rocprofv3 CSV output (kernel stats, FETCH_SIZE / WRITE_SIZE counter runs) into the
short text summaries kept under profiles/.

    python -m paper_2605_11581_amd.profile_summary stats  <dir> <out.txt> "<command line>"
    python -m paper_2605_11581_amd.profile_summary pmc    <fetch_dir> <write_dir> <out.txt> "<command lines>" [kernel name]

The counter summary scales FETCH_SIZE and WRITE_SIZE (KiB per dispatch) by what the same counters
read for the runtime's plain 1 GiB device-to-device copy kernel in the same run.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys

GIB_KIB = float(1 << 20)


def _one(pattern: str) -> str:
    hits = glob.glob(pattern, recursive=True)
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return hits[0]


def stats(src: str, out: str, cmd: str) -> None:
    rows = list(csv.DictReader(open(_one(os.path.join(src, "**", "*_kernel_stats.csv")))))
    with open(out, "w") as f:
        f.write(f"# rocprofv3 --kernel-trace --stats summary\n# command: {cmd}\n")
        f.write("# kernel, calls, total_ms, avg_us, min_us, max_us, percent\n")
        for r in rows:
            f.write(f"{r['Name'][:70]}, {r['Calls']}, {float(r['TotalDurationNs']) / 1e6:.3f}, "
                    f"{float(r['AverageNs']) / 1e3:.2f}, {float(r['MinNs']) / 1e3:.2f}, {float(r['MaxNs']) / 1e3:.2f}, "
                    f"{r['Percentage']}\n")


def _counter(src: str, name: str):
    """kernel name -> counter values of its dispatches, in dispatch order."""
    rows = [r for r in csv.DictReader(open(_one(os.path.join(src, "**", "*_counter_collection.csv")))) if r["Counter_Name"] == name]
    rows.sort(key=lambda r: int(r.get("Dispatch_Id") or 0))
    acc = collections.defaultdict(list)
    for r in rows:
        acc[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return acc


def _calibration(values) -> float:
    """The benchmark runs its three 1 GiB calibration copies before anything else: the median of the first three
    dispatches of the runtime's copy kernel (later copies of other sizes belong to the workload)."""
    first = sorted(values[:3])
    return first[len(first) // 2] if first else 0.0


def pmc(fetch_dir: str, write_dir: str, out: str, cmd: str, kernel: str = "mk_megakernel") -> None:
    fe, wr = _counter(fetch_dir, "FETCH_SIZE"), _counter(write_dir, "WRITE_SIZE")
    copy_f = _calibration(fe.get("__amd_rocclr_copyBuffer", []))
    copy_w = _calibration(wr.get("__amd_rocclr_copyBuffer", []))
    # the calibration copy moves exactly 1 GiB each way
    kf = GIB_KIB / copy_f if copy_f else float("nan")
    kw = GIB_KIB / copy_w if copy_w else float("nan")
    mf = sum(fe[kernel]) / len(fe[kernel])
    mw = sum(wr[kernel]) / len(wr[kernel])
    fetch_b, write_b = mf * kf * 1024.0, mw * kw * 1024.0
    with open(out, "w") as f:
        f.write(f"# rocprofv3 --pmc FETCH_SIZE / --pmc WRITE_SIZE summary (two runs)\n# commands: {cmd}\n")
        f.write(f"calibration_copy_1GiB_FETCH_SIZE: {copy_f:.1f}  -> scale {kf:.4f}\n")
        f.write(f"calibration_copy_1GiB_WRITE_SIZE: {copy_w:.1f}  -> scale {kw:.4f}\n")
        f.write(f"{kernel}_dispatches: {len(fe[kernel])}\n")
        f.write(f"{kernel}_FETCH_SIZE_mean_raw: {mf:.1f}\n{kernel}_WRITE_SIZE_mean_raw: {mw:.1f}\n")
        f.write(f"fetch_bytes_per_launch: {fetch_b:.0f}\nwrite_bytes_per_launch: {write_b:.0f}\n")
        f.write(f"traffic_bytes_per_launch: {fetch_b + write_b:.0f}\n")


if __name__ == "__main__":
    if sys.argv[1] == "stats":
        stats(sys.argv[2], sys.argv[3], sys.argv[4])
    else:
        pmc(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5], *(sys.argv[6:7]))

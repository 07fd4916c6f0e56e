"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2205_12268_amd.profsum stats   <dir>/<prefix>_kernel_stats.csv
  python -m paper_2205_12268_amd.profsum traffic <fetch>/..._counter_collection.csv \\
         <write>/..._counter_collection.csv <copy_bytes>

  python -m paper_2205_12268_amd.profsum traffic_scaled <fetch csv> <write csv> <fs> <ws>

  python -m paper_2205_12268_amd.profsum counters <dir>/..._counter_collection.csv

`counters` lists the per-launch means of whatever counters one `--pmc` run collected, in
millions, with the launch duration under the counter run.  Where the run holds
GRBM_GUI_ACTIVE it adds mfma_busy, the share of SIMD cycles on which the matrix cores were
busy: SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 x 1024).  GRBM_GUI_ACTIVE is summed over
the 8 dies (it reads 8 x duration x clock), SQ_VALU_MFMA_BUSY_CYCLES over the 1024 SIMDs (for
the contraction it reads flops / 1017 flops per SIMD cycle, the published bf16 rate).

`traffic` scales FETCH_SIZE and WRITE_SIZE (KiB per dispatch) by what the same counters read
for the plain copy kernel of known size that `bench.py --copy-probe` runs in the same process;
`traffic_scaled` takes the two factors as given (for a workload that has no copy probe).
"""
from __future__ import annotations

import collections
import csv
import re
import sys


def short(name: str) -> str:
    m = re.search(r"(\w+_kernel)(<[^>]*>)?", name)
    return (m.group(1) + (m.group(2) or "")) if m else name.split("(")[0][:48]


def stats(path: str) -> str:
    out = [f"{'kernel':58s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}"]
    for r in csv.DictReader(open(path)):
        out.append(f"{short(r['Name']).replace(' ', ''):58s} {r['Calls']:>6s} "
                   f"{float(r['AverageNs']) / 1e3:9.2f} {float(r['MinNs']) / 1e3:9.2f} "
                   f"{float(r['MaxNs']) / 1e3:9.2f} {float(r['Percentage']):6.2f}")
    return "\n".join(out)


def _is_copy(kernel: str) -> bool:
    """The runtime's device-to-device copy kernel (what torch's copy_ launches)."""
    return "copyBuffer" in kernel


def _mean_counter(path: str, counter: str):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            acc[short(r["Kernel_Name"]).replace(" ", "")].append(float(r["Counter_Value"]))
    # The runtime's copy kernel also serves the framework's own small copies (a scale vector,
    # a scalar): only the probe's launches, the large ones, calibrate the counter.
    for k, v in acc.items():
        if _is_copy(k):
            acc[k] = [x for x in v if x >= 0.5 * max(v)]
    return {k: sum(v) / len(v) for k, v in acc.items()}


def traffic(fetch_csv: str, write_csv: str, copy_bytes: float) -> str:
    f = _mean_counter(fetch_csv, "FETCH_SIZE")
    w = _mean_counter(write_csv, "WRITE_SIZE")
    copy = next(k for k in f if _is_copy(k))
    fs = copy_bytes / (f[copy] * 1024.0)
    ws = copy_bytes / (w[copy] * 1024.0)
    out = [f"# copy kernel {copy}: {copy_bytes:.0f} bytes read and written per launch; "
           f"FETCH_SIZE read {f[copy]:.1f} KiB -> scale {fs:.4f}; WRITE_SIZE read {w[copy]:.1f} KiB -> scale {ws:.4f}",
           f"# {'kernel':56s} {'fetch_bytes':>14s} {'write_bytes':>14s} {'total_bytes':>14s}"]
    for k in f:
        if k == copy:
            continue
        fb, wb = f[k] * 1024 * fs, w.get(k, 0.0) * 1024 * ws
        out.append(f"{k:58s} {fb:14.0f} {wb:14.0f} {fb + wb:14.0f}")
    return "\n".join(out)


def traffic_scaled(fetch_csv: str, write_csv: str, fs: float, ws: float) -> str:
    f = _mean_counter(fetch_csv, "FETCH_SIZE")
    w = _mean_counter(write_csv, "WRITE_SIZE")
    out = [f"# FETCH_SIZE scale {fs:.4f}, WRITE_SIZE scale {ws:.4f} (as calibrated for the single layers)",
           f"# {'kernel':56s} {'fetch_bytes':>14s} {'write_bytes':>14s} {'total_bytes':>14s}"]
    for k in f:
        fb, wb = f[k] * 1024 * fs, w.get(k, 0.0) * 1024 * ws
        out.append(f"{k:58s} {fb:14.0f} {wb:14.0f} {fb + wb:14.0f}")
    return "\n".join(out)


def counters(path: str, n_simd: int = 1024, n_dies: int = 8) -> str:
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    dur = collections.defaultdict(list)
    seen = set()
    for r in csv.DictReader(open(path)):
        k = short(r["Kernel_Name"]).replace(" ", "")
        acc[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
        if r["Dispatch_Id"] not in seen:
            seen.add(r["Dispatch_Id"])
            dur[k].append((float(r["End_Timestamp"]) - float(r["Start_Timestamp"])) / 1e3)
    names = sorted({c for v in acc.values() for c in v})
    out = ["# per-launch means, counters in millions; us = launch duration under the counter run",
           f"# {'kernel':56s} {'n':>4s} {'us':>8s} " + " ".join(f"{c.replace('SQ_', ''):>14s}" for c in names)
           + f" {'mfma_busy':>10s}"]
    for k, v in acc.items():
        mean = {c: sum(x) / len(x) for c, x in v.items()}
        line = f"{k:58s} {len(dur[k]):4d} {sum(dur[k]) / len(dur[k]):8.1f} "
        line += " ".join(f"{mean.get(c, 0.0) / 1e6:14.3f}" for c in names)
        gui = mean.get("GRBM_GUI_ACTIVE", 0.0)
        c = "SQ_VALU_MFMA_BUSY_CYCLES"
        line += f" {mean[c] / (gui / n_dies * n_simd):10.4f}" if gui > 0 and c in mean else f" {'-':>10s}"
        out.append(line)
    return "\n".join(out)


if __name__ == "__main__":
    if sys.argv[1] == "stats":
        print(stats(sys.argv[2]))
    elif sys.argv[1] == "traffic":
        print(traffic(sys.argv[2], sys.argv[3], float(sys.argv[4])))
    elif sys.argv[1] == "counters":
        print(counters(sys.argv[2]))
    elif sys.argv[1] == "traffic_scaled":
        print(traffic_scaled(sys.argv[2], sys.argv[3], float(sys.argv[4]), float(sys.argv[5])))
    else:
        sys.exit(__doc__)

"""Summarises rocprofv3 runs of bench.py into the text and JSON kept under profiles/.

    python -m paper_1412_2302_amd.pmc_summary --key fp32_b128 --fetch F.csv --write W.csv [--mfma M.csv]
        --command "<the rocprofv3 command lines, ';;' between them>" --txt profiles/<name>.txt
        [--json profiles/gemm_traffic.json]
    python -m paper_1412_2302_amd.pmc_summary --key fp32_b128 --trace kt_kernel_stats.csv
        --command "<the rocprofv3 --kernel-trace --stats command line>" --txt profiles/<name>.txt

F.csv / W.csv / M.csv are the *_counter_collection.csv files of three `rocprofv3 --pmc` runs of
`bench.py --only-step --traffic-calibration ...` collecting FETCH_SIZE, WRITE_SIZE and
(MfmaUtil, GRBM_GUI_ACTIVE) respectively.  FETCH_SIZE / WRITE_SIZE (KiB per dispatch at the memory side of
L2) are scaled by what the same counter reads for the three plain 1 GiB elementwise copies that
--traffic-calibration runs first; the factor is printed.  The JSON maps a configuration key to the measured
HBM bytes per GEMM launch, which bench.py reports as roofline.traffic.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import re


def _short(k: str) -> str:
    k = re.sub(r"\(.*$", "", k.replace("void ", "").replace("ax::", ""))
    k = re.sub(r"Tile<(\d+), (\d+), (\d+), \d, \d(, \d+)?>", r"T\1x\2x\3", k)
    return k[:100]


def _load(path, counter):
    return [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == counter]


def _scaled(path, counter):
    rows = _load(path, counter)
    cal = [float(r["Counter_Value"]) for r in rows
           if "at::native" in r["Kernel_Name"] and "Fill" not in r["Kernel_Name"] and int(r["Grid_Size"]) >= (1 << 24)]
    if not cal:
        raise SystemExit(f"{path}: no 1 GiB calibration copies found (run bench.py with --traffic-calibration)")
    factor = (1 << 20) / (sum(cal) / len(cal))  # true KiB per counter unit
    agg = collections.OrderedDict()
    for r in rows:
        agg.setdefault(_short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]) * factor)
    return cal, factor, agg


def trace_summary(a):
    rows = list(csv.DictReader(open(a.trace)))
    tot = sum(float(r["TotalDurationNs"]) for r in rows)
    lines = [f"rocprofv3 kernel trace, configuration {a.key}", "", "Command:", "  " + a.command.strip(), "",
             f"{'kernel':102s} {'calls':>6s} {'total ms':>9s} {'avg us':>9s} {'min us':>8s} {'max us':>8s} {'%':>6s}"]
    g_calls = g_ns = 0
    for r in sorted(rows, key=lambda r: -float(r["TotalDurationNs"])):
        k, c, t = _short(r["Name"]), int(r["Calls"]), float(r["TotalDurationNs"])
        if t / tot < 0.001:
            continue
        lines.append(f"{k:102s} {c:6d} {t / 1e6:9.3f} {float(r['AverageNs']) / 1e3:9.2f} {float(r['MinNs']) / 1e3:8.2f} "
                     f"{float(r['MaxNs']) / 1e3:8.2f} {100 * t / tot:6.2f}")
        if k.startswith("gemm"):
            g_calls += c
            g_ns += t
    lines += ["", f"total kernel time {tot / 1e6:.3f} ms",
              f"all GEMM instantiations together: {g_calls} launches, {g_ns / 1e6:.3f} ms, average {g_ns / max(g_calls, 1) / 1e3:.2f} us per launch"]
    os.makedirs(os.path.dirname(os.path.abspath(a.txt)), exist_ok=True)
    with open(a.txt, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines[-2:]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--key", required=True)
    ap.add_argument("--trace", help="the *_kernel_stats.csv of a `rocprofv3 --kernel-trace --stats` run")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--mfma")
    ap.add_argument("--command", required=True)
    ap.add_argument("--txt", required=True)
    ap.add_argument("--json")
    a = ap.parse_args()
    if a.trace:
        return trace_summary(a)
    if not (a.fetch and a.write):
        raise SystemExit("--fetch and --write (or --trace) are required")
    cal_r, f_r, rd = _scaled(a.fetch, "FETCH_SIZE")
    cal_w, f_w, wr = _scaled(a.write, "WRITE_SIZE")
    util = {}
    if a.mfma:
        for r in _load(a.mfma, "MfmaUtil"):
            util.setdefault(_short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    lines = [f"rocprofv3 hardware counters, configuration {a.key}", "", "Commands (one counter set per run):"]
    lines += ["  " + c.strip() for c in a.command.split(";;")]
    lines += ["",
              f"FETCH_SIZE: 1 GiB elementwise copies read {', '.join('%.1f' % c for c in cal_r)} units -> {f_r:.4f} KiB per unit",
              f"WRITE_SIZE: 1 GiB elementwise copies read {', '.join('%.1f' % c for c in cal_w)} units -> {f_w:.4f} KiB per unit",
              "", f"{'kernel':102s} {'launches':>8s} {'read MiB':>10s} {'write MiB':>10s} {'MfmaUtil %':>10s}"]
    tot = n = 0
    for k, fr in rd.items():
        w = wr.get(k, [0.0])
        r_mib, w_mib = sum(fr) / len(fr) / 1024, sum(w) / len(w) / 1024
        u = util.get(k)
        lines.append(f"{k:102s} {len(fr):8d} {r_mib:10.2f} {w_mib:10.2f} {('%.1f' % (sum(u) / len(u))) if u else '-':>10s}")
        if k.startswith("gemm"):
            tot += (sum(fr) + sum(w)) * 1024
            n += len(fr)
    per = tot / max(n, 1)
    lines += ["", f"all GEMM launches: {n} launches, {per:.0f} bytes of HBM traffic per launch (read + write)"]
    os.makedirs(os.path.dirname(os.path.abspath(a.txt)), exist_ok=True)
    with open(a.txt, "w") as f:
        f.write("\n".join(lines) + "\n")
    if a.json:
        try:
            cur = json.load(open(a.json))
        except (OSError, ValueError):
            cur = {}
        cur[a.key] = {"bytes_per_launch": round(per), "launches": n, "source": os.path.relpath(a.txt, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))}
        with open(a.json, "w") as f:
            json.dump(cur, f, indent=1, sort_keys=True)
            f.write("\n")
    print("\n".join(lines[-3:]))


if __name__ == "__main__":
    main()

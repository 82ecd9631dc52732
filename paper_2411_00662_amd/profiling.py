"""Turns rocprofv3 CSV output of a bench.py run into the short summaries kept under profiles/.

Usage (after the three rocprofv3 runs whose commands the summaries quote):

  python -m paper_2411_00662_amd.profiling stats   <kernel_stats.csv>  <out.txt>  "<command>"
  python -m paper_2411_00662_amd.profiling traffic <fetch counter_collection.csv> <write counter_collection.csv> \
         <copy MiB> <key> <out.txt> <traffic.json> "<fetch command>" "<write command>"
  python -m paper_2411_00662_amd.profiling counters <counter_collection.csv> <out.txt> "<command>"

`traffic` scales FETCH_SIZE / WRITE_SIZE (KiB per dispatch) by what the same counters read for the
plain copy kernel of known size that the run also launched (bench.py --calib-copy-mib), and stores
bytes per launch for every kernel of the path under <key> in <traffic.json>, which bench.py reads
for its roofline.traffic field.
"""
from __future__ import annotations

import collections
import csv
import json
import sys


def short(name: str) -> str:
    name = name.split("(")[0]
    return name.replace("void ", "").replace("monta::", "")


def stats(csv_path: str, out_path: str, command: str) -> None:
    rows = list(csv.DictReader(open(csv_path)))
    with open(out_path, "w") as f:
        f.write(f"# rocprofv3 kernel statistics\n# command: {command}\n")
        f.write(f"{'kernel':34s} {'calls':>7s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'total_ms':>10s} {'share_%':>8s}\n")
        for r in rows:
            f.write(f"{short(r['Name'])[:34]:34s} {int(r['Calls']):7d} {float(r['AverageNs']) / 1e3:10.2f} "
                    f"{float(r['MinNs']) / 1e3:10.2f} {float(r['MaxNs']) / 1e3:10.2f} "
                    f"{float(r['TotalDurationNs']) / 1e6:10.3f} {float(r['Percentage']):8.2f}\n")


def _avg_counter(csv_path: str, counter: str) -> dict:
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(csv_path)):
        if r["Counter_Name"] == counter:
            acc[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def traffic(fetch_csv, write_csv, copy_mib, key, out_path, json_path, fetch_cmd, write_cmd) -> None:
    fetch = _avg_counter(fetch_csv, "FETCH_SIZE")
    write = _avg_counter(write_csv, "WRITE_SIZE")
    copy_kib = int(copy_mib) * 1024
    f_scale = copy_kib / fetch["copy_kernel"][0]       # true KiB per counted unit
    w_scale = copy_kib / write["copy_kernel"][0]
    table = {}
    with open(out_path, "w") as f:
        f.write("# HBM-side traffic per kernel launch from rocprofv3 counters (L2 <-> fabric requests)\n")
        f.write(f"# fetch command: {fetch_cmd}\n# write command: {write_cmd}\n")
        f.write(f"# calibration: the plain copy kernel moved {copy_mib} MiB each way in the same runs; FETCH_SIZE read "
                f"{fetch['copy_kernel'][0]:.1f}, WRITE_SIZE read {write['copy_kernel'][0]:.1f} per dispatch\n")
        f.write(f"# => one FETCH_SIZE unit = {f_scale:.4f} KiB, one WRITE_SIZE unit = {w_scale:.4f} KiB\n")
        f.write(f"{'kernel':28s} {'launches':>8s} {'FETCH_SIZE':>12s} {'WRITE_SIZE':>12s} {'read_MiB':>10s} {'write_MiB':>10s} {'total_MiB':>10s}\n")
        for k in fetch:
            if k not in write or k == "copy_kernel" or "at::native" in k:
                continue
            rd = fetch[k][0] * f_scale * 1024
            wr = write[k][0] * w_scale * 1024
            f.write(f"{k[:28]:28s} {fetch[k][1]:8d} {fetch[k][0]:12.1f} {write[k][0]:12.1f} {rd / 2**20:10.2f} "
                    f"{wr / 2**20:10.2f} {(rd + wr) / 2**20:10.2f}\n")
            table[k] = {"read_bytes": int(rd), "write_bytes": int(wr), "total_bytes": int(rd + wr)}
    try:
        allj = json.load(open(json_path))
    except (OSError, ValueError):
        allj = {}
    allj[key] = table
    json.dump(allj, open(json_path, "w"), indent=1, sort_keys=True)


def counters(csv_path: str, out_path: str, command: str) -> None:
    """Per kernel, the average over its dispatches of every counter of one --pmc run (summed over the
    instances a counter is reported for), plus the ratios that read directly as utilisation.  Every value is the
    chip-wide sum: GRBM_GUI_ACTIVE, the elapsed cycles, is summed over the 8 XCDs, so one eighth of it is the
    kernel's duration in shader clocks (it matches the traced duration at 2.1-2.4 GHz)."""
    XCDS, SIMDS = 8, 1024
    per = collections.defaultdict(lambda: collections.defaultdict(float))     # (kernel, dispatch) -> counter -> value
    for r in csv.DictReader(open(csv_path)):
        per[(short(r["Kernel_Name"]), r["Dispatch_Id"])][r["Counter_Name"]] += float(r["Counter_Value"])
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for (kname, _), cs in per.items():
        for c, v in cs.items():
            agg[kname][c].append(v)
    names = sorted({c for cs in agg.values() for c in cs})
    with open(out_path, "w") as f:
        f.write(f"# rocprofv3 counters, average per dispatch\n# command: {command}\n")
        for kname in sorted(agg, key=lambda k_: -sum(agg[k_].get("SQ_BUSY_CYCLES", agg[k_][names[0]]))):
            if "at::native" in kname or "rocclr" in kname:
                continue
            n = len(next(iter(agg[kname].values())))
            f.write(f"{kname}  ({n} dispatches)\n")
            avg = {c: sum(v) / len(v) for c, v in agg[kname].items()}
            for c in names:
                if c in avg:
                    f.write(f"    {c:34s} {avg[c]:18.1f}\n")
            if "SQ_VALU_MFMA_BUSY_CYCLES" in avg and "GRBM_GUI_ACTIVE" in avg and avg["GRBM_GUI_ACTIVE"] > 0:
                # SQ counters are summed over the chip's SIMDs (1024 on MI355X): busy cycles per SIMD over elapsed cycles
                elapsed = avg["GRBM_GUI_ACTIVE"] / XCDS
                f.write(f"    {'=> elapsed shader clocks':34s} {elapsed:18.1f}   (GRBM_GUI_ACTIVE / 8 XCDs)\n")
                f.write(f"    {'=> matrix cores busy':34s} {100 * avg['SQ_VALU_MFMA_BUSY_CYCLES'] / (elapsed * SIMDS):17.1f}%"
                        "   (SQ_VALU_MFMA_BUSY_CYCLES / (elapsed x 1024 SIMDs))\n")
            if "SQ_LDS_BANK_CONFLICT" in avg and avg.get("SQ_LDS_IDX_ACTIVE", 0) > 0:
                f.write(f"    {'=> LDS cycles lost to conflicts':34s} {100 * avg['SQ_LDS_BANK_CONFLICT'] / avg['SQ_LDS_IDX_ACTIVE']:17.1f}%"
                        "   (SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE)\n")
            if "SQ_WAIT_INST_LDS" in avg and avg.get("SQ_WAVE_CYCLES", 0) > 0:
                f.write(f"    {'=> wave cycles waiting on LDS':34s} {100 * avg['SQ_WAIT_INST_LDS'] / avg['SQ_WAVE_CYCLES']:17.1f}%"
                        "   (SQ_WAIT_INST_LDS / SQ_WAVE_CYCLES)\n")
            if "SQ_WAIT_INST_ANY" in avg and avg.get("SQ_WAVE_CYCLES", 0) > 0:
                f.write(f"    {'=> wave cycles waiting on anything':34s} {100 * avg['SQ_WAIT_INST_ANY'] / avg['SQ_WAVE_CYCLES']:17.1f}%"
                        "   (SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES)\n")


if __name__ == "__main__":
    if len(sys.argv) >= 5 and sys.argv[1] == "counters":
        counters(sys.argv[2], sys.argv[3], sys.argv[4])
    elif len(sys.argv) >= 5 and sys.argv[1] == "stats":
        stats(sys.argv[2], sys.argv[3], sys.argv[4])
    elif len(sys.argv) >= 10 and sys.argv[1] == "traffic":
        traffic(*sys.argv[2:10])
    else:
        print(__doc__)
        sys.exit(2)

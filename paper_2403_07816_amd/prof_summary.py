"""Turn rocprofv3 CSV output (kernel stats, PMC counter collections) into the short text
summaries kept under profiles/.

  python -m paper_2403_07816_amd.prof_summary stats  <bench_kernel_stats.csv>
  python -m paper_2403_07816_amd.prof_summary pmc    [--calib KERNEL:READ_KIB:WRITE_KIB] <pmc_counter_collection.csv> [...]

--calib names a plain streaming kernel of the same run whose traffic is known (KiB read and written per
dispatch): FETCH_SIZE and WRITE_SIZE of every kernel are to be divided by what those counters read per
KiB that kernel moved.  The factors and a digest of the GEMM kernel source go into "#" lines that
bench.py parses.
"""
from __future__ import annotations

import collections
import csv
import sys

MODES = {0: "up_swiglu", 1: "down", 2: "bwd_act", 3: "bwd_dx", 4: "dw13", 5: "dw2"}


def short(name: str) -> str:
    name = name.replace("btx::(anonymous namespace)::", "").replace("void ", "").split("(")[0]
    if name.startswith("mfma_gemm_kernel<"):
        args = name[len("mfma_gemm_kernel<"):-1].split(",")   # BM, BN, BK, WM, WN, NSA, NSB, MODE, TAIL
        name += " " + MODES.get(int(args[7]), "?")
    return name


def stats(path: str) -> None:
    rows = list(csv.DictReader(open(path)))
    print(f"{'kernel':72s} {'calls':>5s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'pct':>7s}")
    for r in rows:
        if "btx::" not in r["Name"]:
            continue
        print(f"{short(r['Name'])[:72]:72s} {r['Calls']:>5s} {float(r['AverageNs']) / 1e3:10.1f} "
              f"{float(r['MinNs']) / 1e3:10.1f} {float(r['MaxNs']) / 1e3:10.1f} {float(r['Percentage']):7.2f}")


def source_digest() -> str:
    import hashlib
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "gemm_mfma.hip")
    return hashlib.sha256(open(path, "rb").read()).hexdigest()[:16]


def pmc(paths, calib=None) -> None:
    agg = collections.OrderedDict()
    dur = collections.OrderedDict()     # kernel -> counter -> durations (ns) of the dispatches it was read on
    for path in paths:
        for r in csv.DictReader(open(path)):
            if "btx" not in r["Kernel_Name"]:
                continue
            k = short(r["Kernel_Name"])
            agg.setdefault(k, collections.OrderedDict()).setdefault(r["Counter_Name"], []).append(
                float(r["Counter_Value"]))
            dur.setdefault(k, {}).setdefault(r["Counter_Name"], []).append(
                float(r["End_Timestamp"]) - float(r["Start_Timestamp"]))
    print(f"# gemm_mfma.hip sha256/16: {source_digest()}")
    if calib:
        kname, read_kib, write_kib = calib.split(":")
        match = [k for k in agg if k.startswith(kname)]
        if match:
            c = agg[match[0]]
            parts = []
            if "FETCH_SIZE" in c:
                parts.append(f"FETCH_SIZE={sum(c['FETCH_SIZE']) / len(c['FETCH_SIZE']) / float(read_kib):.4f}")
            if "WRITE_SIZE" in c:
                parts.append(f"WRITE_SIZE={sum(c['WRITE_SIZE']) / len(c['WRITE_SIZE']) / float(write_kib):.4f}")
            print(f"# calibration: {' '.join(parts)}   (counter KiB per KiB that {match[0]} is known to move: "
                  f"{read_kib} KiB read, {write_kib} KiB written per dispatch)")
    for name, counters in agg.items():
        print(name)
        for c, v in counters.items():
            print(f"    {c:34s} {sum(v) / len(v):18.0f}   (mean of {len(v)} dispatches)")
        mean = {c: sum(v) / len(v) for c, v in counters.items()}
        if "GRBM_GUI_ACTIVE" in mean:
            # GRBM_GUI_ACTIVE is summed over the 8 XCDs, SQ_VALU_MFMA_BUSY_CYCLES over the 1024 SIMDs
            cyc = mean["GRBM_GUI_ACTIVE"] / 8.0
            d = dur[name]["GRBM_GUI_ACTIVE"]
            ns = sum(d) / len(d)
            line = f"    derived: {ns / 1e3:9.1f} us per dispatch in this run, {cyc / ns:5.2f} GHz mean clock"
            if mean.get("SQ_VALU_MFMA_BUSY_CYCLES", 0) > 0:
                line += f", MFMA busy {mean['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024.0 / cyc * 100:4.1f} % of active cycles"
            print(line)


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("stats", "pmc"):
        sys.exit(__doc__)
    if sys.argv[1] == "stats":
        stats(sys.argv[2])
    else:
        rest, calib = sys.argv[2:], None
        if rest[0] == "--calib":
            calib, rest = rest[1], rest[2:]
        pmc(rest, calib)

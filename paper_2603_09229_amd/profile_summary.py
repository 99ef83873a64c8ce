"""Turns raw rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2603_09229_amd.profile_summary kernel-stats <dir>/<name>_kernel_stats.csv <out.txt> "<command>" ["<note>"]
    python -m paper_2603_09229_amd.profile_summary traffic <fetch_dir> <write_dir> <kernel substring> <kernel name> <workload> <out.txt> "<command>"
    python -m paper_2603_09229_amd.profile_summary counters <dir1> <dir2> <kernel substring> <out.txt> "<command 1>" "<command 2>"
    python -m paper_2603_09229_amd.profile_summary ooc-overlap <dir> <out.txt> "<command>"
    python -m paper_2603_09229_amd.profile_summary bench-json <bench output.json> <out.txt> "<command>" "<title>"

The raw output (CSV files, databases) stays where rocprofv3 wrote it; only the summary is meant
to be committed.  Every summary starts with the command that produced its input.
"""
from __future__ import annotations

import csv
import glob
import os
import sys
from collections import defaultdict


def _one(pattern: str) -> str:
    hits = sorted(glob.glob(pattern, recursive=True))
    if not hits:
        raise FileNotFoundError(pattern)
    return hits[0]


def kernel_stats(stats_csv: str, out: str, command: str, note: str = "") -> None:
    rows = list(csv.DictReader(open(stats_csv)))
    with open(out, "w") as o:
        o.write("rocprofv3 --kernel-trace --stats summary (one MI355X)\n")
        o.write(f"command: {command}\n")
        if note:
            o.write(f"note: {note}\n")
        o.write(f"{'kernel':72s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'total_ms':>9s} {'pct':>6s}\n")
        for r in rows:
            if not (r["Name"].startswith("void fk::") or r["Name"].startswith("fk::")):
                continue
            o.write(f"{r['Name'][:72]:72s} {r['Calls']:>6s} {float(r['AverageNs']) / 1e3:10.1f} "
                    f"{float(r['MinNs']) / 1e3:10.1f} {float(r['MaxNs']) / 1e3:10.1f} "
                    f"{float(r['TotalDurationNs']) / 1e6:9.2f} {float(r['Percentage']):6.2f}\n")
        o.write("(kernels of the input generator and torch copies omitted; percentages are of all GPU "
                "kernel time in the run)\n")


def _counter(dirname: str, counter: str, ksub: str):
    vals, copy = [], []
    f = _one(os.path.join(dirname, "**", "*counter_collection.csv"))
    for r in csv.DictReader(open(f)):
        if r["Counter_Name"] != counter:
            continue
        if ksub in r["Kernel_Name"]:
            vals.append(float(r["Counter_Value"]))
        if "rocclr_copyBuffer" in r["Kernel_Name"]:
            copy.append(float(r["Counter_Value"]))
    return vals, (max(copy) if copy else None)


def traffic(fetch_dir: str, write_dir: str, ksub: str, kname: str, workload: str, out: str, command: str) -> None:
    """HBM bytes per launch from FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled by what
    the same counter reads for the plain 1 GiB device copy of bench.py --calibrate-copy."""
    fv, fcopy = _counter(fetch_dir, "FETCH_SIZE", ksub)
    wv, wcopy = _counter(write_dir, "WRITE_SIZE", ksub)
    gib_kib = 1048576.0
    ff, wf = gib_kib / fcopy, gib_kib / wcopy
    fa, wa = sum(fv) / len(fv), sum(wv) / len(wv)
    hbm = (fa * ff + wa * wf) * 1024
    with open(out, "w") as o:
        o.write(f"HBM traffic of {kname} on workload {workload} (one MI355X), from two rocprofv3 --pmc runs\n")
        o.write(f"command 1: {command}\n")
        o.write("command 2: same with --pmc WRITE_SIZE\n")
        o.write(f"calibration: the plain 1 GiB device-to-device copy issued by --calibrate-copy (kernel "
                f"__amd_rocclr_copyBuffer) reads FETCH_SIZE = {fcopy:.1f} KiB and WRITE_SIZE = {wcopy:.1f} KiB "
                f"for 1048576 KiB each way\n")
        o.write(f"scale factors (true KiB per counter KiB): fetch {ff:.4f}, write {wf:.4f}\n")
        o.write(f"dispatches averaged: {len(fv)} (fetch run), {len(wv)} (write run)\n")
        o.write(f"FETCH_SIZE avg per launch: {fa:.1f} KiB raw -> {fa * ff:.1f} KiB scaled\n")
        o.write(f"WRITE_SIZE avg per launch: {wa:.1f} KiB raw -> {wa * wf:.1f} KiB scaled\n")
        o.write(f"hbm_bytes_per_launch: {hbm:.0f}\n")
    print(f"{kname} {workload}: {hbm / 1e6:.1f} MB per launch")


def _counters_of(dirname: str, ksub: str):
    acc, dur, seen = defaultdict(list), [], set()
    trace = {r["Dispatch_Id"]: r for r in csv.DictReader(open(_one(os.path.join(dirname, "**", "*kernel_trace.csv"))))}
    for r in csv.DictReader(open(_one(os.path.join(dirname, "**", "*counter_collection.csv")))):
        if ksub not in r["Kernel_Name"]:
            continue
        acc[r["Counter_Name"]].append(float(r["Counter_Value"]))
        if r["Dispatch_Id"] not in seen and r["Dispatch_Id"] in trace:
            seen.add(r["Dispatch_Id"])
            t = trace[r["Dispatch_Id"]]
            dur.append((int(t["End_Timestamp"]) - int(t["Start_Timestamp"])) / 1e3)
    return {k: sum(v) / len(v) for k, v in acc.items()}, sum(dur) / len(dur), len(dur)


def counters(dir1: str, dir2: str, ksub: str, out: str, command1: str, command2: str) -> None:
    """MFMA / VALU / LDS counters of one kernel (two --pmc runs, averaged over its dispatches), with
    the derived figures: MFMA pipe utilisation at the clock the kernel ran at, VALU per MFMA."""
    a, d1, n1 = _counters_of(dir1, ksub)
    b, d2, n2 = _counters_of(dir2, ksub)
    with open(out, "w") as o:
        o.write(f"MFMA / VALU / LDS counters of {ksub} (one MI355X), two rocprofv3 --pmc runs\n")
        o.write(f"command 1: {command1}\ncommand 2: {command2}\n")
        o.write(f"dispatches averaged: {n1} / {n2}; mean kernel duration {d1:.1f} us / {d2:.1f} us "
                "(counter collection slows the kernel slightly)\n")
        for k, v in list(a.items()) + list(b.items()):
            o.write(f"{k:34s} {v:.6g}\n")
        o.write("derived:\n")
        if "SQ_INSTS_MFMA" in a and "SQ_VALU_MFMA_BUSY_CYCLES" in a and "GRBM_GUI_ACTIVE" in a:
            mf, busy, gui = a["SQ_INSTS_MFMA"], a["SQ_VALU_MFMA_BUSY_CYCLES"], a["GRBM_GUI_ACTIVE"]
            o.write(f"  MFMA instructions per launch            {mf:.4g}\n")
            o.write(f"  MFMA pipe busy cycles per SIMD          {busy / 1024:.4g}  (1024 SIMDs)\n")
            o.write(f"  GPU active cycles (GRBM_GUI_ACTIVE / 8 XCDs) {gui / 8:.4g} -> clock during the kernel ~ "
                    f"{gui / 8 / d1 / 1e3:.2f} GHz\n")
            o.write(f"  MFMA pipe utilisation at that clock     {busy / 1024 / (gui / 8):.3f}\n")
            if "SQ_INSTS_VALU" in a:
                o.write(f"  VALU issue (non-MFMA) per MFMA          {(a['SQ_INSTS_VALU'] - mf) / mf:.2f} instructions\n")
            if "SQ_LDS_BANK_CONFLICT" in a:
                o.write(f"  LDS bank conflicts                      {a['SQ_LDS_BANK_CONFLICT']:.4g}\n")
        for name in ("SQ_INSTS_VALU_MFMA_MOPS_F16", "SQ_INSTS_VALU_MFMA_MOPS_BF16"):
            if name in b:
                o.write(f"  flop from {name} (x512)    {b[name] * 512:.4g}\n")
        if "SQ_WAIT_ANY" in b and "SQ_WAVE_CYCLES" in a:
            o.write(f"  SQ_WAIT_ANY / SQ_WAVE_CYCLES            {b['SQ_WAIT_ANY'] / a['SQ_WAVE_CYCLES']:.3f}\n")
    print(open(out).read())


def _union_len(intervals):
    total, end = 0, None
    for s, e in sorted(intervals):
        if end is None or s > end:
            total += e - s
            end = e
        elif e > end:
            total += e - end
            end = e
    return total


def _overlap_with(intervals, s, e):
    """Length of [s, e) covered by the union of `intervals` (sorted, disjoint)."""
    cov = 0
    for a, b in intervals:
        if b <= s:
            continue
        if a >= e:
            break
        cov += min(b, e) - max(a, s)
    return cov


def ooc_overlap(dirname: str, out: str, command: str) -> None:
    """Out-of-core run: how much of the host-to-device copy time ran while kernels were running
    (kernel trace + memory-copy trace of the same run)."""
    kt = list(csv.DictReader(open(_one(os.path.join(dirname, "**", "*kernel_trace.csv")))))
    mc = list(csv.DictReader(open(_one(os.path.join(dirname, "**", "*memory_copy_trace.csv")))))
    kern = [(int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Kernel_Name"]) for r in kt
            if r["Kernel_Name"].startswith("void fk::") or r["Kernel_Name"].startswith("fk::")]
    big = max(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in mc)
    # the chunk copies: host-to-device, long (the input generator's copies go the other way)
    copies = [(int(r["Start_Timestamp"]), int(r["End_Timestamp"])) for r in mc
              if "HOST_TO_DEVICE" in r["Direction"].upper().replace(" ", "_") and
              int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) > big / 20]
    t0 = min(s for s, _ in copies)
    t1 = max(e for _, e, _ in kern)
    kin = [(s, e) for s, e, _ in kern if s >= t0]
    # disjoint, sorted union of the kernel intervals
    merged = []
    for s, e in sorted(kin):
        if merged and s <= merged[-1][1]:
            merged[-1] = (merged[-1][0], max(merged[-1][1], e))
        else:
            merged.append((s, e))
    ksum = sum(e - s for s, e in kin)
    kunion = sum(e - s for s, e in merged)
    csum = sum(e - s for s, e in copies)
    cov = sum(_overlap_with(merged, s, e) for s, e in copies)
    by = defaultdict(lambda: [0, 0])
    for s, e, n in kern:
        if s >= t0:
            by[n.split("(")[0][:60]][0] += e - s
            by[n.split("(")[0][:60]][1] += 1
    with open(out, "w") as o:
        o.write("Out-of-core Lloyd iterations: overlap of the host-to-device chunk stream with the kernels (one MI355X)\n")
        o.write(f"command: {command}\n")
        o.write(f"window: first chunk copy .. last kernel = {(t1 - t0) / 1e6:.2f} ms\n")
        o.write(f"chunk copies (host to device): {len(copies)}, total {csum / 1e6:.2f} ms, "
                f"mean {csum / len(copies) / 1e6:.2f} ms each\n")
        o.write(f"kernels in the window: {len(kin)}, summed durations {ksum / 1e6:.2f} ms, "
                f"time with at least one kernel running {kunion / 1e6:.2f} ms "
                f"({kunion / (t1 - t0):.3f} of the window)\n")
        o.write(f"copy time that ran while a kernel was running: {cov / 1e6:.2f} ms = {cov / csum:.3f} of all copy time\n")
        o.write(f"window / summed kernel time = {(t1 - t0) / ksum:.3f} (1.0 = the copies cost nothing)\n")
        o.write("kernel time by kernel (ms, launches):\n")
        for n, (ns, c) in sorted(by.items(), key=lambda kv: -kv[1][0]):
            o.write(f"  {n:60s} {ns / 1e6:9.2f} {c:6d}\n")
    print(open(out).read())


def bench_json(json_file: str, out: str, command: str, title: str) -> None:
    """One JSON line printed by bench.py (a run, a sweep, a comparison) as readable text: scalars
    one per line, every list of records one record per line."""
    import json
    d = json.loads(open(json_file).read().strip().splitlines()[-1])

    def emit(o, key, val, indent=""):
        if isinstance(val, list) and val and isinstance(val[0], dict):
            o.write(f"{indent}{key}:\n")
            for r in val:
                o.write(f"{indent}  " + json.dumps(r, separators=(", ", ": ")) + "\n")
        elif isinstance(val, dict) and any(isinstance(v, (dict, list)) for v in val.values()):
            o.write(f"{indent}{key}:\n")
            for k, v in val.items():
                emit(o, k, v, indent + "  ")
        else:
            o.write(f"{indent}{key}: " + (json.dumps(val, separators=(", ", ": ")) if isinstance(val, (dict, list)) else str(val)) + "\n")

    with open(out, "w") as o:
        o.write(f"{title} (one MI355X)\n")
        o.write(f"command: {command}\n")
        for k, v in d.items():
            emit(o, k, v)


def main(argv) -> int:
    if len(argv) < 2:
        print(__doc__)
        return 2
    mode, a = argv[1], argv[2:]
    if mode == "kernel-stats":
        kernel_stats(*a)
    elif mode == "traffic":
        traffic(*a)
    elif mode == "counters":
        counters(*a)
    elif mode == "ooc-overlap":
        ooc_overlap(*a)
    elif mode == "bench-json":
        bench_json(*a)
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))

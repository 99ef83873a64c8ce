#!/usr/bin/env python3
"""Benchmark of the Lloyd k-means hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c1|c3|c4|c5|p512|p8m|pk8k]

A step is one full Lloyd iteration (fused assign, sort-inverse, segment reduction,
merge/normalise) over a synthetic Gaussian mixture already resident in HBM.  The default
workload is the headline one: N = 2^20, d = 128, K = 1024, fp16.  Prints ONE JSON line.

The line carries, besides the throughput, the roofline of the dominant kernel (its
algorithmic flops or bytes over its mean duration measured with HIP events inside the
library, on the stream the kernels run on) and the fp64 CPU oracle timed on this machine's
host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

PEAK_MFMA_F16_TFLOPS = 2500.0     # MI355X dense fp16 / bf16 MFMA
PEAK_HBM_GBPS = 8000.0            # MI355X HBM3E
PEAK_FP32_VALU_TFLOPS = 157.3


def _traffic_from_profiles(kernel: str, workload: str):
    """HBM bytes per launch measured offline with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
    read from profiles/<kernel>_<workload>_traffic.txt if that summary has been committed."""
    f = ROOT / "profiles" / f"{kernel}_{workload}_traffic.txt"
    if not f.exists():
        return None
    for line in f.read_text().splitlines():
        if line.startswith("hbm_bytes_per_launch:"):
            return float(line.split(":", 1)[1])
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--repeats", type=int, default=7,
                    help="timed blocks of --steps iterations; the median block is reported")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="default workload only: leave out the short runs of the other in-core "
                         "configurations (other_configs in the JSON line)")
    ap.add_argument("--sweep-variants", action="store_true",
                    help="time the assign kernel's tile shapes exhaustively over a grid of shapes "
                         "and compare with the shape heuristic's pick (prints one JSON line)")
    ap.add_argument("--compare-standard", action="store_true",
                    help="time the fused assign and the sort-inverse update against the standard "
                         "implementation (materialised distances, atomic scatter) on a few shapes")
    ap.add_argument("--sweep-choices", action="store_true",
                    help="time both sides of the host's other kernel choices over a grid of shapes: "
                         "streaming vs sweeping assign kernel for few centroids, LDS-staged vs "
                         "direct scatter in the counting sort (prints one JSON line)")
    ap.add_argument("--clock-trace", action="store_true",
                    help="loop the assign kernel (and a device copy) for a few seconds each while "
                         "sampling the shader clock with rocm-smi; also times the headline shape "
                         "on operands that toggle less (zeros, ones) to show what the power limit "
                         "costs (prints one JSON line)")
    ap.add_argument("--general-update", action="store_true",
                    help="few-cluster shapes: use the general assign + sort-inverse path instead "
                         "of the fused one-hot pass (for comparing the two)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy first (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2603_09229_amd import binding as fk
    from paper_2603_09229_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    short = {"c1": wl.C1, "c2": wl.C2, "c3": wl.C3, "c4": wl.C4, "c5": wl.C5, "p512": wl.P512,
             "p8m": wl.P8M, "pk8k": wl.PK8K}
    if args.workload not in short:
        print(f"unknown workload {args.workload}", file=sys.stderr)
        return 2
    if args.sweep_variants:
        return sweep_variants(torch, fk, dev)
    if args.compare_standard:
        return compare_standard(torch, fk, wl, dev)
    if args.sweep_choices:
        return sweep_choices(torch, fk, dev)
    if args.clock_trace:
        return clock_trace(torch, fk, dev)
    if args.general_update:
        fk.fk_set_option("fused_update", 0)
    w = short[args.workload]
    steps = args.steps if args.steps is not None else w.iters
    if args.workload == "c5":
        return bench_ooc(args, w, steps, torch, fk, wl, dev)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # 1 GiB read + 1 GiB written per launch
        torch.cuda.synchronize()
        del src, dst

    out = measure(w, steps, args.warmup, args.repeats, torch, fk, wl, dev,
                  cpu=not args.no_cpu_baseline)
    if args.workload == "c2" and not args.no_other_configs:
        # the other in-core configurations, each at its own iteration count (short: < 1 s each)
        others = {}
        for ow in (wl.C1, wl.C3, wl.C4):
            r = measure(ow, ow.iters, args.warmup, max(5, min(args.repeats, 7)), torch, fk, wl, dev, cpu=False)
            others[ow.name] = {k: r[k] for k in ("config", "steps", "repeats", "ms_per_step", "ms_per_step_min",
                                                 "ms_per_step_max", "value", "dtype", "roofline",
                                                 "kernel_ms", "stage_interval_ms") if k in r}
            for k in ("assign_tflops", "update_gbps", "update_frac_of_hbm_peak", "fused_pass_gbps"):
                if k in r:
                    others[ow.name][k] = r[k]
        out["other_configs"] = others
    print(json.dumps(out))
    return 0


def _median(v):
    v = sorted(v)
    n = len(v)
    return v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def measure(w, steps, warmup, repeats, torch, fk, wl, dev, cpu=True):
    """One in-core configuration: throughput (median of `repeats` blocks of `steps` iterations,
    each block between a HIP event pair on the kernels' stream), per-stage event intervals, and
    kernel-only durations of the big kernels (stage timer with back-to-back repeats)."""
    X, lab = wl.make_points(w, device=dev, return_labels=True)
    idx = wl.init_rows(w, lab if w.zipf_s > 0 else None)
    C0 = wl.gather_rows(X, idx).contiguous()
    del lab
    ws = fk.make_workspace(w.B, w.N, w.d, w.K, w.torch_dtype, dev)
    C = C0.clone()
    assign = torch.empty((w.B, w.N), dtype=torch.int32, device=dev)
    counts = torch.empty((w.B, w.K), dtype=torch.int32, device=dev)
    C_lp = torch.empty((w.B, w.K, w.d), dtype=w.torch_dtype, device=dev)

    def run(iters):
        fk.fk_lloyd_iter(X, C, iters, ws=ws, C_lp=C_lp, assign=assign, counts=counts)

    # ---------------------------------------------------------------- throughput
    # The part leaves its idle clock only under sustained load (1.2 GHz idle; the first tens of
    # milliseconds of work run below the clock it then holds), so the device is first kept busy
    # for ~0.2 s with the same iteration, untimed; every timed block then starts from the initial
    # centroids, runs W untimed warm-up steps and K timed steps between two events recorded on
    # the stream the kernels run on (torch's current stream), with a device synchronisation on
    # both sides.  The median block is the reported figure.
    t_pre = time.perf_counter()
    prewarm = 0
    while time.perf_counter() - t_pre < 0.2:
        run(10)
        torch.cuda.synchronize()
        prewarm += 10
    block_ms, host_ms = [], []
    for _ in range(max(1, repeats)):
        C.copy_(C0)
        if warmup > 0:
            run(warmup)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        run(steps)
        e1.record()
        torch.cuda.synchronize()
        host_ms.append((time.perf_counter() - t0) * 1e3 / steps)
        block_ms.append(e0.elapsed_time(e1) / steps)
        assert int(counts.sum()) == w.B * w.N
    ms_per_step = _median(block_ms)

    # ---------------------------------------------------------------- per-stage (instrumented reruns)
    def staged(repeat):
        C.copy_(C0)
        if warmup > 0:
            run(warmup)
        torch.cuda.synchronize()
        fk.fk_set_option("timer_repeat", repeat)
        fk.fk_stage_timer_start()
        run(steps)
        st = fk.fk_stage_timer_stop()
        fk.fk_set_option("timer_repeat", 1)
        return {k: (v[0] / v[1] if v[1] else 0.0) for k, v in st.items()}   # ms per launch

    interval = staged(1)          # one launch between two events: over-reads the kernel
    kernel = staged(8)            # eight launches back to back per interval: the kernel's own time

    es = 4 if w.dtype == "fp32" else 2
    flops = 2.0 * w.B * w.N * w.K * w.d
    plan = fk.fk_plan(w.B, w.N, w.d, w.K, w.torch_dtype)
    fused = any(k in plan for k in ("stream_update", "table_update", "f32_update"))
    out = {
        "metric": "lloyd_iterations_per_s",
        "value": 1e3 / ms_per_step,
        "unit": "iterations/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step,
        "repeats": len(block_ms),
        "ms_per_step_min": min(block_ms), "ms_per_step_max": max(block_ms),
        "ms_per_step_host_clock_median": _median(host_ms),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"fp16": "f16", "bf16": "bf16", "fp32": "f32"}[w.dtype],
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "N": w.N, "d": w.d, "K": w.K,
                   "storage": w.dtype, "accumulate": "f32"},
        "plan": plan,
        "kernel_ms": kernel,
        "stage_interval_ms": interval,
        "prewarm_iterations_untimed": prewarm,
    }
    pass_bytes = w.B * (w.N * w.d * es + w.K * w.d * es + 4 * w.K + 4 * w.N)
    if fused and "f32_update" in plan:
        # fp32 storage, few clusters: the same one-pass structure, distances by direct differences
        # on the fp32 vector ALU (3 flop per point, centroid and feature): ALU-bound
        out["config"]["update"] = "fused into the assignment pass (fp32 table in registers)"
        t = 1.5 * flops / (kernel["assign"] * 1e-3) / 1e12
        out["assign_tflops"] = flops / (kernel["assign"] * 1e-3) / 1e12
        out["fused_pass_gbps"] = pass_bytes / (kernel["assign"] * 1e-3) / 1e9
        out["roofline"] = _roof("f32_update_kernel", "alu", t, PEAK_FP32_VALU_TFLOPS, "TFLOP/s", w,
                                kernel["assign"], interval["assign"])
    elif fused:
        # assignment and sums come out of ONE streaming pass over X (booked under "assign"; no
        # sort, no gather), followed by the merge/normalise.  HBM-bound: X and C read once, the
        # assignment written once.
        kname = "table_update_kernel" if "table_update" in plan else "stream_update_kernel"
        g = pass_bytes / (kernel["assign"] * 1e-3) / 1e9
        out["config"]["update"] = "fused into the assignment pass (one-hot MFMA table)"
        out["assign_tflops"] = flops / (kernel["assign"] * 1e-3) / 1e12
        out["fused_pass_gbps"] = g
        out["roofline"] = _roof(kname, "hbm", g, PEAK_HBM_GBPS, "GB/s", w, kernel["assign"], interval["assign"])
    else:
        assign_tflops = flops / (kernel["assign"] * 1e-3) / 1e12
        upd_bytes = w.B * (w.N * (w.d * es + 12) + w.K * w.d * (4 + es))
        # the update's share of an iteration: the timed iteration minus the assignment kernel's own
        # duration (everything else, launch gaps included); the sum of the stage intervals, which
        # also holds one event pair per stage, is kept beside it
        upd_ms = ms_per_step - kernel["assign"]
        upd_ms_stages = kernel["sort"] + kernel["reduce"] + kernel["finalize"]
        update_gbps = upd_bytes / (upd_ms * 1e-3) / 1e9
        out.update({
            "assign_tflops": assign_tflops,
            "assign_frac_of_mfma_peak": assign_tflops / PEAK_MFMA_F16_TFLOPS,
            "assign_gbps": pass_bytes / (kernel["assign"] * 1e-3) / 1e9,
            "update_gbps": update_gbps,
            "update_frac_of_hbm_peak": update_gbps / PEAK_HBM_GBPS,
            "update_ms": upd_ms,
            "update_ms_sum_of_stage_intervals": upd_ms_stages,
        })
        # dominant kernel: the assignment kernel wherever its contraction outweighs streaming X
        # (K above the MFMA/HBM ridge of ~312 flop/byte); otherwise the update's row gather
        if w.dtype != "fp32" and w.K >= 312:
            out["roofline"] = _roof("assign_mfma_kernel", "mfma", assign_tflops, PEAK_MFMA_F16_TFLOPS,
                                    "TFLOP/s", w, kernel["assign"], interval["assign"])
        elif w.dtype == "fp32":
            # 3 fp32 VALU flops (sub, mul, add) per (point, centroid, feature)
            t = 1.5 * flops / (kernel["assign"] * 1e-3) / 1e12
            out["roofline"] = _roof("assign_f32_kernel", "alu", t, PEAK_FP32_VALU_TFLOPS, "TFLOP/s", w,
                                    kernel["assign"], interval["assign"])
        else:
            # few centroids: both big kernels stream X; the row gather of the update is reported
            red_bytes = w.B * (w.N * (w.d * es + 4))
            g = red_bytes / (kernel["reduce"] * 1e-3) / 1e9
            out["roofline"] = _roof("segment_reduce_kernel", "hbm", g, PEAK_HBM_GBPS, "GB/s", w,
                                    kernel["reduce"], interval["reduce"])
    if cpu:
        out["cpu_baseline"] = cpu_baseline(w, X, C0, torch)
    del X, ws, assign
    torch.cuda.empty_cache()
    return out


def _roof(kname, bound, achieved, peak, unit, w, kernel_ms, interval_ms):
    """Roofline entry of the dominant kernel.  `achieved` uses the kernel's own mean duration
    (back-to-back launches between one event pair, live in this run); the single-launch event
    interval, which also holds the events' own cost, is kept beside it.  `traffic` is not measured
    in this run: it is the figure of the committed rocprofv3 --pmc summary, when there is one."""
    traffic = _traffic_from_profiles(kname, w.name)
    return {"kernel": kname, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
            "frac": achieved / peak, "avg_launch_ms": kernel_ms,
            "avg_launch_ms_single_event_interval": interval_ms,
            "traffic": traffic,
            "traffic_source": (f"profiles/{kname}_{w.name}_traffic.txt (offline rocprofv3 --pmc run)"
                               if traffic is not None else None)}


def _time_us(torch, fn, reps=5):
    fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e3


def compare_standard(torch, fk, wl, dev):
    """Kernel-level comparison of the paper's Section 5.2 on this machine: fused assign vs
    distance-matrix + argmin, sort-inverse update vs atomic scatter (fp16, Gaussian mixtures)."""
    out = {"metric": "kernel_level_comparison", "assign": [], "update": []}
    for (N, K, d) in [(1 << 16, 1024, 128), (1 << 20, 1024, 128), (1 << 20, 8192, 128), (1 << 18, 65536, 128)]:
        w = wl.C2.scaled(N=N, K=K, d=d)
        X = wl.make_points(w, device=dev)
        C = wl.gather_rows(X, wl.init_rows(w)).to(torch.float16)
        ws = fk.make_workspace(1, N, d, K, torch.float16, dev)
        D = torch.empty((1, N, K), dtype=torch.float32, device=dev)
        a = torch.empty((1, N), dtype=torch.int32, device=dev)
        t_fused = _time_us(torch, lambda: fk.fk_assign(X, C, ws=ws, out=a))
        t_std = _time_us(torch, lambda: fk.fk_standard_assign(X, C, D=D, ws=ws))
        a2, _ = fk.fk_standard_assign(X, C, D=D, ws=ws)
        same = float((a2 == fk.fk_assign(X, C, ws=ws)).float().mean())
        out["assign"].append({"N": N, "K": K, "d": d, "fused_us": t_fused, "standard_us": t_std,
                              "speedup": t_std / t_fused, "distance_matrix_bytes": 4 * N * K,
                              "same_assignment_fraction": same})
        del D, X
    for (N, K, d, zipf) in [(1 << 20, 1024, 128, 0.0), (1 << 25, 4096, 128, 0.0), (1 << 24, 16, 64, 1.2)]:
        w = wl.C2.scaled(N=N, K=K, d=d, zipf_s=zipf)
        X, lab = wl.make_points(w, device=dev, return_labels=True)
        C = torch.zeros((1, K, d), dtype=torch.float32, device=dev)
        ws = fk.make_workspace(1, N, d, K, torch.float16, dev)
        sums = torch.empty((1, K, d), dtype=torch.float32, device=dev)
        fk.fk_set_option("fused_update", 0)
        t_si = _time_us(torch, lambda: fk.fk_update(X, lab, C, ws=ws))
        fk.fk_set_option("fused_update", -1)
        t_at = _time_us(torch, lambda: fk.fk_standard_update(X, lab, C, sums=sums))
        nbytes = N * (d * 2 + 12)
        row = {"N": N, "K": K, "d": d, "zipf_s": zipf, "sort_inverse_us": t_si,
               "atomic_scatter_us": t_at, "speedup": t_at / t_si,
               "sort_inverse_gbps": nbytes / t_si / 1e3,
               "atomic_scatter_gbps": N * (d * 2 + 4) / t_at / 1e3}
        if "stream_update" in fk.fk_plan(1, N, d, K, torch.float16):
            # few clusters: the sort-free one-hot MFMA update reads X (and the ids) once, streaming
            t_oh = _time_us(torch, lambda: fk.fk_update(X, lab, C, ws=ws))
            row.update({"streamed_onehot_us": t_oh, "streamed_onehot_gbps": N * (d * 2 + 4) / t_oh / 1e3,
                        "speedup_onehot_over_sort_inverse": t_si / t_oh})
        out["update"].append(row)
        del X, lab
    print(json.dumps(out))
    return 0


def clock_trace(torch, fk, dev):
    """What shader clock the part holds under each kind of load (rocm-smi, sampled twice a second
    from a side thread while the kernel is launched back to back)."""
    import re
    import subprocess
    import threading

    def sclk():
        try:
            out = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=10).stdout
            m = re.search(r"sclk clock level: \d+: \((\d+)Mhz\)", out)
            return int(m.group(1)) if m else None
        except Exception:
            return None

    def loop(fn, secs=3.0):
        seen, stop = [], threading.Event()

        def sampler():
            while not stop.is_set():
                v = sclk()
                if v is not None:
                    seen.append(v)
                time.sleep(0.5)
        th = threading.Thread(target=sampler)
        th.start()
        t0 = time.time()
        while time.time() - t0 < secs:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()
        stop.set()
        th.join()
        return seen[1:] if len(seen) > 1 else seen          # the first sample may predate the load

    N, d = 1 << 20, 128
    X = (torch.randn(1, N, d, device=dev) * 4).half()
    # The headline shape (same instructions, same schedule) on operands that toggle the
    # multipliers less: what the instruction stream sustains with the power limit out of the way.
    # Timed before the first rocm-smi call (median of three interleaved rounds); the clocks under
    # each are sampled further down.
    Kp = 1024
    ws_p = fk.make_workspace(1, N, d, Kp, torch.float16, dev)
    a_p = torch.empty((1, N), dtype=torch.int32, device=dev)
    Cp = (torch.randn(1, Kp, d, device=dev) * 4).half()
    probe = [{"operands": name, "_ops": ops} for name, ops in (
        ("gaussian X, gaussian C", (X, Cp)),
        ("all-zero X and C", (torch.zeros_like(X), torch.zeros_like(Cp))),
        ("all-one X and C", (torch.ones_like(X), torch.ones_like(Cp))),
        ("gaussian X, all-zero C", (X, torch.zeros_like(Cp))))]
    t0 = time.time()
    while time.time() - t0 < 0.3:
        fk.fk_assign(X, Cp, ws=ws_p, out=a_p)
    torch.cuda.synchronize()
    rounds = [[_time_us(torch, lambda: fk.fk_assign(*row["_ops"], ws=ws_p, out=a_p), reps=40) for row in probe]
              for _ in range(3)]
    for i, row in enumerate(probe):
        us = sorted(r[i] for r in rounds)[1]
        row["us_per_call_incl_centroid_layout"] = us
        row["tflops"] = 2.0 * N * Kp * d / us / 1e6
    out = {"metric": "shader_clock_under_load_mhz", "idle": sclk(), "loads": []}
    for K in (16384, 1024, 256):
        C = (torch.randn(1, K, d, device=dev) * 4).half()
        ws = fk.make_workspace(1, N, d, K, torch.float16, dev)
        a = torch.empty((1, N), dtype=torch.int32, device=dev)
        us = _time_us(torch, lambda: fk.fk_assign(X, C, ws=ws, out=a))
        out["loads"].append({"load": f"fk_assign N=2^20 d=128 K={K} fp16", "sclk_mhz": loop(lambda: fk.fk_assign(X, C, ws=ws, out=a)),
                             "tflops": 2.0 * N * K * d / us / 1e6})
    for row in probe:
        Xo, Co = row.pop("_ops")
        row["sclk_mhz"] = loop(lambda: fk.fk_assign(Xo, Co, ws=ws_p, out=a_p), secs=2.0)
    out["operand_data"] = probe
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    out["loads"].append({"load": "1 GiB device-to-device copy", "sclk_mhz": loop(lambda: dst.copy_(src))})
    print(json.dumps(out))
    return 0


def sweep_choices(torch, fk, dev):
    """Both sides of two host-side choices, with the side the shape rule picks."""
    out = {"metric": "kernel_choice_rules", "assign_small_k": [], "sort_scatter": []}
    f16 = torch.float16
    for (N, d) in ((1 << 24, 64), (1 << 22, 64), (1 << 20, 64), (1 << 22, 128), (1 << 20, 128), (1 << 22, 32)):
        X = (torch.randn(1, N, d, device=dev) * 4).half()
        for K in (16, 64, 128, 256):
            if K > 32 * (16 // max(2, d // 16)):
                continue                                   # C no longer fits one LDS stage
            C = (torch.randn(1, K, d, device=dev) * 4).half()
            ws = fk.make_workspace(1, N, d, K, f16, dev)
            a = torch.empty((1, N), dtype=torch.int32, device=dev)
            us = {}
            for name, v in (("sweep", 0), ("stream", 1), ("rule", -1)):
                fk.fk_set_option("assign_stream", v)
                us[name] = round(_time_us(torch, lambda: fk.fk_assign(X, C, ws=ws, out=a)), 1)
            fk.fk_set_option("assign_stream", -1)
            plan = fk.fk_plan(1, N, d, K, f16)
            out["assign_small_k"].append({"N": N, "d": d, "K": K, "us": us,
                                          "rule_picks": "stream" if "mfma_stream" in plan else "sweep"})
        del X
    for (B, N, K) in ((1, 1 << 20, 256), (1, 1 << 20, 1024), (1, 1 << 20, 2048), (32, 32768, 256), (1, 1 << 24, 16),
                      (1, 1 << 24, 64), (1, 1 << 24, 1024), (1, 1 << 22, 2048), (1, 1 << 24, 65536), (1, 1 << 25, 4096)):
        a = torch.randint(0, K, (B, N), dtype=torch.int32, device=dev)
        ws = torch.empty(fk.fk_workspace_bytes(B, N, 8, K, torch.float32), dtype=torch.uint8, device=dev)
        us = {}
        for name, v in (("direct", 0), ("staged_up_to_2048_bins", 2048), ("rule", -1)):
            fk.fk_set_option("sort_stage_bins", v)
            us[name] = round(_time_us(torch, lambda: fk.fk_sort_inverse(a, K, ws=ws)), 1)
        fk.fk_set_option("sort_stage_bins", -1)
        out["sort_scatter"].append({"B": B, "N": N, "K": K, "us": us})
        del a, ws
    print(json.dumps(out))
    return 0


def sweep_variants(torch, fk, dev):
    """Exhaustive sweep of the sweeping assign kernel's four tile shapes against the pick of
    the shape heuristic (fk_plan), fp16, over a grid of (N, K, d)."""
    rows = []
    t_sweep = 0.0
    for d in (64, 128):
        for K in (256, 1024, 4096, 16384):
            for N in (1 << 16, 1 << 18, 300000, 1 << 20, 1 << 22):
                if N * K * d > 2 ** 41:
                    continue
                X = (torch.randn(1, N, d, device=dev) * 4).half()
                C = (torch.randn(1, K, d, device=dev) * 4).half()
                ws = fk.make_workspace(1, N, d, K, torch.float16, dev)
                a = torch.empty((1, N), dtype=torch.int32, device=dev)
                # three rounds over all candidates (so that clock drift hits them alike), the best
                # round of each kept; every timing is 10 launches after 3 untimed ones
                us = {v: float("inf") for v in (0, 1, 2, 3, -1)}
                for _ in range(3):
                    for v in (0, 1, 2, 3, -1):
                        fk.fk_set_option("assign_variant", v)
                        t0 = time.perf_counter()
                        for _ in range(3):
                            fk.fk_assign(X, C, ws=ws, out=a)
                        torch.cuda.synchronize()
                        e0 = torch.cuda.Event(enable_timing=True)
                        e1 = torch.cuda.Event(enable_timing=True)
                        e0.record()
                        for _ in range(10):
                            fk.fk_assign(X, C, ws=ws, out=a)
                        e1.record()
                        torch.cuda.synchronize()
                        us[v] = min(us[v], e0.elapsed_time(e1) / 10 * 1e3)
                        if v >= 0:
                            t_sweep += time.perf_counter() - t0
                best = min(us[v] for v in (0, 1, 2, 3))
                rows.append({"d": d, "K": K, "N": N, "us": {str(k): round(x, 1) for k, x in us.items()},
                             "plan": next(p for p in fk.fk_plan(1, N, d, K, torch.float16).split() if "mfma_" in p),
                             "heuristic_over_best": round(us[-1] / best, 3)})
    fk.fk_set_option("assign_variant", -1)
    r = [x["heuristic_over_best"] for x in rows]
    print(json.dumps({"metric": "assign_variant_heuristic", "shapes": len(rows),
                      "mean_heuristic_over_best": sum(r) / len(r), "worst_heuristic_over_best": max(r),
                      "exhaustive_sweep_seconds": t_sweep, "rows": rows}))
    return 0


def cpu_baseline(w, X, C0, torch):
    """The fp64 oracle as it stands, timed on this machine's host cores on a bounded sample."""
    import numpy as np
    import oracle
    # sample: instance 0, the first n_s points against all K centroids, sized for ~10-20 s
    budget_pairs = 6.0e11            # (point, centroid, feature) triples for the timed sample
    n_s = int(min(w.N, max(1024, budget_pairs / (w.K * w.d) / 2)))
    Xs = X[0, :n_s].to(torch.float32).cpu().numpy()
    Cs = C0[0].cpu().numpy().astype(np.float64)
    oracle.assign(Xs[:256], Cs)      # load the library, warm the threads
    reps, t0 = 0, time.perf_counter()
    while reps < 2 or (time.perf_counter() - t0 < 10.0 and reps < 64):   # about 10 s of wall clock
        r = oracle.assign(Xs, Cs)
        u = oracle.update(Xs, r["assign"], Cs)
        Cs = u["C"]
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    full = dt * (w.N / n_s) * w.B    # one iteration over the whole workload, extrapolated
    return {"value": 1.0 / full, "unit": "iterations/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{reps} iterations (assign+update) on the first {n_s} of {w.N} points of "
                      f"instance 0, all {w.K} centroids; {dt:.3f} s each, scaled by "
                      f"{w.N / n_s * w.B:g} to the full workload"}


def bench_ooc(args, w, steps, torch, fk, wl, dev):
    """Out-of-core configuration: X in pinned host memory, streamed in 2^24-row chunks through
    a device working set capped at 32 GB.  FK_OOC_ROWS overrides N (smaller boxes)."""
    cap = 32 << 30
    N = int(os.environ.get("FK_OOC_ROWS", w.N))
    w = w.scaled(N=N)
    t0 = time.perf_counter()
    Xh = torch.empty((1, w.N, w.d), dtype=w.torch_dtype, pin_memory=True)
    print(f"pinned {Xh.numel() * 2 / 2**30:.1f} GiB in {time.perf_counter() - t0:.1f} s",
          file=sys.stderr, flush=True)
    # generated on the GPU block by block, each block copied down into the pinned buffer
    wl.make_points(w, device=dev, rows_per_block=1 << 24, out=Xh)
    print(f"generated in {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)
    idx = wl.init_rows(w)
    C = Xh[0][idx[0]].to(torch.float32).to(dev).contiguous()
    C0 = C.clone()
    chunk = min(1 << 24, w.N)
    need = fk.fk_ooc_workspace_bytes(chunk, w.d, w.K, w.torch_dtype)
    assert 0 < need <= cap - (1 << 30), need
    dev_ws = torch.empty(need, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    if args.warmup > 0:
        fk.fk_lloyd_ooc(Xh[0], C, 1, dev_ws=dev_ws, chunk_rows=chunk, keep_assign=False)
    print(f"warm-up done at {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)
    t1 = time.perf_counter()
    a, counts = fk.fk_lloyd_ooc(Xh[0], C, steps, dev_ws=dev_ws, chunk_rows=chunk, keep_assign=False)
    elapsed = time.perf_counter() - t1
    assert int(counts.sum()) == w.N
    ms = elapsed * 1e3 / steps
    flops = 2.0 * w.N * w.K * w.d
    tf = flops / (ms * 1e-3) / 1e12
    out = {"metric": "lloyd_iterations_per_s", "value": 1e3 / ms, "unit": "iterations/s",
           "n_gpus": 1, "steps": steps, "warmup": min(args.warmup, 1), "ms_per_step": ms,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
           "data": "synthetic",
           "config": {"workload": w.name, "B": 1, "N": w.N, "d": w.d, "K": w.K,
                      "storage": w.dtype, "chunk_rows": chunk, "device_workspace_bytes": need,
                      "device_cap_bytes": cap, "x": "pinned host memory"},
           "end_to_end_tflops": tf,
           "host_to_device_gbps": w.N * w.d * 2 / (ms * 1e-3) / 1e9,
           "roofline": {"kernel": "assign_mfma_kernel", "bound": "mfma", "achieved": tf,
                        "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s",
                        "frac": tf / PEAK_MFMA_F16_TFLOPS, "traffic": None,
                        "note": "whole iteration including the PCIe stream, not the kernel alone"}}
    if not args.no_cpu_baseline:
        # sampled: the oracle cannot redo this size; its rate on the sample is scaled up
        out["cpu_baseline"] = cpu_baseline(w, Xh, C0[None], torch)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

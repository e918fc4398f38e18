#!/usr/bin/env python3
"""Benchmark of the brick SpMM hot path on one MI355X.

A step is one spmm_exec (C = A.B) over a seeded synthetic matrix that is already
resident in HBM together with its plan; plan construction (the paper's
pre-processing, excluded from its kernel timings in Section 6.2/6.3) is timed
separately and reported as `plan_ms`.  The headline workload is the largest
single-GPU configuration, the FEM-like matrix (M = K = 923,136, 41 M entries) at
N = 128.  The default run also times two more workloads and reports them under
`extra`: the clustered 262,144-row matrix and the million-row High-synergy sweep
(the input on which the HBM-roofline target is stated).

Prints one JSON line:  metric = effective GFLOP/s = 2 nnz N / t.

`--sweep` instead prints the config-5 grid (five fills x six widths, brick kernel
against CSR kernel) plus configs 1 and 3 per route, one JSON object per line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X published dense fp32 matrix peak
DEFAULT_WORKLOAD = "fem_923k"
EXTRA_WORKLOADS = ("clustered_262k", "sweepxl_f0.8")

WORKLOADS = {
    # name: (config index, kwargs, default N)
    "tiny_banded_4k": (1, {}, 32),
    "clustered_262k": (2, {}, 128),
    "powerlaw_326k": (3, {}, 128),
    "fem_923k": (4, {}, 128),
    "sweep_65k_f0.05": (5, {"fill": 0.05}, 128),
    "sweep_65k_f0.1": (5, {"fill": 0.1}, 128),
    "sweep_65k_f0.2": (5, {"fill": 0.2}, 128),
    "sweep_65k_f0.4": (5, {"fill": 0.4}, 128),
    "sweep_65k_f0.8": (5, {"fill": 0.8}, 128),
}
ROUTES = {"auto": 0, "mfma": 1, "valu": 2, "class": 3}


def make_workload(name):
    from paper_2504_06443_amd import workloads as W
    if name.startswith("sweepxl_"):            # scaled-up sweep: exceeds the 256 MB Infinity Cache
        fill = float(name.split("_f")[1])
        return W.brick_sweep(fill, M=1 << 20, target_nnz=32_000_000, seed=1005), 128
    if name.startswith("paired_"):             # 32-row groups with common active columns
        rows = {"262k": 262144, "923k": 923136}[name.split("_")[1]]
        return W.paired_panels(rows, cols_per_group=240, half_width=1024, row_fill=0.19,
                               seed=1006), 128
    idx, kw, n = WORKLOADS[name]
    A, _ = W.config(idx, **kw)
    return A, n


def kernel_source_hash():
    """Identifies the kernels a stored traffic figure was measured with."""
    h = hashlib.sha256()
    for fn in ("exec_kernels.hip", "exec_bf16.hip", "tm32_kernels.hip", "exec_common.h",
               "spmm_internal.h"):
        with open(os.path.join(ROOT, "paper_2504_06443_amd", "csrc", fn), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def stored_traffic(workload, N, mode):
    """HBM-side bytes per launch from the committed rocprofv3 summary of this workload, or None
    when there is none or it was taken with other kernels than the ones now in the tree."""
    suffix = "" if mode == "fp32" else f"_{mode}"
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}_N{N}{suffix}.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for ln in open(path):
        if ln.strip() and not ln.startswith("#"):
            k, v = ln.split()[:2]
            vals[k] = v
    if vals.get("kernel_source_sha256_16") != kernel_source_hash():
        return None
    return float(vals["hbm_bytes_per_launch"])


def cpu_baseline(A, B, budget_s=20.0):
    """The CPU oracle as it stands, timed on this machine's host cores."""
    import oracle
    t0 = time.perf_counter()
    oracle.spmm_f64(A.rowptr, A.colind, A.vals, B, want_abs=False)     # warm-up
    first = time.perf_counter() - t0
    reps = max(1, min(3, int(budget_s / max(first, 1e-3)) - 1))
    times = []
    for _ in range(reps):
        t0 = time.perf_counter()
        oracle.spmm_f64(A.rowptr, A.colind, A.vals, B, want_abs=False)
        times.append(time.perf_counter() - t0)
    t = statistics.median(times) if times else first
    return {
        "value": 2.0 * A.nnz * B.shape[1] / t / 1e9,
        "unit": "GFLOP/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"full workload (all {A.M} rows, N={B.shape[1]}), fp64 CSR SpMM, "
                  f"median of {max(1, len(times))} run(s) after 1 warm-up",
        "seconds": t,
    }


def measure(spmm, name, N, steps, warmup, route="auto", split=0, order="panel", cold=False,
            mode="fp32", time_plan=True, keep=None, panel_height=16):
    """Plans `name`, runs warmup + steps products and returns the measurements as a dict.
    `keep`, if a dict, receives A and the first B (for the cpu_baseline leg)."""
    import numpy as np
    import torch
    from paper_2504_06443_amd import workloads as W

    dev = torch.device("cuda:0")
    A, n_default = make_workload(name)
    N = N or n_default
    rp = torch.from_numpy(A.rowptr).to(dev)
    ci = torch.from_numpy(A.colind).to(dev)
    va = torch.from_numpy(A.vals).to(dev)

    # plan (pre-processing), timed on its own
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = spmm.spmm_plan(A.M, A.K, rp, ci, va)
    torch.cuda.synchronize()
    plan_first_ms = (time.perf_counter() - t0) * 1e3
    plan_ms = None
    if time_plan:
        t0 = time.perf_counter()
        plan2 = spmm.spmm_plan(A.M, A.K, rp, ci, va)
        torch.cuda.synchronize()
        plan_ms = (time.perf_counter() - t0) * 1e3
        spmm.spmm_plan_destroy(plan2)

    spmm.spmm_plan_set_route(plan, ROUTES[route])
    spmm.spmm_plan_set_split(plan, split)
    spmm.spmm_plan_set_order(plan, 1 if order == "heavy" else 0)
    if mode != "fp32":
        spmm.spmm_plan_set_precision(plan, spmm.PRECISIONS[mode])
    tm32 = None
    if panel_height == 32:
        spmm.spmm_plan_set_panel_height(plan, 32)
        tm32 = spmm.spmm_plan_tm32_sizes(plan)
    syn = spmm.spmm_synergy(plan, N)
    wl = spmm.spmm_plan_worklist(plan, N)

    n_pairs = 1
    if cold:
        pair_bytes = 4.0 * N * (A.K + A.M)
        n_pairs = int(max(2, min(16, np.ceil(1.5e9 / pair_bytes))))
    Bs = [torch.from_numpy(W.dense_b(A.K, N, 2000 + i)).to(dev) for i in range(n_pairs)]
    Cs = [torch.empty((A.M, N), dtype=torch.float32, device=dev) for _ in range(n_pairs)]
    if keep is not None:
        keep["A"], keep["B"] = A, Bs[0].cpu().numpy()

    stream = torch.cuda.current_stream()
    for i in range(warmup):
        spmm.spmm_exec(plan, Bs[i % n_pairs], Cs[i % n_pairs], stream)
    torch.cuda.synchronize()

    # HIP events on the stream the kernels are launched on bracket every product
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        starts[i].record(stream)
        spmm.spmm_exec(plan, Bs[i % n_pairs], Cs[i % n_pairs], stream)
        stops[i].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps
    ev_ms = [a.elapsed_time(b) for a, b in zip(starts, stops)]
    kernel_ms = statistics.fmean(ev_ms)          # all kernels of one exec, on their own stream
    kernel_ms_med = statistics.median(ev_ms)

    flops = 2.0 * A.nnz * N
    # algorithmic work of the dominant kernel (the MFMA brick kernel unless everything is
    # routed to the CSR kernel): issued flops = 128 flop per brick and column of C
    issued_flops = 128.0 * (tm32["n_bricks"] if tm32 else
                            sum(b1 - b0 for _, b0, b1, _, _ in wl["items"])) * N
    hbm_achieved = syn["bytes_min"] / (kernel_ms * 1e-3) / 1e9
    mfma_achieved = issued_flops / (kernel_ms * 1e-3) / 1e12
    traffic = stored_traffic(name, N, mode) if (route == "auto" and split == 0) else None
    time_note = "mean HIP-event time of one spmm_exec (kernel_ms_mean)"
    roof_hbm = {"bound": "hbm", "achieved": hbm_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": hbm_achieved / HBM_PEAK_GBS, "traffic": traffic,
                "bytes_model": "bytes_min = 4 nnz + 28 bricks + 4 + 4 (panels + 1) + 4 N distinct "
                               "columns + 4 N M", "time": time_note,
                "traffic_over_bytes_min": (traffic / syn["bytes_min"]) if traffic else None}
    roof_mfma = {"bound": "mfma", "achieved": mfma_achieved, "peak": MFMA_FP32_PEAK_TFLOPS,
                 "unit": "TFLOP/s", "frac": mfma_achieved / MFMA_FP32_PEAK_TFLOPS,
                 "traffic": traffic, "flops_model": "issued = 128 flop x bricks x N "
                 "(zero-filled 16x4 bricks; useful flops / alpha)", "time": time_note}
    mfma_binds = wl["n_mfma_items"] > 0 and syn["roof_gflops_mfma"] < syn["roof_gflops_hbm"] \
        and mode == "fp32"
    return {
        "workload": name, "M": A.M, "K": A.K, "nnz": A.nnz, "N": N,
        "value": flops / (ms_per_step * 1e-3) / 1e9,
        "ms_per_step": ms_per_step,
        "kernel_ms_mean": kernel_ms,
        "kernel_ms_median": kernel_ms_med,
        "plan_ms": plan_ms,
        "plan_first_ms": plan_first_ms,
        "bc_pairs": n_pairs,
        "synergy": {"alpha_brick": syn["alpha_brick"], "class": syn["synergy_class"],
                    "oi_shmem": syn["oi_shmem"], "n_bricks": syn["n_bricks"],
                    "panels_by_class": syn["panels_by_class"],
                    "roof_gflops_hbm": syn["roof_gflops_hbm"],
                    "roof_gflops_mfma": syn["roof_gflops_mfma"],
                    "bytes_min": syn["bytes_min"], "bytes_noreuse": syn["bytes_noreuse"]},
        "worklist": {k: wl[k] for k in ("n_mfma_items", "n_valu_panels", "n_split_panels",
                                        "num_waves", "n_tile", "n_tiles", "num_cus",
                                        "resident_waves_per_cu")},
        "tm32": tm32,
        "roofline": roof_mfma if mfma_binds else roof_hbm,
        "roofline_hbm": roof_hbm,
        "roofline_mfma": roof_mfma,
    }


def sweep(spmm, steps, warmup):
    """Config-5 grid and configs 1/3 per route, one JSON line each."""
    for f in ("0.05", "0.1", "0.2", "0.4", "0.8"):
        for n in (16, 32, 64, 128, 256, 512):
            for route in ("mfma", "valu"):
                r = measure(spmm, f"sweep_65k_f{f}", n, steps, warmup, route=route, time_plan=False)
                print(json.dumps({k: r[k] for k in ("workload", "N", "kernel_ms_mean", "value")} |
                                 {"route": route, "alpha": r["synergy"]["alpha_brick"],
                                  "class": r["synergy"]["class"]}), flush=True)
    for name, routes in (("powerlaw_326k", ("auto", "class", "valu")),
                         ("tiny_banded_4k", ("mfma", "valu")),
                         ("clustered_262k", ("auto", "valu")), ("fem_923k", ("auto", "valu"))):
        for route in routes:
            r = measure(spmm, name, 0, steps, warmup, route=route, time_plan=False)
            print(json.dumps({k: r[k] for k in ("workload", "N", "kernel_ms_mean", "value")} |
                             {"route": route, "split_panels": r["worklist"]["n_split_panels"],
                              "valu_panels": r["worklist"]["n_valu_panels"]}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--n", type=int, default=0, help="columns of B (default: the workload's)")
    ap.add_argument("--route", default="auto", choices=list(ROUTES))
    ap.add_argument("--split", type=int, default=0,
                    help="0: Eq. 6-7, split from ratio 2; -1: Eq. 6-7, nearest; 1: never; k: force k")
    ap.add_argument("--order", default="panel", choices=["panel", "heavy"],
                    help="work-item order: panel order, or heaviest first (the schedule the paper rejects)")
    ap.add_argument("--mode", default="fp32", choices=["fp32", "bf16x3", "bf16x6"],
                    help="arithmetic of the brick kernel: fp32 (default), or the opt-in split-bf16 "
                         "modes (three / six bf16 products per FP32 product)")
    ap.add_argument("--panel-height", type=int, default=16, choices=[16, 32],
                    help="32: build and use the 32-row panel format (two bricks per brick column "
                         "share one B operand)")
    ap.add_argument("--cold", action="store_true",
                    help="rotate over several B/C pairs so that no step finds its operands in cache")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-extra", action="store_true",
                    help="time only --workload (the default run adds two more workloads under `extra`)")
    ap.add_argument("--sweep", action="store_true", help="print the synergy-sweep grid instead")
    ap.add_argument("--calibrate-gather", action="store_true",
                    help="measure the random-row gather bandwidth of this GPU (the memory ceiling "
                         "for inputs whose B rows cannot be reused) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of known size (1 GiB, 10 times): the "
                         "reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    if not os.path.exists(os.path.join(ROOT, "paper_2504_06443_amd", "libspmm_brick.so")):
        from paper_2504_06443_amd.build import build_library   # nothing built yet: build once
        build_library(verbose=False)
    from paper_2504_06443_amd import binding as spmm

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.calibrate_copy:
        n = (1 << 30) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n * 4, "calibrate_copy_bytes_written": n * 4,
                          "launches": 10}), flush=True)
        return
    if args.calibrate_gather:
        # what the memory system delivers for the brick kernel's way of reading B (random rows of
        # 512 bytes), from buffers that fit one L2, the L2s together, the Infinity Cache, and only HBM
        sink = torch.zeros(256, dtype=torch.float32, device=dev)
        buf = torch.zeros((2 << 30) // 4, dtype=torch.float32, device=dev)
        st = torch.cuda.current_stream()
        n_waves, loads = 256 * 16, 2048
        for mb in (2, 16, 128, 2048):
            n_rows = (mb << 20) // 512
            for _ in range(2):
                spmm.spmm_calibrate_gather(buf, n_rows, loads, n_waves, sink, st)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(5):
                spmm.spmm_calibrate_gather(buf, n_rows, loads, n_waves, sink, st)
            e1.record(st)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            print(json.dumps({"calibrate_gather_buffer_MB": mb, "ms": ms,
                              "TB_per_s": n_waves * loads * 1024 / (ms * 1e-3) / 1e12}), flush=True)
        return
    if args.sweep:
        sweep(spmm, args.steps, args.warmup)
        return

    keep = {}
    r = measure(spmm, args.workload, args.n, args.steps, args.warmup, route=args.route,
                split=args.split, order=args.order, cold=args.cold, mode=args.mode, keep=keep,
                panel_height=args.panel_height)
    out = {
        "metric": "SpMM effective GFLOP/s (2*nnz*N/t)",
        "value": r["value"],
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if args.mode == "fp32" else args.mode,
        "data": "synthetic",
        "config": {"workload": args.workload, "M": r["M"], "K": r["K"], "nnz": r["nnz"], "N": r["N"],
                   "route": args.route, "split": args.split, "order": args.order,
                   "mode": args.mode, "panel_height": args.panel_height, "cold": bool(args.cold),
                   "bc_pairs": r["bc_pairs"]},
    }
    for k in ("kernel_ms_mean", "kernel_ms_median", "plan_ms", "plan_first_ms", "synergy", "worklist", "tm32",
              "roofline", "roofline_hbm", "roofline_mfma"):
        out[k] = r[k]
    out["achieved_hbm_gbs_model"] = r["roofline_hbm"]["achieved"]
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(keep["A"], keep["B"])
    keep.clear()
    default_run = (args.workload == DEFAULT_WORKLOAD and args.n == 0 and args.route == "auto"
                   and args.split == 0 and args.order == "panel" and args.mode == "fp32"
                   and args.panel_height == 16 and not args.cold)
    if default_run and not args.no_extra:
        extra = {}
        for name in EXTRA_WORKLOADS:
            torch.cuda.empty_cache()
            e = measure(spmm, name, 0, max(20, args.steps // 2), args.warmup, time_plan=False)
            extra[name] = {
                "N": e["N"], "nnz": e["nnz"], "ms": e["kernel_ms_mean"],
                "ms_per_step": e["ms_per_step"], "gflops": e["value"],
                "alpha_brick": e["synergy"]["alpha_brick"],
                "frac_mfma_peak": e["roofline_mfma"]["frac"],
                "frac_hbm_bytes_min": e["roofline_hbm"]["frac"],
                "bytes_min": e["synergy"]["bytes_min"],
                "traffic": e["roofline_hbm"]["traffic"],
                "traffic_over_bytes_min": e["roofline_hbm"]["traffic_over_bytes_min"],
                "time": e["roofline_hbm"]["time"],
            }
        out["extra"] = extra
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

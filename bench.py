#!/usr/bin/env python3
"""Benchmark of the brick SpMM hot path on one MI355X.

A step is one spmm_exec (C = A.B) over a seeded synthetic matrix that is already
resident in HBM together with its plan; plan construction (the paper's
pre-processing, excluded from its kernel timings in Section 6.2/6.3) is timed
separately and reported as `plan_ms`.  The default workload is the
clustered-structural configuration at N = 128.

Prints one JSON line:  metric = effective GFLOP/s = 2 nnz N / t.
"""
from __future__ import annotations

import argparse
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
L2_PEAK_GBS = 128 * 64 * 2.3   # derived: 8 XCDs x 16 channels x 64 B/clk x 2.3 GHz (measured clock)

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


def make_workload(name):
    from paper_2504_06443_amd import workloads as W
    if name.startswith("sweepxl_"):            # scaled-up sweep: exceeds the 256 MB Infinity Cache
        fill = float(name.split("_f")[1])
        return W.brick_sweep(fill, M=1 << 20, target_nnz=32_000_000, seed=1005), 128
    idx, kw, n = WORKLOADS[name]
    A, _ = W.config(idx, **kw)
    return A, n


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="clustered_262k")
    ap.add_argument("--n", type=int, default=0, help="columns of B (default: the workload's)")
    ap.add_argument("--route", default="auto", choices=["auto", "mfma", "valu", "class"])
    ap.add_argument("--split", type=int, default=0)
    ap.add_argument("--order", default="panel", choices=["panel", "heavy"],
                    help="work-item order: panel order, or heaviest first (the schedule the paper rejects)")
    ap.add_argument("--cold", action="store_true",
                    help="rotate over several B/C pairs so that no step finds its operands in cache")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of known size (1 GiB, 10 times): the "
                         "reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
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

    A, n_default = make_workload(args.workload)
    N = args.n or n_default
    rng_seed = 2000
    rp = torch.from_numpy(A.rowptr).to(dev)
    ci = torch.from_numpy(A.colind).to(dev)
    va = torch.from_numpy(A.vals).to(dev)

    # plan (pre-processing), timed on its own
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = spmm.spmm_plan(A.M, A.K, rp, ci, va)
    torch.cuda.synchronize()
    plan_first_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    plan2 = spmm.spmm_plan(A.M, A.K, rp, ci, va)
    torch.cuda.synchronize()
    plan_ms = (time.perf_counter() - t0) * 1e3
    spmm.spmm_plan_destroy(plan2)

    spmm.spmm_plan_set_route(plan, {"auto": 0, "mfma": 1, "valu": 2, "class": 3}[args.route])
    spmm.spmm_plan_set_split(plan, args.split)
    spmm.spmm_plan_set_order(plan, 1 if args.order == "heavy" else 0)
    syn = spmm.spmm_synergy(plan, N)
    wl = spmm.spmm_plan_worklist(plan, N)

    from paper_2504_06443_amd import workloads as W
    n_pairs = 1
    if args.cold:
        pair_bytes = 4.0 * N * (A.K + A.M)
        n_pairs = int(max(2, min(16, np.ceil(1.5e9 / pair_bytes))))
    Bs = [torch.from_numpy(W.dense_b(A.K, N, rng_seed + i)).to(dev) for i in range(n_pairs)]
    Cs = [torch.empty((A.M, N), dtype=torch.float32, device=dev) for _ in range(n_pairs)]

    stream = torch.cuda.current_stream()
    for i in range(args.warmup):
        spmm.spmm_exec(plan, Bs[i % n_pairs], Cs[i % n_pairs], stream)
    torch.cuda.synchronize()

    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        starts[i].record(stream)
        spmm.spmm_exec(plan, Bs[i % n_pairs], Cs[i % n_pairs], stream)
        stops[i].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    ev_ms = [a.elapsed_time(b) for a, b in zip(starts, stops)]
    kernel_ms = statistics.fmean(ev_ms)          # all kernels of one exec, on their own stream
    kernel_ms_med = statistics.median(ev_ms)

    flops = 2.0 * A.nnz * N
    value = flops / (ms_per_step * 1e-3) / 1e9

    # roofline of the dominant kernel (the MFMA brick kernel unless everything is routed to VALU)
    issued_flops = 128.0 * sum(b1 - b0 for _, b0, b1, _, _ in wl["items"]) * \
        wl["n_tiles"] * wl["n_tile"]
    hbm_achieved = syn["bytes_min"] / (kernel_ms * 1e-3) / 1e9
    mfma_achieved = issued_flops / (kernel_ms * 1e-3) / 1e12
    roof_hbm = {"bound": "hbm", "achieved": hbm_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": hbm_achieved / HBM_PEAK_GBS, "traffic": None}
    roof_mfma = {"bound": "mfma", "achieved": mfma_achieved, "peak": MFMA_FP32_PEAK_TFLOPS,
                 "unit": "TFLOP/s", "frac": mfma_achieved / MFMA_FP32_PEAK_TFLOPS,
                 "traffic": None}
    # third ceiling, not one of the published peaks: every panel pulls its B rows through the
    # XCD's L2 (bytes_noreuse); 128 L2 channels x 64 B/clk x 2.3 GHz = 18.8 TB/s
    l2_achieved = syn["bytes_noreuse"] / (kernel_ms * 1e-3) / 1e9
    roof_l2 = {"bound": "l2", "achieved": l2_achieved, "peak": L2_PEAK_GBS, "unit": "GB/s",
               "frac": l2_achieved / L2_PEAK_GBS, "traffic": None}
    mfma_binds = wl["n_mfma_items"] > 0 and syn["roof_gflops_mfma"] < syn["roof_gflops_hbm"]
    roofline = roof_mfma if mfma_binds else roof_hbm
    traffic_file = os.path.join(ROOT, "profiles", f"traffic_{args.workload}_N{N}.txt")
    if os.path.exists(traffic_file) and args.route == "auto":
        for ln in open(traffic_file):
            if ln.startswith("hbm_bytes_per_launch"):
                roofline["traffic"] = roof_hbm["traffic"] = float(ln.split()[1])

    out = {
        "metric": "SpMM effective GFLOP/s (2*nnz*N/t)",
        "value": value,
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "M": A.M, "K": A.K, "nnz": A.nnz, "N": N,
                   "route": args.route, "order": args.order, "cold": bool(args.cold), "bc_pairs": n_pairs},
        "kernel_ms_mean": kernel_ms,
        "kernel_ms_median": kernel_ms_med,
        "plan_ms": plan_ms,
        "plan_first_ms": plan_first_ms,
        "synergy": {"alpha_brick": syn["alpha_brick"], "class": syn["synergy_class"],
                    "oi_shmem": syn["oi_shmem"], "n_bricks": syn["n_bricks"],
                    "panels_by_class": syn["panels_by_class"],
                    "roof_gflops_hbm": syn["roof_gflops_hbm"],
                    "roof_gflops_mfma": syn["roof_gflops_mfma"],
                    "bytes_min": syn["bytes_min"], "bytes_noreuse": syn["bytes_noreuse"]},
        "worklist": {k: wl[k] for k in ("n_mfma_items", "n_valu_panels", "n_split_panels",
                                        "num_waves", "n_tile", "n_tiles")},
        "achieved_hbm_gbs_model": hbm_achieved,
        "roofline": roofline,
        "roofline_hbm": roof_hbm,
        "roofline_mfma": roof_mfma,
        "roofline_l2": roof_l2,
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(A, Bs[0].cpu().numpy())
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

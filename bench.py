#!/usr/bin/env python3
"""Benchmark of the K-means hot path on one MI355X.

A step is one Lloyd iteration (assignment + update) over the whole synthetic workload, with X
resident in HBM.  Prints ONE JSON line: Lloyd iterations/s (the metric), the roofline position
of the dominant kernel (the assignment contraction, timed with HIP events on its own stream
inside the library), the CPU oracle timed on a bounded sample of the same workload, and the
fault-tolerance overhead.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2] [--ft off|on|both]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"f32": 157.3, "f64": 78.6}          # dense MFMA TFLOP/s, MI355X datasheet
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the assignment kernel (FT off), from two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE) scaled by the readings of a device copy of X in the same run;
# the summaries and commands are in profiles/<workload>_assign_update.txt
MEASURED_TRAFFIC_BYTES = {"c2": 43.0e6, "c3": 296.5e6, "c4": 5889.9e6, "c5": 3753.3e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--ft", default="both", choices=["off", "on", "both"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    return ap.parse_args()


def time_steps(ftk, torch, Xd, C, labels, mind, counts, absmax, ws, ft_mode, stats, steps):
    """Run `steps` Lloyd iterations (assign + update in place on C); returns seconds."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ftk.kmeans_assign(Xd, C, labels=labels, mindist=mind, ft_mode=ft_mode, stats=stats, workspace=ws)
        ftk.kmeans_update(Xd, labels, C, counts=counts, x_absmax=absmax, workspace=ws)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def cpu_baseline(w, X, C0, seconds):
    """The oracle as it stands, timed on the host cores for about `seconds`.

    If one full Lloyd iteration (assign + update over all N points) does not fit the budget, the
    first S points are used against all K centroids and the rate is scaled linearly in N;
    otherwise whole iterations are repeated (continuing the Lloyd sequence) until the budget is
    used."""
    from oracle import cpu as oracle
    N = X.shape[0]
    S = min(N, 2048)
    t0 = time.perf_counter()
    oracle.assign(X[:S], C0)
    t_probe = max(time.perf_counter() - t0, 1e-4)
    S = int(min(N, max(S, S * seconds / t_probe)))
    C = C0
    iters = 0
    t0 = time.perf_counter()
    while True:
        lab, _, _ = oracle.assign(X[:S], C)
        C, _ = oracle.update(X[:S], lab, C)
        iters += 1
        t = time.perf_counter() - t0
        if S < N or t >= seconds or iters >= 1000:
            break
    return {
        "value": iters * (S / N) / t,
        "unit": "iters/s",
        "cores": oracle.threads(),
        "kind": "oracle",
        "sample": "%d x (assign+update) of the first %d of %d points against all K=%d centroids took %.2f s%s"
                  % (iters, S, N, C0.shape[0], t, "; scaled linearly in N" if S < N else ""),
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only (this build has no multi-GPU path); got --gpus %d" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2408_01391_amd import binding as ftk, synth

    w = synth.WORKLOADS[args.workload]
    steps = args.steps if args.steps is not None else {"c1": 500, "c2": 200, "c3": 200, "c4": 40, "c5": 30}[w.name]
    dev = torch.device("cuda:0")
    X, _ = synth.make_points(w)
    C0 = X[synth.init_indices(w, w.N)].copy()
    Xd = torch.from_numpy(X).to(dev)
    C0d = torch.from_numpy(C0).to(dev)
    N, D, K = w.N, w.D, w.K
    labels = torch.empty(N, dtype=torch.int32, device=dev)
    mind = torch.empty(N, dtype=Xd.dtype, device=dev)
    counts = torch.empty(K, dtype=torch.int32, device=dev)
    ws = ftk.new_workspace(Xd, K, ftk.FT_CORRECT)
    absmax = ftk.absmax(Xd)
    stats = ftk.new_stats(dev)
    # one plain device-to-device copy of X: a kernel of known traffic (N*D*esz read + written)
    # against which the HBM byte counters of a profiler run can be scaled
    Xcopy = Xd.clone()
    del Xcopy

    results = {}
    modes = {"off": [("off", ftk.FT_OFF)], "on": [("on", ftk.FT_CORRECT)],
             "both": [("off", ftk.FT_OFF), ("on", ftk.FT_CORRECT), ("strict", ftk.FT_STRICT)]}[args.ft]
    for name, mode in modes:
        C = C0d.clone()
        time_steps(ftk, torch, Xd, C, labels, mind, counts, absmax, ws, mode, stats, args.warmup)
        sec = time_steps(ftk, torch, Xd, C, labels, mind, counts, absmax, ws, mode, stats, steps)
        # separate short pass with HIP events around the assignment kernel itself
        ftk.profile_enable(True)
        time_steps(ftk, torch, Xd, C, labels, mind, counts, absmax, ws, mode, stats, min(steps, 10))
        ftk.profile_enable(False)
        ms, launches = ftk.profile_read()
        results[name] = dict(sec=sec, kernel_ms=ms / max(launches, 1))

    primary = results["off"] if "off" in results else results["on"]
    flops = 2.0 * N * D * K
    esz = 4 if w.dtype == "f32" else 8
    algo_bytes = N * D * esz + N * (4 + esz) + K * D * esz
    kern_s = primary["kernel_ms"] * 1e-3
    tflops = flops / kern_s / 1e12
    out = {
        "metric": "lloyd_iterations_per_second",
        "value": steps / primary["sec"],
        "unit": "iters/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * primary["sec"] / steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: N=%d D=%d K=%d %s, seeded blobs, FT %s" % (
            w.name, N, D, K, w.dtype, "off" if "off" in results else "on")},
        "roofline": {
            "bound": "mfma",
            "kernel": "assign",
            "achieved": tflops,
            "peak": PEAK[w.dtype],
            "unit": "TFLOP/s",
            "frac": tflops / PEAK[w.dtype],
            "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
            "flops_per_launch": flops,
            "kernel_ms": primary["kernel_ms"],
            "hbm_gbs_algorithmic": algo_bytes / kern_s / 1e9,
            "hbm_frac": algo_bytes / kern_s / 1e9 / HBM_PEAK_GBS,
        },
    }
    out["stats"] = ftk.stats_dict(stats)
    if "off" in results and "on" in results:
        out["ft"] = {
            "iters_per_s_ft_on": steps / results["on"]["sec"],
            "overhead_step": results["on"]["sec"] / results["off"]["sec"] - 1.0,
            "overhead_assign_kernel": results["on"]["kernel_ms"] / results["off"]["kernel_ms"] - 1.0,
            "stats": ftk.stats_dict(stats),
        }
        if "strict" in results:  # labels guaranteed equal to a fault-free run (near-ties settled exactly)
            out["ft"]["strict_overhead_step"] = results["strict"]["sec"] / results["off"]["sec"] - 1.0
            out["ft"]["strict_overhead_assign_kernel"] = (results["strict"]["kernel_ms"] /
                                                          results["off"]["kernel_ms"] - 1.0)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, X, C0, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

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
MEASURED_TRAFFIC_BYTES = {"c2": 42.6e6, "c3": 311.5e6, "c4": 4687.5e6, "c5": 290.8e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--ft", default="both", choices=["off", "on", "both"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fast", action="store_true",
                    help="skip the extra timing of the split-bf16 fast assignment (fp32 workloads with D <= 32)")
    ap.add_argument("--ablation", action="store_true",
                    help="also time the naive and the unfused GEMM + arg-min variants of the assignment "
                         "(Section 3.1.1 / 3.1.2) and report them next to the fused kernel")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--inject-seconds", type=float, default=2.0,
                    help="run time of the bit-flip injection leg (workloads with a flip rate; 0 = skip)")
    return ap.parse_args()


def time_steps(ftk, torch, Xd, C, labels, mind, counts, absmax, ws, ft_mode, stats, steps):
    """Run `steps` Lloyd iterations (assign + update in place on C); returns seconds."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ftk.kmeans_assign(Xd, C, labels=labels, mindist=mind, ft_mode=ft_mode, stats=stats, workspace=ws)
        ftk.kmeans_update(Xd, labels, C, counts=counts, x_absmax=absmax, workspace=ws, ft_mode=ft_mode,
                          stats=stats if ft_mode != ftk.FT_OFF else None)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def time_updates(ftk, torch, Xd, C, labels, counts, absmax, ws, ft_mode, stats, reps):
    """`reps` update steps alone (labels fixed; C is rewritten with the same values); seconds."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        ftk.kmeans_update(Xd, labels, C, counts=counts, x_absmax=absmax, workspace=ws, ft_mode=ft_mode,
                          stats=stats if ft_mode != ftk.FT_OFF else None)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def time_steps_injected(ftk, torch, np, w, Xd, C, labels, mind, counts, absmax, ws, stats, rate, step_s, seconds):
    """FT on (correct mode) with single-bit flips arriving as a Poisson process of `rate` per second
    of run time (fault model of Section 2.1): a seeded schedule draws, per Lloyd step, how many
    accumulator elements of that step's assignment are corrupted, at uniformly random positions and
    bits.  Runs for about `seconds`; returns (steps, seconds, flips scheduled)."""
    code = ftk.F32 if w.dtype == "f32" else ftk.F64
    geom = ftk.assign_geometry(code, w.N, w.D, w.K, ftk.FT_CORRECT)
    steps = max(50, int(seconds / step_s))
    rng = np.random.default_rng(w.seed + 77)
    per_step = rng.poisson(rate * step_s, size=steps)
    plan = {}
    for i in np.flatnonzero(per_step):
        rows = [(int(rng.integers(geom.workgroups)), int(rng.integers(geom.waves_per_workgroup)),
                 int(rng.integers(geom.tiles_per_wave)), int(rng.integers(geom.regs_per_tile)),
                 int(rng.integers(geom.lanes)), int(rng.integers(geom.bits))) for _ in range(per_step[i])]
        plan[int(i)] = ftk.make_faults(rows, Xd.device)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ftk.kmeans_assign(Xd, C, labels=labels, mindist=mind, ft_mode=ftk.FT_CORRECT, faults=plan.get(i),
                          stats=stats, workspace=ws)
        ftk.kmeans_update(Xd, labels, C, counts=counts, x_absmax=absmax, workspace=ws, ft_mode=ftk.FT_CORRECT,
                          stats=stats)
    torch.cuda.synchronize()
    return steps, time.perf_counter() - t0, int(per_step.sum())


def fast_mode_times(ftk, torch, Xd, C0d, labels, mind, counts, absmax, ws, warmup, steps, sec_per_step_fp32):
    """Lloyd steps with the assignment on the split-bf16 matrix path (the counterpart of the paper's
    TF32 variant): reported next to the headline, never as the headline."""
    def run(n, C):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            ftk.kmeans_assign_fast(Xd, C, labels=labels, mindist=mind, workspace=ws)
            ftk.kmeans_update(Xd, labels, C, counts=counts, x_absmax=absmax, workspace=ws)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    C = C0d.clone()
    run(warmup, C)
    sec = run(steps, C)
    ftk.profile_enable(True)
    run(min(steps, 10), C)
    ftk.profile_enable(False)
    ms, launches = ftk.profile_read()
    ref, _ = ftk.kmeans_assign(Xd, C0d, workspace=ws)
    fast, _ = ftk.kmeans_assign_fast(Xd, C0d, workspace=ws)
    N, D = Xd.shape
    K = C0d.shape[0]
    kern_ms = ms / max(launches, 1)
    return {"iters_per_s": steps / sec, "ms_per_step": 1e3 * sec / steps,
            "speedup_vs_fp32_step": sec_per_step_fp32 / (sec / steps),
            "assign_kernels_ms": kern_ms, "dtype": "bf16x3 split of f32, f32 accumulate",
            "fp32_equivalent_tflops": 2.0 * N * D * K / (kern_ms * 1e-3) / 1e12,
            "labels_differing_from_fp32_path": int((ref != fast).sum().item())}


def ablation_times(ftk, torch, Xd, C, labels, mind, ws, esz):
    """Whole assignment (all its kernels) by the three steps of Section 3.1: milliseconds per call
    and the labels each variant changes against the fused kernel."""
    from paper_2408_01391_amd import ablation

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / reps

    N, K = Xd.shape[0], C.shape[0]
    res = {}
    ref = labels.clone()
    res["fused_ms"] = timed(lambda: ftk.kmeans_assign(Xd, C, labels=ref, mindist=mind, workspace=ws), 20)
    lab = torch.empty_like(labels)
    res["naive_ms"] = timed(lambda: ablation.naive_assign(Xd, C, labels=lab, mindist=mind), 3)
    res["naive_labels_differing"] = int((lab != ref).sum().item())
    if N * K * esz <= 48e9:
        gws = ablation.gemm_workspace(Xd, K)
        res["gemm_unfused_ms"] = timed(lambda: ablation.gemm_assign(Xd, C, labels=lab, mindist=mind, workspace=gws), 5)
        res["gemm_unfused_labels_differing"] = int((lab != ref).sum().item())
        res["gemm_unfused_product_bytes"] = N * K * esz
        del gws
    else:
        res["gemm_unfused_ms"] = None  # the N x K product alone would take more than 48 GB
    return res


def cpu_baseline(w, X, C0, seconds, gpu_labels0):
    """The oracle as it stands, timed on the host cores for about `seconds`.

    Its first assignment (against the initial centroids) doubles as a parity sample: the GPU
    labels of the same rows are compared and the disagreements classified by the tie band.

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
    agreement = None
    t0 = time.perf_counter()
    while True:
        lab, best, _ = oracle.assign(X[:S], C)
        if iters == 0:
            t_pause = time.perf_counter()
            import numpy as np
            g = gpu_labels0[:S]
            diff = np.flatnonzero(g != lab)
            tol = 1e-5 if w.dtype == "f32" else 1e-12
            d_gpu = ((X[diff].astype(np.float64) - C0[g[diff]].astype(np.float64)) ** 2).sum(1)
            inside = int((d_gpu - best[diff] <= tol * best[diff]).sum())
            agreement = {"rows": int(S), "identical": int(S - diff.size), "differ_inside_tie_band": inside,
                         "differ_outside_tie_band": int(diff.size - inside), "tie_band_rel": tol}
            t0 += time.perf_counter() - t_pause  # the comparison is not oracle time
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
        "label_agreement_first_assign": agreement,
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
        "config": {"workload": "%s: N=%d D=%d K=%d %s, seeded %s, FT %s" % (
            w.name, N, D, K, w.dtype, w.kind, "off" if "off" in results else "on")},
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
        # update step alone, plain and under dual modular redundancy
        reps = max(20, steps // 2)
        time_updates(ftk, torch, Xd, C, labels, counts, absmax, ws, ftk.FT_OFF, stats, 10)
        t_plain = time_updates(ftk, torch, Xd, C, labels, counts, absmax, ws, ftk.FT_OFF, stats, reps)
        time_updates(ftk, torch, Xd, C, labels, counts, absmax, ws, ftk.FT_CORRECT, stats, 10)
        t_dmr = time_updates(ftk, torch, Xd, C, labels, counts, absmax, ws, ftk.FT_CORRECT, stats, reps)
        out["ft"]["update_ms"] = 1e3 * t_plain / reps
        out["ft"]["update_dmr_overhead"] = t_dmr / t_plain - 1.0
        if w.flips_per_s > 0 and args.inject_seconds > 0:
            inj_stats = ftk.new_stats(dev)
            C = C0d.clone()
            time_steps(ftk, torch, Xd, C, labels, mind, counts, absmax, ws, ftk.FT_CORRECT, stats, args.warmup)
            n_inj, sec_inj, flips = time_steps_injected(ftk, torch, np, w, Xd, C, labels, mind, counts, absmax, ws,
                                                        inj_stats, w.flips_per_s, results["on"]["sec"] / steps,
                                                        args.inject_seconds)
            st = ftk.stats_dict(inj_stats)
            out["ft"]["under_injection"] = {
                "flips_per_s": w.flips_per_s, "steps": n_inj, "seconds": sec_inj,
                "iters_per_s": n_inj / sec_inj,
                "overhead_step": (sec_inj / n_inj) / (results["off"]["sec"] / steps) - 1.0,
                "scheduled": flips, "injected": st["injected"], "detected": st["detected"],
                "corrected": st["corrected"], "recomputed": st["recomputed"],
                "uncorrectable": st["uncorrectable"],
                "below_threshold": st["injected"] - st["detected"],
            }
        if "strict" in results:  # labels guaranteed equal to a fault-free run (near-ties settled exactly)
            out["ft"]["strict_overhead_step"] = results["strict"]["sec"] / results["off"]["sec"] - 1.0
            out["ft"]["strict_overhead_assign_kernel"] = (results["strict"]["kernel_ms"] /
                                                          results["off"]["kernel_ms"] - 1.0)
    if w.dtype == "f32" and D <= 32 and D % 4 == 0 and not args.no_fast:
        out["fast_mode"] = fast_mode_times(ftk, torch, Xd, C0d, labels, mind, counts, absmax, ws, args.warmup, steps,
                                           primary["sec"] / steps)
    if args.ablation:
        out["ablation"] = ablation_times(ftk, torch, Xd, C0d, labels, mind, ws, esz)
    if not args.no_cpu_baseline:
        lab0, _ = ftk.kmeans_assign(Xd, C0d, labels=labels, mindist=mind, workspace=ws)
        torch.cuda.synchronize()
        out["cpu_baseline"] = cpu_baseline(w, X, C0, args.cpu_seconds, lab0.cpu().numpy())
    print(json.dumps(out))


if __name__ == "__main__":
    main()

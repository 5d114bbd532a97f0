#!/usr/bin/env python3
"""Benchmark of the K-means hot path on one MI355X.

A step is one Lloyd iteration (assignment + update) over a whole synthetic workload, with X
resident in HBM.  Prints ONE JSON line.  The headline (`value`, `roofline`, `cpu_baseline`) is the
largest workload, c5; the `configs` object carries the same measurements for all five workloads:
Lloyd iterations/s, the roofline position of the dominant kernel (the assignment contraction,
timed with HIP events on its own stream inside the library) and of the whole assignment call,
the fault-tolerance overhead in the mode that guarantees fault-free results (strict) and in the
paper's mode, and - where the workload names a flip rate - a run under injected bit flips that is
compared, step by step, with the fault-free run on the same inputs.

Every timing is the median of `--repeats` repetitions of a `--steps`-long loop, after `--warmup`
untimed steps, so that the figure does not depend on how far the clocks had ramped up.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5] [--configs all|none|c2,c3]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"f32": 157.3, "f64": 78.6}          # dense MFMA TFLOP/s, MI355X datasheet
HBM_PEAK_GBS = 8000.0
DEFAULT_STEPS = {"c1": 200, "c2": 100, "c3": 100, "c4": 20, "c5": 10}
ALL = ["c1", "c2", "c3", "c4", "c5"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="Lloyd steps per timed repetition (default: per workload, 10 for c5 ... 200 for c1)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--repeats", type=int, default=11, help="timed repetitions; the median is reported")
    ap.add_argument("--workload", default="c5", choices=ALL, help="headline workload")
    ap.add_argument("--configs", default="all",
                    help="workloads measured into the `configs` object: all, none, or a comma list")
    ap.add_argument("--ft", default="both", choices=["off", "both"],
                    help="off: skip the fault-tolerance legs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fast", action="store_true",
                    help="skip the extra timing of the split-bf16 fast assignment (fp32 workloads with D <= 128)")
    ap.add_argument("--ablation", action="store_true",
                    help="also time the naive and the unfused GEMM + arg-min variants of the assignment "
                         "(Section 3.1.1 / 3.1.2) of the headline workload")
    ap.add_argument("--batched", action="store_true",
                    help="also time the batched Lloyd step (ftk_kmeans_step_batched: assign a batch of rows, add "
                         "it to the sums while cache-resident) of the headline workload at several batch sizes")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--inject-seconds", type=float, default=1.5,
                    help="run time of the bit-flip injection leg (workloads with a flip rate; 0 = skip)")
    return ap.parse_args()


class State:
    """Device-resident inputs and scratch of one workload."""

    def __init__(self, w, torch, ftk, synth):
        self.w = w
        self.X, _ = synth.make_points(w)
        self.C0 = self.X[synth.init_indices(w, w.N)].copy()
        dev = torch.device("cuda:0")
        self.dev = dev
        self.Xd = torch.from_numpy(self.X).to(dev)
        self.C0d = torch.from_numpy(self.C0).to(dev)
        self.labels = torch.empty(w.N, dtype=torch.int32, device=dev)
        self.mind = torch.empty(w.N, dtype=self.Xd.dtype, device=dev)
        self.counts = torch.empty(w.K, dtype=torch.int32, device=dev)
        self.ws = ftk.new_workspace(self.Xd, w.K, ftk.FT_STRICT)
        self.absmax = ftk.absmax(self.Xd)
        # one plain device-to-device copy of X: a kernel of known traffic (N*D*esz read + written)
        # against which the HBM byte counters of a profiler run can be scaled
        Xcopy = self.Xd.clone()
        del Xcopy


def lloyd_steps(ftk, s, C, mode, stats, n, faults_by_step=None):
    """n Lloyd iterations in place on C (assignment + update, both in fault-tolerance `mode`)."""
    for i in range(n):
        ftk.kmeans_assign(s.Xd, C, labels=s.labels, mindist=s.mind, ft_mode=mode, stats=stats, workspace=s.ws,
                          faults=None if faults_by_step is None else faults_by_step.get(i))
        ftk.kmeans_update(s.Xd, s.labels, C, counts=s.counts, x_absmax=s.absmax, workspace=s.ws, ft_mode=mode,
                          stats=stats if mode != ftk.FT_OFF else None)


def median_step_seconds(torch, ftk, s, mode, stats, steps, warmup, repeats):
    """Median over `repeats` of the wall time of a `steps`-long Lloyd loop, per step."""
    C = s.C0d.clone()
    lloyd_steps(ftk, s, C, mode, stats, warmup)
    times = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        lloyd_steps(ftk, s, C, mode, stats, steps)
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) / steps)
    return statistics.median(times), times, C


def event_ms(torch, fn, reps):
    """Median GPU time of fn() in milliseconds, HIP events on the current stream around each call."""
    out = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        out.append(e0.elapsed_time(e1))
    return statistics.median(out)


def kernel_and_call_ms(torch, ftk, s, C, mode, reps=15):
    """(contraction kernel, whole assignment call, update call) in ms for centroids C.
    Kernel: HIP events recorded by the library around the kernel on the caller's stream, median of
    per-launch readings.  Calls: events around the binding call (prologue + kernel + refine)."""
    def assign():
        ftk.kmeans_assign(s.Xd, C, labels=s.labels, mindist=s.mind, ft_mode=mode, workspace=s.ws)

    for _ in range(3):
        assign()
    ks = []
    for _ in range(reps):
        ftk.profile_enable(True)
        assign()
        ftk.profile_enable(False)
        ms, n = ftk.profile_read()
        ks.append(ms / max(n, 1))
    call = event_ms(torch, assign, reps)
    Cu = C.clone()
    upd = event_ms(torch, lambda: ftk.kmeans_update(s.Xd, s.labels, Cu, counts=s.counts, x_absmax=s.absmax,
                                                    workspace=s.ws, ft_mode=mode), reps)
    return statistics.median(ks), call, upd


def injection_leg(torch, ftk, np, s, rate, step_s, seconds, warmup):
    """Strict fault tolerance under single-bit flips arriving as a Poisson process of `rate` per
    second of run time (fault model of Section 2.1): a seeded schedule draws, per Lloyd step, how
    many accumulator elements of that step's assignment are corrupted, at uniformly random
    positions and bits.

    Timing: the schedule is run for about `seconds`.  Verification: every step of the schedule that
    carries a flip is then replayed next to a fault-free twin on the same centroids - labels after
    the assignment and centroids after the update must be identical, and the counts are reported."""
    w = s.w
    code = ftk.F32 if w.dtype == "f32" else ftk.F64
    geom = ftk.assign_geometry(code, w.N, w.D, w.K, ftk.FT_STRICT)
    steps = max(50, int(seconds / step_s))
    rng = np.random.default_rng(w.seed + 77)
    per_step = rng.poisson(rate * step_s, size=steps)
    plan = {}
    for i in np.flatnonzero(per_step):
        rows = [(int(rng.integers(geom.workgroups)), int(rng.integers(geom.waves_per_workgroup)),
                 int(rng.integers(geom.tiles_per_wave)), int(rng.integers(geom.regs_per_tile)),
                 int(rng.integers(geom.lanes)), int(rng.integers(geom.bits))) for _ in range(per_step[i])]
        plan[int(i)] = ftk.make_faults(rows, s.dev)
    stats = ftk.new_stats(s.dev)
    C = s.C0d.clone()
    lloyd_steps(ftk, s, C, ftk.FT_STRICT, None, warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    lloyd_steps(ftk, s, C, ftk.FT_STRICT, stats, steps, plan)
    torch.cuda.synchronize()
    sec = time.perf_counter() - t0
    st = ftk.stats_dict(stats)

    # replay of the faulty steps against a fault-free twin, from the initial centroids on
    C = s.C0d.clone()
    lab_twin = torch.empty_like(s.labels)
    n_lab = n_cen = n_rep = 0
    for i in sorted(plan):
        Cf, Ct = C.clone(), C.clone()
        ftk.kmeans_assign(s.Xd, C, labels=s.labels, mindist=s.mind, ft_mode=ftk.FT_STRICT, faults=plan[i],
                          workspace=s.ws)
        ftk.kmeans_update(s.Xd, s.labels, Cf, counts=s.counts, x_absmax=s.absmax, workspace=s.ws,
                          ft_mode=ftk.FT_STRICT)
        ftk.kmeans_assign(s.Xd, C, labels=lab_twin, mindist=s.mind, ft_mode=ftk.FT_STRICT, workspace=s.ws)
        ftk.kmeans_update(s.Xd, lab_twin, Ct, counts=s.counts, x_absmax=s.absmax, workspace=s.ws,
                          ft_mode=ftk.FT_STRICT)
        n_lab += int((s.labels != lab_twin).sum().item())
        n_cen += int((Cf != Ct).any(dim=1).sum().item())
        n_rep += 1
        C = Cf
    return {
        "mode": "strict", "flips_per_s": rate, "steps": steps, "seconds": sec, "iters_per_s": steps / sec,
        "scheduled": int(per_step.sum()), "injected": st["injected"], "detected": st["detected"],
        "corrected": st["corrected"], "recomputed": st["recomputed"], "uncorrectable": st["uncorrectable"],
        "below_threshold": st["injected"] - st["detected"],
        "vs_no_fault_run": {"steps_replayed_with_fault_free_twin": n_rep, "labels_differing": n_lab,
                            "centroid_rows_differing": n_cen},
    }, sec / steps


def fast_mode_times(torch, ftk, s, steps, warmup, repeats, sec_per_step_fp32):
    """Lloyd steps with the assignment on the split-bf16 matrix path (the counterpart of the paper's
    TF32 variant), without and with its checksums (strict mode, DMR update): reported next to the
    headline, never as the headline."""
    def run(n, C, mode):
        for _ in range(n):
            ftk.kmeans_assign_fast(s.Xd, C, labels=s.labels, mindist=s.mind, workspace=s.ws, ft_mode=mode)
            ftk.kmeans_update(s.Xd, s.labels, C, counts=s.counts, x_absmax=s.absmax, workspace=s.ws, ft_mode=mode)

    def step_seconds(mode):
        C = s.C0d.clone()
        run(warmup, C, mode)
        times = []
        for _ in range(repeats):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(steps, C, mode)
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) / steps)
        return statistics.median(times), C

    sec, C = step_seconds(ftk.FT_OFF)
    ftk.profile_enable(True)
    run(5, C, ftk.FT_OFF)
    ftk.profile_enable(False)
    ms, launches = ftk.profile_read()
    sec_strict, _ = step_seconds(ftk.FT_STRICT)
    ref, _ = ftk.kmeans_assign(s.Xd, s.C0d, workspace=s.ws)
    fast, _ = ftk.kmeans_assign_fast(s.Xd, s.C0d, workspace=s.ws)
    stats = ftk.new_stats(s.Xd.device)
    fast_ft, _ = ftk.kmeans_assign_fast(s.Xd, s.C0d, workspace=s.ws, ft_mode=ftk.FT_STRICT, stats=stats)
    torch.cuda.synchronize()
    w = s.w
    kern_ms = ms / max(launches, 1)
    return {"iters_per_s": 1.0 / sec, "ms_per_step": 1e3 * sec, "speedup_vs_fp32_step": sec_per_step_fp32 / sec,
            "assign_kernels_ms": kern_ms,
            "dtype": "bf16x%d split of f32, f32 accumulate" % (3 if w.D <= 32 else 2),
            "fp32_equivalent_tflops": 2.0 * w.N * w.D * w.K / (kern_ms * 1e-3) / 1e12,
            "labels_differing_from_fp32_path": int((ref != fast).sum().item()),
            "ft_strict": {"iters_per_s": 1.0 / sec_strict, "overhead_step": sec_strict / sec - 1.0,
                          "speedup_vs_fp32_step_ft_off": sec_per_step_fp32 / sec_strict,
                          "labels_differing_from_fp32_path": int((ref != fast_ft).sum().item()),
                          "stats": ftk.stats_dict(stats)}}


def ablation_times(ftk, torch, s, esz):
    """Whole assignment (all its kernels) by the steps of Section 3.1: milliseconds per call
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

    N, K = s.w.N, s.w.K
    res = {}
    ref = s.labels.clone()
    res["fused_ms"] = timed(lambda: ftk.kmeans_assign(s.Xd, s.C0d, labels=ref, mindist=s.mind, workspace=s.ws), 20)
    lab = torch.empty_like(s.labels)
    res["naive_ms"] = timed(lambda: ablation.naive_assign(s.Xd, s.C0d, labels=lab, mindist=s.mind), 3)
    res["naive_labels_differing"] = int((lab != ref).sum().item())
    if N * K * esz <= 48e9:
        gws = ablation.gemm_workspace(s.Xd, K)
        res["gemm_unfused_ms"] = timed(lambda: ablation.gemm_assign(s.Xd, s.C0d, labels=lab, mindist=s.mind,
                                                                    workspace=gws), 5)
        res["gemm_unfused_labels_differing"] = int((lab != ref).sum().item())
        res["gemm_unfused_product_bytes"] = N * K * esz
        del gws
    else:
        res["gemm_unfused_ms"] = None  # the N x K product alone would take more than 48 GB
    for variant in (2, 3):  # Sections 3.1.3 / 3.1.4: GEMM on the plain ALUs with the minimum fused in
        if variant == 3 and esz == 8:
            continue  # its atomic key packs an fp32 distance
        fws = ablation.fused_alu_workspace(s.Xd, K, variant)
        res["fused_alu_v%d_ms" % variant] = timed(
            lambda: ablation.fused_alu_assign(s.Xd, s.C0d, variant, labels=lab, mindist=s.mind, workspace=fws), 3)
        res["fused_alu_v%d_labels_differing" % variant] = int((lab != ref).sum().item())
        del fws
    return res


def batched_step_times(torch, ftk, s, steps, warmup, repeats, sec_per_step):
    """The single-pass idea of Section 2.2 as batches: milliseconds per Lloyd step of
    ftk_kmeans_step_batched by batch size, next to the two-call step."""
    w = s.w
    esz = 4 if w.dtype == "f32" else 8
    rows_out = []
    for mb in (32, 64, 128, 256, 512, 1024):
        rows = int(mb * 2 ** 20 // (w.D * esz))
        if rows >= w.N:
            break
        C = s.C0d.clone()

        def run(n):
            for _ in range(n):
                ftk.kmeans_step_batched(s.Xd, C, rows, labels=s.labels, mindist=s.mind, counts=s.counts,
                                        x_absmax=s.absmax, workspace=s.ws)
        run(warmup)
        times = []
        for _ in range(repeats):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(steps)
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) / steps)
        sec = statistics.median(times)
        rows_out.append({"batch_MB": mb, "batch_rows": rows, "batches": -(-w.N // rows), "ms_per_step": 1e3 * sec,
                         "vs_two_call_step": sec / sec_per_step - 1.0})
    return {"two_call_ms_per_step": 1e3 * sec_per_step, "by_batch_size": rows_out}


def cpu_baseline(w, X, C0, seconds, gpu_labels0):
    """The oracle as it stands, timed on the host cores for about `seconds`.

    Its first assignment (against the initial centroids) doubles as a parity sample: the GPU
    labels of the same rows are compared and the disagreements classified by the tie band.

    If one full Lloyd iteration (assign + update over all N points) does not fit the budget, the
    first S points are used against all K centroids and the rate is scaled linearly in N;
    otherwise whole iterations are repeated (continuing the Lloyd sequence) until the budget is
    used."""
    import numpy as np
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


def profiled_traffic(name):
    """HBM bytes per launch of the assignment kernel (FT off) from the committed rocprofv3 counter
    summary of this workload (FETCH_SIZE + WRITE_SIZE, scaled by a device copy of known size), or
    None if the summary does not hold it."""
    path = os.path.join(ROOT, "profiles", "%s_assign_update.txt" % name)
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bytes_per_launch_assign_ft_off\s*[:=]\s*([0-9.eE+]+)", text, flags=re.M)
    return float(m.group(1)) if m else None


def measure(name, args, torch, ftk, synth, np, headline):
    """All measurements of one workload; returns (summary dict, State)."""
    w = synth.WORKLOADS[name]
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[name]
    s = State(w, torch, ftk, synth)
    esz = 4 if w.dtype == "f32" else 8
    flops = 2.0 * w.N * w.D * w.K
    algo_bytes = w.N * w.D * esz + w.N * (4 + esz) + w.K * w.D * esz
    upd_bytes = w.N * (w.D * esz + 4) + w.K * w.D * esz
    legs = [("off", ftk.FT_OFF)]
    if args.ft == "both":
        legs += [("strict", ftk.FT_STRICT), ("correct", ftk.FT_CORRECT)]
    res = {}
    for leg, mode in legs:
        stats = ftk.new_stats(s.dev)   # a fresh counter block per leg
        sec, times, C_end = median_step_seconds(torch, ftk, s, mode, stats, steps, args.warmup, args.repeats)
        k_ms, call_ms, upd_ms = kernel_and_call_ms(torch, ftk, s, C_end, mode)
        res[leg] = dict(sec=sec, spread=(min(times), max(times)), kernel_ms=k_ms, call_ms=call_ms, update_ms=upd_ms,
                        stats=ftk.stats_dict(stats))
    off = res["off"]
    t_hbm, t_mfma = algo_bytes / (HBM_PEAK_GBS * 1e9), flops / (PEAK[w.dtype] * 1e12)
    tflops_k = flops / (off["kernel_ms"] * 1e-3) / 1e12
    tflops_c = flops / (off["call_ms"] * 1e-3) / 1e12
    out = {
        "workload": "%s: N=%d D=%d K=%d %s, seeded %s" % (w.name, w.N, w.D, w.K, w.dtype, w.kind),
        "dtype": w.dtype, "steps": steps, "repeats": args.repeats, "warmup": args.warmup,
        "iters_per_s": 1.0 / off["sec"], "ms_per_step": 1e3 * off["sec"],
        "ms_per_step_min_max": [1e3 * off["spread"][0], 1e3 * off["spread"][1]],
        "assign": {
            "bound": "mfma" if t_mfma >= t_hbm else "hbm",
            "kernel_ms": off["kernel_ms"], "call_ms": off["call_ms"],
            "tflops_kernel": tflops_k, "frac_mfma_kernel": tflops_k / PEAK[w.dtype],
            "tflops_call": tflops_c, "frac_mfma_call": tflops_c / PEAK[w.dtype],
            "hbm_gbs_algorithmic_kernel": algo_bytes / (off["kernel_ms"] * 1e-3) / 1e9,
            "frac_hbm_kernel": algo_bytes / (off["kernel_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "traffic_bytes_profiled": profiled_traffic(name), "algorithmic_bytes": algo_bytes,
        },
        "update": {"ms": off["update_ms"], "hbm_gbs_algorithmic": upd_bytes / (off["update_ms"] * 1e-3) / 1e9,
                   "frac_hbm": upd_bytes / (off["update_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if args.ft == "both":
        ft = {}
        for leg in ("strict", "correct"):
            r = res[leg]
            ft[leg] = {"iters_per_s": 1.0 / r["sec"],
                       "overhead_step": r["sec"] / off["sec"] - 1.0,
                       "overhead_assign_kernel": r["kernel_ms"] / off["kernel_ms"] - 1.0,
                       "overhead_assign_call": r["call_ms"] / off["call_ms"] - 1.0,
                       "overhead_update_dmr": r["update_ms"] / off["update_ms"] - 1.0,
                       "stats": r["stats"]}
        ft["guarantee"] = ("strict: labels and centroids equal the fault-free run under any single flip per "
                           "checked tile; correct: the paper's scheme, flips below the detection threshold pass")
        if w.flips_per_s > 0 and args.inject_seconds > 0:
            inj, sec_inj = injection_leg(torch, ftk, np, s, w.flips_per_s, res["strict"]["sec"],
                                         args.inject_seconds, args.warmup)
            inj["overhead_step_vs_ft_off"] = sec_inj / off["sec"] - 1.0
            ft["under_injection"] = inj
        out["ft"] = ft
    if w.dtype == "f32" and w.D <= 128 and w.D % 4 == 0 and not args.no_fast:
        out["fast_mode"] = fast_mode_times(torch, ftk, s, steps, args.warmup, args.repeats, off["sec"])
    if headline:
        if args.ablation:
            out["ablation"] = ablation_times(ftk, torch, s, esz)
        if args.batched:
            out["batched_step"] = batched_step_times(torch, ftk, s, steps, args.warmup, max(3, args.repeats // 2),
                                                     off["sec"])
    return out, s


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only (this build has no multi-GPU path); got --gpus %d" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2408_01391_amd import binding as ftk, synth

    if args.configs == "all":
        names = list(ALL)
    elif args.configs == "none":
        names = []
    else:
        names = [n for n in args.configs.split(",") if n in ALL]
    if args.workload not in names:
        names.append(args.workload)
    names.sort(key=lambda n: (n == args.workload, n))   # headline last: its state is kept for the CPU leg

    configs = {}
    head = head_state = None
    for name in names:
        is_head = name == args.workload
        summary, state = measure(name, args, torch, ftk, synth, np, is_head)
        configs[name] = summary
        if is_head:
            head, head_state = summary, state
        else:
            del state
            torch.cuda.empty_cache()

    w = head_state.w
    a = head["assign"]
    mfma_bound = a["bound"] == "mfma"
    out = {
        "metric": "lloyd_iterations_per_second",
        "value": head["iters_per_s"],
        "unit": "iters/s",
        "n_gpus": 1,
        "steps": head["steps"],
        "warmup": args.warmup,
        "repeats": args.repeats,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": head["workload"] + ", FT off (FT legs under configs.%s.ft)" % w.name,
                   "timing": "median of %d repetitions of a %d-step loop" % (args.repeats, head["steps"])},
        "roofline": {
            "bound": a["bound"],
            "kernel": "assignment contraction (fused arg-min)",
            "achieved": a["tflops_kernel"] if mfma_bound else a["hbm_gbs_algorithmic_kernel"],
            "peak": PEAK[w.dtype] if mfma_bound else HBM_PEAK_GBS,
            "unit": "TFLOP/s" if mfma_bound else "GB/s",
            "frac": a["frac_mfma_kernel"] if mfma_bound else a["frac_hbm_kernel"],
            "traffic": a["traffic_bytes_profiled"],
            "flops_per_launch": 2.0 * w.N * w.D * w.K,
            "kernel_ms": a["kernel_ms"],
            "frac_whole_call": a["frac_mfma_call"] if mfma_bound else None,
            "call_ms": a["call_ms"],
            "frac_hbm_algorithmic": a["frac_hbm_kernel"],
        },
        "configs": configs,
    }
    if "ft" in head:
        out["ft"] = {"mode": "strict", "overhead_step": head["ft"]["strict"]["overhead_step"],
                     "overhead_assign_kernel": head["ft"]["strict"]["overhead_assign_kernel"]}
    if not args.no_cpu_baseline:
        s = head_state
        lab0, _ = ftk.kmeans_assign(s.Xd, s.C0d, labels=s.labels, mindist=s.mind, workspace=s.ws)
        torch.cuda.synchronize()
        out["cpu_baseline"] = cpu_baseline(w, s.X, s.C0, args.cpu_seconds, lab0.cpu().numpy())
    print(json.dumps(out))


if __name__ == "__main__":
    main()

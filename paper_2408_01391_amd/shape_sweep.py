"""Shape sweep of the assignment step: an 8 x 8 grid of (D, K) at fixed N, as in the paper's
evaluation over 64 problem sizes (Section 5.1), reporting for every shape the kernel variant the
dispatcher picks, the kernel time and the fraction of the MFMA roofline.

    python -m paper_2408_01391_amd.shape_sweep [--dtype f32|f64] [--logn 17] [--ft off|on] [--tune]

With --tune it plays the part of the paper's kernel selection (Section 3.2: time the candidate
kernels per shape, keep the fastest): every assignment candidate (small-D kernel; generic kernel
with 1, 2 or 4 centroid tiles per chunk) and both update paths are forced in turn through
ftk_tuning_override, and the table shows the winner, its time, and what the built-in rule picks
when that differs.

Prints a markdown table (rows D, columns K).  Inputs are seeded loose blobs (synth.random_problem);
times are means over 10 launches after 3 warm-up launches, from the library's own HIP events."""
from __future__ import annotations

import argparse

import torch

from . import binding as ftk, synth

PEAK = {"f32": 157.3, "f64": 78.6}
GRID = (8, 16, 32, 64, 128, 256, 512, 1024)


def _time_assign(Xd, Cd, lab, md, ws, mode):
    for _ in range(3):
        ftk.kmeans_assign(Xd, Cd, labels=lab, mindist=md, ft_mode=mode, workspace=ws)
    ftk.profile_enable(True)
    for _ in range(10):
        ftk.kmeans_assign(Xd, Cd, labels=lab, mindist=md, ft_mode=mode, workspace=ws)
    ftk.profile_enable(False)
    ms, n = ftk.profile_read()
    return ms / n * 1e3  # us


def _time_update(Xd, lab, Cd, counts, absmax, ws):
    import time
    for _ in range(5):
        ftk.kmeans_update(Xd, lab, Cd, counts=counts, x_absmax=absmax, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        ftk.kmeans_update(Xd, lab, Cd, counts=counts, x_absmax=absmax, workspace=ws)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / 20 * 1e6


def tune(args):
    """Winner per shape among the forced candidates, against the built-in rule."""
    dev = torch.device("cuda:0")
    N = 1 << args.logn
    mode = ftk.FT_CORRECT if args.ft == "on" else ftk.FT_OFF
    rows_a, rows_u = [], []
    disagree = 0
    for D in args.grid_d:
        ca, cu = [], []
        for K in args.grid_k:
            X, C = synth.random_problem(100 + D + K, N, D, K, args.dtype, spread=6.0)
            Xd, Cd = torch.from_numpy(X).to(dev), torch.from_numpy(C).to(dev)
            ws = ftk.new_workspace(Xd, K, ftk.FT_CORRECT)
            lab = torch.empty(N, dtype=torch.int32, device=dev)
            md = torch.empty(N, dtype=Xd.dtype, device=dev)
            cands = {"g1": (0, 1), "g2": (0, 2), "g4": (0, 4)}
            if args.dtype == "f32" and D <= 32 and D % 4 == 0:
                cands["s"] = (1, -1)
            if args.dtype == "f32" and 32 < D <= 128 and D % 4 == 0:
                cands["m"] = (1, -1)
            if args.dtype == "f64":
                cands["g8"] = (0, 8)  # eight centroid tiles of one point tile (fp64 only)
            times = {}
            for name, (variant, tiles) in cands.items():
                ftk.tuning_override(variant, tiles, -1)
                times[name] = _time_assign(Xd, Cd, lab, md, ws, mode)
            ftk.tuning_override(-1, -1, -1)
            t_rule = _time_assign(Xd, Cd, lab, md, ws, mode)
            best = min(times, key=times.get)
            # the rule's pick is whichever candidate it coincides with in time (within noise)
            cell = "%s %.0f us" % (best, times[best])
            if t_rule > 1.05 * times[best]:
                cell += " (rule %.0f us)" % t_rule
                disagree += 1
            ca.append(cell)
            counts = torch.empty(K, dtype=torch.int32, device=dev)
            absmax = ftk.absmax(Xd)
            tu = {}
            for name, path in (("tables", 0), ("sorted", 1)):
                ftk.tuning_override(-1, -1, path)
                tu[name] = _time_update(Xd, lab, Cd, counts, absmax, ws)
            ftk.tuning_override(-1, -1, -1)
            tu_rule = _time_update(Xd, lab, Cd, counts, absmax, ws)
            bestu = min(tu, key=tu.get)
            cellu = "%s %.0f us" % (bestu, tu[bestu])
            if tu_rule > 1.05 * tu[bestu]:
                cellu += " (rule %.0f us)" % tu_rule
                disagree += 1
            cu.append(cellu)
            print("D=%d K=%d assign %s | rule %.1f ; update %s | rule %.1f" % (
                D, K, {k: round(v, 1) for k, v in times.items()}, t_rule,
                {k: round(v, 1) for k, v in tu.items()}, tu_rule), flush=True)
        rows_a.append((D, ca))
        rows_u.append((D, cu))
    for title, rows in (("Assignment kernel: fastest candidate (s = small-D, m = mid-D, gN = generic with N centroid tiles per chunk)", rows_a),
                        ("Update: fastest path (labels of the rule-picked assignment)", rows_u)):
        print()
        print("%s; N = 2^%d, %s, FT %s; in brackets the built-in rule where it is more than 5 %% slower" % (
            title, args.logn, args.dtype, args.ft))
        print("| D \\\\ K | " + " | ".join(str(k) for k in args.grid_k) + " |")
        print("|---|" + "---|" * len(args.grid_k))
        for D, cells in rows:
            print("| %d | " % D + " | ".join(cells) + " |")
    print()
    print("cells where the rule loses more than 5 %%: %d of %d" % (disagree, 2 * len(args.grid_d) * len(args.grid_k)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f32", choices=["f32", "f64"])
    ap.add_argument("--logn", type=int, default=17)
    ap.add_argument("--ft", default="off", choices=["off", "on"])
    ap.add_argument("--tune", action="store_true")
    ap.add_argument("--ds", default=None, help="comma-separated feature counts instead of the 8-point grid")
    ap.add_argument("--ks", default=None, help="comma-separated cluster counts instead of the 8-point grid")
    args = ap.parse_args()
    args.grid_d = tuple(int(v) for v in args.ds.split(",")) if args.ds else GRID
    args.grid_k = tuple(int(v) for v in args.ks.split(",")) if args.ks else GRID
    if args.tune:
        tune(args)
        return
    dev = torch.device("cuda:0")
    N = 1 << args.logn
    mode = ftk.FT_CORRECT if args.ft == "on" else ftk.FT_OFF
    rows = []
    for D in args.grid_d:
        cells = []
        for K in args.grid_k:
            X, C = synth.random_problem(100 + D + K, N, D, K, args.dtype, spread=6.0)
            Xd, Cd = torch.from_numpy(X).to(dev), torch.from_numpy(C).to(dev)
            ws = ftk.new_workspace(Xd, K, ftk.FT_CORRECT)
            lab = torch.empty(N, dtype=torch.int32, device=dev)
            md = torch.empty(N, dtype=Xd.dtype, device=dev)
            for _ in range(3):
                ftk.kmeans_assign(Xd, Cd, labels=lab, mindist=md, ft_mode=mode, workspace=ws)
            ftk.profile_enable(True)
            for _ in range(10):
                ftk.kmeans_assign(Xd, Cd, labels=lab, mindist=md, ft_mode=mode, workspace=ws)
            ftk.profile_enable(False)
            ms, n = ftk.profile_read()
            t = ms / n * 1e-3
            tf = 2.0 * N * D * K / t / 1e12
            # the register-resident kernels run eight waves per workgroup, the generic one four
            code = ftk.F32 if args.dtype == "f32" else ftk.F64
            resident = ftk.assign_geometry(code, N, D, K, mode).waves_per_workgroup == 8
            variant = ("s" if D <= 32 else "m") if resident else "g"
            cell = "%s %.0f us %.0f%%" % (variant, t * 1e6, 100.0 * tf / PEAK[args.dtype])
            # the split-bf16 fast path covers fp32 rows of up to 128 features
            if args.dtype == "f32" and D <= 128 and D % 4 == 0 and args.ft == "off":
                for _ in range(3):
                    ftk.kmeans_assign_fast(Xd, Cd, labels=lab, mindist=md, workspace=ws)
                ftk.profile_enable(True)
                for _ in range(10):
                    ftk.kmeans_assign_fast(Xd, Cd, labels=lab, mindist=md, workspace=ws)
                ftk.profile_enable(False)
                ms, n = ftk.profile_read()
                cell += " (fast %.0f us)" % (ms / n * 1e3)
            cells.append(cell)
            print("D=%d K=%d %s: %.1f us, %.1f TFLOP/s (%.0f%% of %.1f)" % (
                D, K, variant, t * 1e6, tf, 100.0 * tf / PEAK[args.dtype], PEAK[args.dtype]), flush=True)
        rows.append((D, cells))
    print()
    print("N = 2^%d, %s, FT %s; cell: variant (s = small-D, m = mid-D, g = generic), kernel time, %% of the MFMA peak"
          " (in brackets: kernels of the split-bf16 fast path on the same shape)" % (args.logn, args.dtype, args.ft))
    print("| D \\\\ K | " + " | ".join(str(k) for k in args.grid_k) + " |")
    print("|---|" + "---|" * len(args.grid_k))
    for D, cells in rows:
        print("| %d | " % D + " | ".join(cells) + " |")


if __name__ == "__main__":
    main()

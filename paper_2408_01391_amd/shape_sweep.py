"""Shape sweep of the assignment step: an 8 x 8 grid of (D, K) at fixed N, as in the paper's
evaluation over 64 problem sizes (Section 5.1), reporting for every shape the kernel variant the
dispatcher picks, the kernel time and the fraction of the MFMA roofline.

    python -m paper_2408_01391_amd.shape_sweep [--dtype f32|f64] [--logn 17] [--ft off|on]

Prints a markdown table (rows D, columns K).  Inputs are seeded loose blobs (synth.random_problem);
times are means over 10 launches after 3 warm-up launches, from the library's own HIP events."""
from __future__ import annotations

import argparse

import torch

from . import binding as ftk, synth

PEAK = {"f32": 157.3, "f64": 78.6}
GRID = (8, 16, 32, 64, 128, 256, 512, 1024)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f32", choices=["f32", "f64"])
    ap.add_argument("--logn", type=int, default=17)
    ap.add_argument("--ft", default="off", choices=["off", "on"])
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    N = 1 << args.logn
    mode = ftk.FT_CORRECT if args.ft == "on" else ftk.FT_OFF
    rows = []
    for D in GRID:
        cells = []
        for K in GRID:
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
            variant = "s" if (args.dtype == "f32" and D <= 32 and D % 4 == 0) else "g"
            cell = "%s %.0f us %.0f%%" % (variant, t * 1e6, 100.0 * tf / PEAK[args.dtype])
            if variant == "s" and args.ft == "off":  # the split-bf16 fast path covers the same shapes
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
    print("N = 2^%d, %s, FT %s; cell: variant (s = small-D, g = generic), kernel time, %% of the MFMA peak"
          " (in brackets: kernels of the split-bf16 fast path on the same shape)" % (args.logn, args.dtype, args.ft))
    print("| D \\\\ K | " + " | ".join(str(k) for k in GRID) + " |")
    print("|---|" + "---|" * len(GRID))
    for D, cells in rows:
        print("| %d | " % D + " | ".join(cells) + " |")


if __name__ == "__main__":
    main()

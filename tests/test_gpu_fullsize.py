"""Parity at the full workload sizes, in the launch configuration bench.py times.

The oracle cannot afford all N x K distances at these sizes, so the assignment is checked on
seeded samples of points (each against all K centroids), and the update - which is O(N D) - is
checked in full.  Where the workload asks for fault tolerance the same run is repeated with
FT on and with injected single-bit flips, and must reproduce the clean labels exactly."""
import numpy as np
import pytest
import torch

from oracle import cpu as oracle
from paper_2408_01391_amd import binding as ftk, synth
from tests.gpu_util import DEV, check_assign, check_centroids, to_dev

pytestmark = pytest.mark.gpu

SAMPLE = 4096


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c5", "c4"])
def test_full_size_workload(name):
    w = synth.WORKLOADS[name]
    print("full size", name, "generating", flush=True)
    X, _ = synth.make_points(w)
    C0 = X[synth.init_indices(w, w.N)].copy()
    Xd, Cd = to_dev(X), to_dev(C0)
    ws = ftk.new_workspace(Xd, w.K, ftk.FT_CORRECT)
    rows = np.sort(np.random.default_rng(w.seed).choice(w.N, size=min(SAMPLE, w.N), replace=False))

    print("full size", name, "assign FT off", flush=True)
    labels_d, mind_d = ftk.kmeans_assign(Xd, Cd, workspace=ws)
    torch.cuda.synchronize()
    labels, mind = labels_d.cpu().numpy(), mind_d.cpu().numpy()
    in_band, n = check_assign(X, C0, labels, mind, rows=rows)
    print("full size", name, "sampled %d points, %d labels inside the tie band" % (n, in_band), flush=True)
    assert labels.min() >= 0 and labels.max() < w.K

    print("full size", name, "update", flush=True)
    C_g = Cd.clone()
    _, counts = ftk.kmeans_update(Xd, labels_d, C_g, workspace=ws)
    torch.cuda.synchronize()
    C_o, counts_o = oracle.update(X, labels, C0)
    assert np.array_equal(counts.cpu().numpy(), counts_o)
    check_centroids(C_g.cpu().numpy(), C_o)

    if w.ft:
        print("full size", name, "assign FT on, clean", flush=True)
        stats = ftk.new_stats(DEV)
        lab_ft, _ = ftk.kmeans_assign(Xd, Cd, ft_mode=ftk.FT_CORRECT, stats=stats, workspace=ws)
        torch.cuda.synchronize()
        st = ftk.stats_dict(stats)
        lab_ft = lab_ft.cpu().numpy()
        check_assign(X, C0, lab_ft, rows=rows)
        assert st["detected"] == 0 and st["tiles_checked"] > 0, st
        assert st["max_residual_ppm"] < 700_000, st
        # FT on groups the centroids differently (30 per tile), so a point whose two nearest
        # centroids are closer than fp32 can tell may be settled by a different (fp32 vs fp64)
        # evaluation: any disagreement with the FT-off labels must lie inside the tie band
        differ = np.flatnonzero(lab_ft != labels)
        print("full size", name, "FT on/off labels differ at", differ.size, "points", flush=True)
        assert differ.size <= 1e-4 * w.N
        if differ.size:
            check_assign(X, C0, lab_ft, rows=differ)
            check_assign(X, C0, labels, rows=differ)

        print("full size", name, "assign FT on, injected flips", flush=True)
        code = ftk.F32 if w.dtype == "f32" else ftk.F64
        geom = ftk.assign_geometry(code, w.N, w.D, w.K, ftk.FT_CORRECT)
        rng = np.random.default_rng(w.seed + 1)
        nf = min(512, geom.workgroups)
        wgs = rng.choice(geom.workgroups, size=nf, replace=False)
        rows_f = [(int(g), int(rng.integers(geom.waves_per_workgroup)), int(rng.integers(geom.tiles_per_wave)),
                   int(rng.integers(geom.regs_per_tile)), int(rng.integers(64)), int(rng.integers(geom.bits)))
                  for g in wgs]
        # strict mode: identical labels whatever was flipped; default mode (the paper's scheme): a
        # flip below the detection threshold may move the one point whose score it hit
        lab_strict, _ = ftk.kmeans_assign(Xd, Cd, ft_mode=ftk.FT_STRICT, workspace=ws)
        lab_strict = lab_strict.cpu().numpy()
        for mode in (ftk.FT_STRICT, ftk.FT_CORRECT):
            stats = ftk.new_stats(DEV)
            lab_inj, _ = ftk.kmeans_assign(Xd, Cd, ft_mode=mode, faults=ftk.make_faults(rows_f, DEV),
                                           stats=stats, workspace=ws)
            torch.cuda.synchronize()
            st = ftk.stats_dict(stats)
            print("full size", name, "mode", mode, "FT stats", st, flush=True)
            assert st["injected"] == nf
            assert st["corrected"] + st["recomputed"] == st["detected"] and st["uncorrectable"] == 0
            if mode == ftk.FT_STRICT:
                assert np.array_equal(lab_inj.cpu().numpy(), lab_strict)
            else:
                assert (lab_inj.cpu().numpy() != lab_ft).sum() <= nf

"""The split-bf16 fast assignment for rows of 36 .. 128 features (two bf16 pieces per operand,
point pieces in registers, centroid pieces LDS-resident or staged in chunks) against the oracle:
the same bar as the fp32 path in every fault-tolerance mode, and the injection experiments of
Sections 2.1 / 5.3 on it."""
import numpy as np
import pytest
import torch

from paper_2408_01391_amd import binding as ftk, synth
from tests.gpu_util import DEV, check_assign, check_moved_labels_within_detection_threshold, to_dev

pytestmark = pytest.mark.gpu

# N, D, K: every compiled width (48, 64, 96, 128 features), rows narrower than the width, ragged
# point blocks, a last tile with padding rows, K below one tile, and centroid sets that do not fit
# LDS at once (staged in chunks)
SHAPES = [
    (3000, 36, 70),
    (1500, 48, 31),
    (5000, 64, 129),
    (2500, 100, 300),
    (4099, 128, 256),
    (9000, 128, 64),
    (3000, 128, 700),
    (2000, 72, 1000),
    (700, 40, 5),
    (150000, 64, 40),
    (1, 128, 1),
]
MODES = [ftk.FT_CORRECT, ftk.FT_STRICT]


def _problem(N, D, K, seed=0, spread=6.0):
    return synth.random_problem(seed + N + D + K, N, D, K, "f32", spread=spread)


def _run(X, C, ft_mode=ftk.FT_OFF, faults=None):
    stats = ftk.new_stats(DEV)
    labels, mind = ftk.kmeans_assign_fast(to_dev(X), to_dev(C), ft_mode=ft_mode, faults=faults, stats=stats)
    torch.cuda.synchronize()
    return labels.cpu().numpy(), mind.cpu().numpy(), ftk.stats_dict(stats)


def _random_faults(geom, n, seed):
    rng = np.random.default_rng(seed)
    wgs = rng.choice(geom.workgroups, size=min(n, geom.workgroups), replace=False)
    return [(int(wg), int(rng.integers(geom.waves_per_workgroup)), int(rng.integers(geom.tiles_per_wave)),
             int(rng.integers(geom.regs_per_tile)), int(rng.integers(geom.lanes)), int(rng.integers(geom.bits)))
            for wg in wgs]


def test_fast_plan_for_wide_rows():
    g, det, band = ftk.fast_plan(ftk.F32, 4099, 128, 256, ftk.FT_OFF)
    assert g.waves_per_workgroup == 8 and g.workgroups == (4099 + 511) // 512
    assert g.tiles_per_wave == 2 * 8 and g.regs_per_tile == 16 and det == 0.0
    g, det, band_on = ftk.fast_plan(ftk.F32, 4099, 128, 256, ftk.FT_CORRECT)
    assert g.tiles_per_wave == 2 * 9 and det > 0.0 and band_on == band  # 30 centroids per tile
    # two bf16 pieces per operand: 2^-15 of the magnitude per score, twice for a comparison
    assert 2.0 ** -14 < band < 2.0 ** -13


@pytest.mark.parametrize("mode", [ftk.FT_OFF, ftk.FT_DETECT, ftk.FT_CORRECT, ftk.FT_STRICT])
@pytest.mark.parametrize("N,D,K", SHAPES)
def test_fast_wide_assignment_matches_oracle(N, D, K, mode):
    X, C = _problem(N, D, K)
    print("fast wide parity", N, D, K, "mode", mode, flush=True)
    labels, mind, st = _run(X, C, mode)
    check_assign(X, C, labels, mind)
    if mode != ftk.FT_OFF:
        assert st["tiles_checked"] > 0 and st["detected"] == 0, st
        assert st["max_residual_ppm"] < 500_000, st  # headroom of the threshold over rounding noise


@pytest.mark.parametrize("N,D,K,spread", [(13619, 36, 1000, 10.0), (20000, 40, 2048, 10.0), (9000, 36, 300, 0.5)])
def test_fast_wide_checksum_rows_truncation_raises_no_alarm(N, D, K, spread):
    """Narrow rows, many far-out centroids: what a checksum row loses when it is reduced to two
    pieces is largest against the threshold here (it does not shrink with D like rounding noise);
    the threshold carries its measured norm, so a clean run stays silent in every mode."""
    X, C = _problem(N, D, K, seed=17, spread=spread)
    for mode in (ftk.FT_DETECT, ftk.FT_STRICT):
        labels, mind, st = _run(X, C, mode)
        check_assign(X, C, labels, mind)
        assert st["tiles_checked"] > 0 and st["detected"] == 0 and st["max_residual_ppm"] < 600_000, st


@pytest.mark.parametrize("N,D,K", [(4099, 128, 256), (2500, 100, 300)])
def test_fast_wide_exact_ties_go_to_the_lowest_index(N, D, K):
    """Duplicated centroids score identically: both lie inside the bound and are settled exactly."""
    X, C = _problem(N, D, K, seed=3)
    C[K // 2] = C[3]          # same tile or another one, another lane group
    C[K - 1] = C[40]
    C[41] = C[40]             # neighbour in the same tile
    labels, mind, _ = _run(X, C)
    check_assign(X, C, labels, mind)
    assert not np.any(labels == K // 2) and not np.any(labels == K - 1) and not np.any(labels == 41)


def test_fast_wide_clustered_data_far_from_the_origin():
    """Large norms against small distances: most scores fall inside the (wider) bound of the
    two-piece form, so nearly every point takes the exact path or the refine kernel."""
    N, D, K = 6000, 96, 200
    X, C = _problem(N, D, K, seed=5, spread=0.5)
    X = (X + 30.0).astype(np.float32)
    C = (C + 30.0).astype(np.float32)
    for mode in (ftk.FT_OFF, ftk.FT_STRICT):
        labels, mind, _ = _run(X, C, mode)
        check_assign(X, C, labels, mind)


def test_fast_wide_dynamic_range_within_rows():
    """Features of very different magnitude in one row: the pieces are taken per element."""
    rng = np.random.default_rng(8)
    scale = np.tile(np.array([1e-3, 1.0, 1e3, 1e-2, 30.0, 1e2, 1e-1, 5.0]), 8)
    X = (rng.normal(size=(6000, 64)) * scale).astype(np.float32)
    C = X[rng.choice(6000, 200, replace=False)].copy()
    labels, mind, _ = _run(X, C)
    check_assign(X, C, labels, mind)


def test_fast_wide_agrees_with_the_fp32_path_on_the_compute_bound_workload():
    """2^18 x 128, K = 256 in the launch configuration the benchmark times: sampled rows against
    the oracle, every row against the fp32 path."""
    w = synth.WORKLOADS["c3"]
    X, _ = synth.make_points(w)
    C = X[synth.init_indices(w, w.N)].copy()
    rows = np.sort(np.random.default_rng(1).choice(w.N, 3000, replace=False))
    lab32, _ = ftk.kmeans_assign(to_dev(X), to_dev(C))
    lab32 = lab32.cpu().numpy()
    for mode in (ftk.FT_OFF, ftk.FT_STRICT):
        labels, mind, st = _run(X, C, mode)
        check_assign(X, C, labels, mind, rows=rows)
        assert int((labels != lab32).sum()) <= w.N // 100000 + 2
        if mode != ftk.FT_OFF:
            assert st["detected"] == 0 and st["max_residual_ppm"] < 500_000, st
            geom, _, _ = ftk.fast_plan(ftk.F32, w.N, w.D, w.K, mode)
            faults = ftk.make_faults(_random_faults(geom, geom.workgroups, seed=7), DEV)
            lab_f, _, st_f = _run(X, C, mode, faults)
            assert st_f["injected"] == geom.workgroups, st_f
            assert st_f["corrected"] + st_f["recomputed"] == st_f["detected"], st_f
            assert np.array_equal(lab_f, labels), "strict mode: labels must equal the fault-free run"


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("N,D,K", [(6000, 128, 256), (5000, 64, 129), (3000, 128, 700)])
def test_fast_wide_one_random_flip_per_workgroup_is_repaired(N, D, K, mode):
    X, C = _problem(N, D, K)
    geom, detect, band = ftk.fast_plan(ftk.F32, N, D, K, mode)
    rows = _random_faults(geom, geom.workgroups, seed=11)
    faults = ftk.make_faults(rows, DEV)
    print("fast wide stress", N, D, K, "mode", mode, "faults", len(rows), flush=True)
    lab_clean, md_clean, st0 = _run(X, C, mode)
    assert st0["detected"] == 0 and st0["tiles_checked"] > 0, st0
    lab, md, st = _run(X, C, mode, faults)
    assert st["injected"] == len(rows), st
    check_moved_labels_within_detection_threshold(X, C, lab, lab_clean, mode, coefs=(detect, band))
    assert st["detected"] <= st["injected"]
    assert st["corrected"] + st["recomputed"] == st["detected"], st
    assert np.allclose(md, md_clean, rtol=1e-4, atol=1e-3 * (1 + np.abs(md_clean).max()))


@pytest.mark.parametrize("reg", [0, 7, 14, 15])
@pytest.mark.parametrize("bit", [31, 30, 27, 22])
def test_fast_wide_every_register_and_bit_class_is_handled(reg, bit):
    N, D, K = 6000, 128, 256
    X, C = _problem(N, D, K)
    faults = ftk.make_faults([(0, 1, 9, reg, 37, bit), (2, 0, 13, reg, 5, bit)], DEV)
    for mode in MODES:
        _, detect, band = ftk.fast_plan(ftk.F32, N, D, K, mode)
        lab_clean, _, _ = _run(X, C, mode)
        lab, _, st = _run(X, C, mode, faults)
        assert st["injected"] == 2
        check_moved_labels_within_detection_threshold(X, C, lab, lab_clean, mode, coefs=(detect, band))
        assert st["corrected"] + st["recomputed"] == st["detected"]
        if bit >= 27:
            assert st["detected"] == 2
            if reg == 15:
                assert st["recomputed"] == 2 and st["corrected"] == 0


def test_fast_wide_flips_corrupt_labels_without_ft_and_not_with_it():
    N, D, K = 20000, 128, 256
    X, C = _problem(N, D, K)
    geom, _, _ = ftk.fast_plan(ftk.F32, N, D, K, ftk.FT_OFF)
    rng = np.random.default_rng(5)
    rows = [(wg, int(rng.integers(geom.waves_per_workgroup)), int(rng.integers(geom.tiles_per_wave)),
             int(rng.integers(15)), int(rng.integers(64)), int(rng.choice([31, 30, 29])))
            for wg in range(geom.workgroups) for _ in range(4)]
    faults = ftk.make_faults(rows, DEV)
    lab_clean, _, _ = _run(X, C, ftk.FT_OFF)
    lab_bad, _, st_off = _run(X, C, ftk.FT_OFF, faults)
    assert st_off["injected"] > 0
    assert (lab_bad != lab_clean).sum() > 0, "injection had no visible effect with FT off"
    for mode in MODES:
        _, detect, band = ftk.fast_plan(ftk.F32, N, D, K, mode)
        lab_ft_clean, _, _ = _run(X, C, mode)
        lab_ft, _, st = _run(X, C, mode, faults)
        check_moved_labels_within_detection_threshold(X, C, lab_ft, lab_ft_clean, mode, coefs=(detect, band))
        assert st["detected"] > 0.9 * st["injected"] > 0


def test_fit_on_the_fast_path_matches_the_fp32_fit_on_wide_rows():
    """Same seeded start, same iteration count on the 2^18 x 128 workload: labels and centroids
    identical to the fp32 Lloyd loop (the update is the same integer accumulation)."""
    w = synth.WORKLOADS["c3"]
    X, _ = synth.make_points(w)
    C0 = X[synth.init_indices(w, w.N)].copy()
    Xd, C0d = to_dev(X), to_dev(C0)
    ref = ftk.kmeans_fit(Xd, w.K, 4, C_init=C0d)
    out = ftk.kmeans_fit(Xd, w.K, 4, C_init=C0d, fast=True, ft_mode=ftk.FT_STRICT)
    torch.cuda.synchronize()
    assert torch.equal(out["labels"], ref["labels"])
    assert torch.equal(out["C"], ref["C"]) and torch.equal(out["counts"], ref["counts"])
    assert np.allclose(out["inertia"], ref["inertia"], rtol=1e-6)


@pytest.mark.parametrize("D", [12, 64, 128])
def test_fast_nonfinite_points_do_not_disturb_the_others(D):
    """Inputs are required to be finite; a NaN or Inf coordinate must not fault, must leave the
    labels in range and every other point's label as it was (both fast kernels)."""
    N, K = 20000, 90
    X, C = _problem(N, D, K, seed=41)
    bad_rows = np.array([5, 777, 19999])
    Xb = X.copy()
    Xb[5, 3] = np.nan
    Xb[777, 0] = np.inf
    Xb[19999, D - 1] = -np.inf
    keep = np.ones(N, dtype=bool)
    keep[bad_rows] = False
    for mode in (ftk.FT_OFF, ftk.FT_STRICT):
        lab_clean, _, _ = _run(X, C, mode)
        lab, _, _ = _run(Xb, C, mode)
        assert lab.min() >= 0 and lab.max() < K
        assert np.array_equal(lab[keep], lab_clean[keep])

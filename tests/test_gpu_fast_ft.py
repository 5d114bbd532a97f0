"""Fault tolerance on the split-bf16 fast assignment (the paper protects its tensor-core variant
with the same checksums as the fp32 one, Sections 3.1.5 and 4): clean runs raise no alarm and
equal the unprotected path, injected single-bit flips are detected and repaired, strict mode
returns the fault-free labels, and the Lloyd loop runs with it."""
import numpy as np
import pytest
import torch

from oracle import cpu as oracle
from paper_2408_01391_amd import binding as ftk, synth
from tests.gpu_util import DEV, check_assign, check_moved_labels_within_detection_threshold, to_dev

pytestmark = pytest.mark.gpu

# (name, N, D, K): every compiled width, all tiles resident / staged in chunks, ragged sizes
SHAPES = [
    ("resident, D = 8", 40000, 8, 1000),
    ("staged in chunks, D = 32", 30000, 32, 1500),
    ("ragged, D = 12", 5000, 12, 77),
    ("few centroids, D = 16", 70000, 16, 40),
    ("D = 24, last tile nearly empty", 9000, 24, 211),
    ("D = 4", 3000, 4, 95),
]
MODES = [ftk.FT_CORRECT, ftk.FT_STRICT]


def _problem(N, D, K, seed=0):
    return synth.random_problem(seed + N + D + K, N, D, K, "f32", spread=6.0)


def _run(X, C, ft_mode, faults=None):
    stats = ftk.new_stats(DEV)
    labels, mind = ftk.kmeans_assign_fast(to_dev(X), to_dev(C), ft_mode=ft_mode, faults=faults, stats=stats)
    torch.cuda.synchronize()
    return labels.cpu().numpy(), mind.cpu().numpy(), ftk.stats_dict(stats)


def _random_faults(geom, n, seed, bits=None):
    rng = np.random.default_rng(seed)
    wgs = rng.choice(geom.workgroups, size=min(n, geom.workgroups), replace=False)
    return [(int(wg), int(rng.integers(geom.waves_per_workgroup)), int(rng.integers(geom.tiles_per_wave)),
             int(rng.integers(geom.regs_per_tile)), int(rng.integers(geom.lanes)),
             int(rng.integers(geom.bits) if bits is None else rng.choice(bits))) for wg in wgs]


def test_fast_plan_reports_the_checksummed_tile_layout():
    g_off, det_off, band = ftk.fast_plan(ftk.F32, 40000, 8, 1000, ftk.FT_OFF)
    g_on, det_on, band_on = ftk.fast_plan(ftk.F32, 40000, 8, 1000, ftk.FT_CORRECT)
    assert det_off == 0.0 and det_on > 0.0 and band == band_on > 0.0
    assert g_off.tiles_per_wave == 2 * 32 and g_on.tiles_per_wave == 2 * 34  # 32 resp. 30 centroids per tile
    assert g_on.workgroups == g_off.workgroups and g_on.regs_per_tile == 16 and g_on.bits == 32
    with pytest.raises(ftk.FtkError):
        ftk.fast_plan(ftk.F32, 1000, 132, 10, ftk.FT_OFF)


@pytest.mark.parametrize("name,N,D,K", SHAPES)
def test_fast_ft_on_without_faults_matches_oracle_and_raises_no_alarm(name, N, D, K):
    X, C = _problem(N, D, K)
    print("fast ft clean", name, flush=True)
    lab_off, md_off, _ = _run(X, C, ftk.FT_OFF)
    for mode in (ftk.FT_DETECT, ftk.FT_CORRECT, ftk.FT_STRICT):
        lab_on, md_on, st = _run(X, C, mode)
        check_assign(X, C, lab_on, md_on)
        assert np.array_equal(lab_on, lab_off)
        assert st["tiles_checked"] > 0
        assert st["detected"] == 0 and st["corrected"] == 0 and st["recomputed"] == 0
        assert st["max_residual_ppm"] < 500_000, st  # headroom of the threshold over rounding noise


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("name,N,D,K", SHAPES)
def test_fast_one_random_flip_per_workgroup_is_repaired(name, N, D, K, mode):
    """The paper's stress model: every workgroup corrupts one random element by one random bit."""
    X, C = _problem(N, D, K)
    geom, detect, band = ftk.fast_plan(ftk.F32, N, D, K, mode)
    rows = _random_faults(geom, geom.workgroups, seed=11)
    faults = ftk.make_faults(rows, DEV)
    print("fast ft stress", name, "mode", mode, "faults", len(rows), flush=True)
    lab_clean, md_clean, _ = _run(X, C, mode)
    lab, md, st = _run(X, C, mode, faults)
    assert st["injected"] == len(rows), st
    check_moved_labels_within_detection_threshold(X, C, lab, lab_clean, mode, coefs=(detect, band))
    assert st["detected"] <= st["injected"]
    assert st["corrected"] + st["recomputed"] == st["detected"], st
    assert np.allclose(md, md_clean, rtol=1e-4, atol=1e-3 * (1 + np.abs(md_clean).max()))


def test_fast_high_bit_flips_corrupt_labels_without_ft_and_not_with_it():
    name, N, D, K = SHAPES[0]
    X, C = _problem(N, D, K)
    geom_off, _, _ = ftk.fast_plan(ftk.F32, N, D, K, ftk.FT_OFF)
    rng = np.random.default_rng(5)
    rows = [(wg, int(rng.integers(geom_off.waves_per_workgroup)), int(rng.integers(geom_off.tiles_per_wave)),
             int(rng.integers(15)), int(rng.integers(64)), int(rng.choice([31, 30, 29])))
            for wg in range(geom_off.workgroups) for _ in range(4)]
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
        assert (lab_ft != lab_clean).sum() <= 1e-4 * N
        assert st["detected"] > 0.9 * st["injected"] > 0


@pytest.mark.parametrize("reg", [0, 7, 14, 15])
@pytest.mark.parametrize("bit", [31, 30, 27, 23])
def test_fast_every_register_and_bit_class_is_handled(reg, bit):
    """Score registers are corrected from the decoded location; register 15 holds the carried
    checksum itself, whose corruption cannot be located and sends the point to recomputation."""
    name, N, D, K = SHAPES[0]
    X, C = _problem(N, D, K)
    faults = ftk.make_faults([(0, 1, 9, reg, 37, bit), (2, 0, 40, reg, 5, bit)], DEV)
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


def test_fast_fit_with_fault_tolerance_follows_the_oracle():
    """The whole loop on the fast path with checksums (and the DMR update): teacher-free, against
    the oracle's trajectory on a well-separated problem."""
    w = synth.WORKLOADS["c1"]
    X, _ = synth.make_points(w)
    C0 = X[synth.init_indices(w, w.N)]
    ref = oracle.fit(X, C0, 4)
    stats = ftk.new_stats(DEV)
    out = ftk.kmeans_fit(to_dev(X), w.K, 4, C_init=to_dev(C0), ft_mode=ftk.FT_STRICT, stats=stats, fast=True)
    torch.cuda.synchronize()
    assert np.array_equal(out["labels"].cpu().numpy(), ref["labels"])
    assert np.allclose(out["C"].cpu().numpy(), ref["C"], rtol=1e-4, atol=1e-5)
    st = ftk.stats_dict(stats)
    assert st["tiles_checked"] > 0 and st["detected"] == 0


@pytest.mark.parametrize("name", ["c2", "c5"])
def test_fast_ft_at_full_size_under_injection(name):
    """BASELINE-sized workloads in the launch configuration the benchmark times: the checksummed
    fast path raises no alarm on a clean run, agrees with the oracle on sampled rows and with the
    unprotected path everywhere outside near-ties, and with 512 flips injected strict mode returns
    the clean labels exactly (CORRECT: moved only within the detection threshold)."""
    w = synth.WORKLOADS[name]
    X, _ = synth.make_points(w)
    C = X[synth.init_indices(w, w.N)].copy()
    rows = np.sort(np.random.default_rng(2).choice(w.N, 3000, replace=False))
    lab_off, _, _ = _run(X, C, ftk.FT_OFF)
    for mode in MODES:
        geom, detect, band = ftk.fast_plan(ftk.F32, w.N, w.D, w.K, mode)
        print("fast ft full size", name, "mode", mode, flush=True)
        lab_clean, md_clean, st = _run(X, C, mode)
        assert st["detected"] == 0 and st["tiles_checked"] > 0 and st["max_residual_ppm"] < 500_000, st
        check_assign(X, C, lab_clean, md_clean, rows=rows)
        assert int((lab_clean != lab_off).sum()) <= w.N // 100000 + 2
        faults = ftk.make_faults(_random_faults(geom, 512, seed=7), DEV)
        lab, _, st = _run(X, C, mode, faults)
        assert st["injected"] == min(512, geom.workgroups), st
        assert st["corrected"] + st["recomputed"] == st["detected"] and st["uncorrectable"] == 0, st
        check_moved_labels_within_detection_threshold(X, C, lab, lab_clean, mode, coefs=(detect, band))

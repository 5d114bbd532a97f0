"""The mid-D assignment kernel (fp32, 32 < D <= 128: point fragments in registers, centroids
LDS-resident or staged in chunks, scores of the best tile kept) against the oracle, forced through
the tuning hook so that the shapes stay small: parity in every fault-tolerance mode, and the
injection experiments of Sections 2.1 / 5.3 on it."""
import numpy as np
import pytest
import torch

from paper_2408_01391_amd import binding as ftk, synth
from tests.gpu_util import DEV, check_assign, check_moved_labels_within_detection_threshold, gpu_assign, to_dev

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
]


@pytest.fixture(autouse=True)
def _force_register_resident_kernel():
    ftk.tuning_override(1, -1, -1)
    yield
    ftk.tuning_override(-1, -1, -1)


def _problem(N, D, K, seed=0, spread=6.0):
    return synth.random_problem(seed + N + D + K, N, D, K, "f32", spread=spread)


def _run(X, C, ft_mode, faults=None):
    Xd, Cd = to_dev(X), to_dev(C)
    stats = ftk.new_stats(DEV)
    labels, mind = ftk.kmeans_assign(Xd, Cd, ft_mode=ft_mode, faults=faults, stats=stats)
    torch.cuda.synchronize()
    return labels.cpu().numpy(), mind.cpu().numpy(), ftk.stats_dict(stats)


def test_the_hook_selects_the_mid_d_geometry():
    g = ftk.assign_geometry(ftk.F32, 4099, 128, 256, ftk.FT_OFF)
    assert g.waves_per_workgroup == 8 and g.workgroups == (4099 + 511) // 512
    assert g.tiles_per_wave == 2 * 8 and g.regs_per_tile == 16
    g = ftk.assign_geometry(ftk.F32, 4099, 128, 256, ftk.FT_CORRECT)
    assert g.tiles_per_wave == 2 * 9  # 30 centroids per tile


@pytest.mark.parametrize("mode", [ftk.FT_OFF, ftk.FT_CORRECT, ftk.FT_STRICT])
@pytest.mark.parametrize("N,D,K", SHAPES)
def test_mid_d_assignment_matches_oracle(N, D, K, mode):
    X, C = _problem(N, D, K)
    print("mid-D parity", N, D, K, "mode", mode, flush=True)
    labels, mind = gpu_assign(X, C, ft_mode=mode)
    check_assign(X, C, labels, mind)


@pytest.mark.parametrize("N,D,K", [(4099, 128, 256), (2500, 100, 300)])
def test_mid_d_exact_ties_go_to_the_lowest_index(N, D, K):
    """Duplicated centroids score identically: both lie inside the bound and are settled exactly."""
    X, C = _problem(N, D, K, seed=3)
    C[K // 2] = C[3]          # same tile or another one, another lane group
    C[K - 1] = C[40]
    C[41] = C[40]             # neighbour in the same tile
    labels, mind = gpu_assign(X, C, ft_mode=ftk.FT_OFF)
    check_assign(X, C, labels, mind)
    assert not np.any(labels == K // 2) and not np.any(labels == K - 1) and not np.any(labels == 41)


def test_mid_d_clustered_data_far_from_the_origin():
    """Large norms against small distances: many scores fall inside the rounding bound."""
    N, D, K = 6000, 96, 200
    X, C = _problem(N, D, K, seed=5, spread=0.5)
    X += 30.0
    C += 30.0
    X = X.astype(np.float32)
    C = C.astype(np.float32)
    for mode in (ftk.FT_OFF, ftk.FT_STRICT):
        labels, mind = gpu_assign(X, C, ft_mode=mode)
        check_assign(X, C, labels, mind)


def _random_faults(geom, n, seed):
    rng = np.random.default_rng(seed)
    wgs = rng.choice(geom.workgroups, size=min(n, geom.workgroups), replace=False)
    return [(int(wg), int(rng.integers(geom.waves_per_workgroup)), int(rng.integers(geom.tiles_per_wave)),
             int(rng.integers(geom.regs_per_tile)), int(rng.integers(geom.lanes)), int(rng.integers(geom.bits)))
            for wg in wgs]


@pytest.mark.parametrize("mode", [ftk.FT_CORRECT, ftk.FT_STRICT])
@pytest.mark.parametrize("N,D,K", [(6000, 128, 256), (5000, 64, 129), (3000, 128, 700)])
def test_mid_d_one_random_flip_per_workgroup_is_repaired(N, D, K, mode):
    X, C = _problem(N, D, K)
    geom = ftk.assign_geometry(ftk.F32, N, D, K, mode)
    rows = _random_faults(geom, geom.workgroups, seed=11)
    faults = ftk.make_faults(rows, DEV)
    print("mid-D stress", N, D, K, "mode", mode, "faults", len(rows), flush=True)
    lab_clean, md_clean, st0 = _run(X, C, mode)
    assert st0["detected"] == 0 and st0["tiles_checked"] > 0 and st0["max_residual_ppm"] < 500_000, st0
    check_assign(X, C, lab_clean, md_clean)
    lab, md, st = _run(X, C, mode, faults)
    assert st["injected"] == len(rows), st
    check_moved_labels_within_detection_threshold(X, C, lab, lab_clean, mode)
    assert st["detected"] <= st["injected"]
    assert st["corrected"] + st["recomputed"] == st["detected"], st
    assert np.allclose(md, md_clean, rtol=1e-4, atol=1e-3 * (1 + np.abs(md_clean).max()))


@pytest.mark.parametrize("reg", [0, 7, 14, 15])
@pytest.mark.parametrize("bit", [31, 30, 27, 22])
def test_mid_d_every_register_and_bit_class_is_handled(reg, bit):
    N, D, K = 6000, 128, 256
    X, C = _problem(N, D, K)
    faults = ftk.make_faults([(0, 1, 9, reg, 37, bit), (2, 0, 13, reg, 5, bit)], DEV)
    for mode in (ftk.FT_CORRECT, ftk.FT_STRICT):
        lab_clean, _, _ = _run(X, C, mode)
        lab, _, st = _run(X, C, mode, faults)
        assert st["injected"] == 2
        check_moved_labels_within_detection_threshold(X, C, lab, lab_clean, mode)
        assert st["corrected"] + st["recomputed"] == st["detected"]
        if bit >= 27:
            assert st["detected"] == 2
            if reg == 15:
                assert st["recomputed"] == 2 and st["corrected"] == 0


def test_mid_d_flips_corrupt_labels_without_ft_and_not_with_it():
    N, D, K = 20000, 128, 256
    X, C = _problem(N, D, K)
    geom = ftk.assign_geometry(ftk.F32, N, D, K, ftk.FT_OFF)
    rng = np.random.default_rng(5)
    rows = [(wg, int(rng.integers(geom.waves_per_workgroup)), int(rng.integers(geom.tiles_per_wave)),
             int(rng.integers(15)), int(rng.integers(64)), int(rng.choice([31, 30, 29])))
            for wg in range(geom.workgroups) for _ in range(4)]
    faults = ftk.make_faults(rows, DEV)
    lab_clean, _, _ = _run(X, C, ftk.FT_OFF)
    lab_bad, _, st_off = _run(X, C, ftk.FT_OFF, faults)
    assert st_off["injected"] > 0
    assert (lab_bad != lab_clean).sum() > 0, "injection had no visible effect with FT off"
    for mode in (ftk.FT_CORRECT, ftk.FT_STRICT):
        lab_ft_clean, _, _ = _run(X, C, mode)
        lab_ft, _, st = _run(X, C, mode, faults)
        check_moved_labels_within_detection_threshold(X, C, lab_ft, lab_ft_clean, mode)
        assert st["detected"] > 0.9 * st["injected"] > 0


@pytest.mark.parametrize("mode", [ftk.FT_OFF, ftk.FT_STRICT])
def test_mid_d_as_dispatched_by_the_built_in_rule_at_a_full_grid(mode):
    """2^17 points fill every compute unit with one workgroup: the size from which the rule picks
    this kernel.  Every row against the oracle; with checksums, one flip per workgroup on top."""
    ftk.tuning_override(-1, -1, -1)
    N, D, K = 1 << 17, 64, 520
    geom = ftk.assign_geometry(ftk.F32, N, D, K, mode)
    assert geom.waves_per_workgroup == 8 and geom.workgroups == N // 512, "the rule no longer picks the mid-D kernel"
    X, C = _problem(N, D, K, seed=21)
    lab, md, st = _run(X, C, mode)
    check_assign(X, C, lab, md)
    if mode != ftk.FT_OFF:
        assert st["detected"] == 0 and st["max_residual_ppm"] < 500_000, st
        faults = ftk.make_faults(_random_faults(geom, geom.workgroups, seed=3), DEV)
        lab_f, _, st_f = _run(X, C, mode, faults)
        assert st_f["injected"] == geom.workgroups
        assert np.array_equal(lab_f, lab), "strict mode: labels must equal the fault-free run"

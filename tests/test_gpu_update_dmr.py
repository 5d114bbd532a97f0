"""Dual modular redundancy on the update step (paper Sections 2.3 and 4: the memory-bound update is
protected by duplicating its arithmetic and comparing).

With DMR on and single-bit flips injected into the first instruction stream of the accumulating
kernel, centroids and counts must equal those of the fault-free run bit for bit; without DMR the
same flips corrupt them."""
import numpy as np
import pytest
import torch

from oracle import cpu as oracle
from paper_2408_01391_amd import binding as ftk, synth
from tests.gpu_util import DEV, check_centroids, to_dev

pytestmark = pytest.mark.gpu

# (name, N, D, K, dtype): both accumulation paths (per-workgroup LDS tables / label-sorted gather),
# both dtypes, rows that are and are not 16-byte aligned
SHAPES = [
    ("tables f32 D=8", 40000, 8, 1000, "f32"),
    ("tables f32 ragged", 5000, 12, 77, "f32"),
    ("tables f32 unaligned", 3000, 33, 50, "f32"),
    ("tables f64", 3000, 6, 40, "f64"),
    ("tables f32 sliced (K*D > one table)", 30000, 40, 300, "f32"),
    ("tables f32, long rows", 70000, 64, 100, "f32"),
    ("sorted f32 (K*D beyond four tables)", 70000, 64, 600, "f32"),
    ("sorted f32 unaligned", 70000, 33, 1000, "f32"),
    ("sorted f64", 66000, 16, 2100, "f64"),
]


def _problem(N, D, K, dtype):
    X, C = synth.random_problem(7 + N + D + K, N, D, K, dtype, spread=6.0)
    labels, _, _ = oracle.assign(X, C)
    return X, C, labels.astype(np.int32)


def _update(X, C, labels, mode, faults=None):
    Xd, Cd, Ld = to_dev(X), to_dev(C.copy()), to_dev(labels)
    stats = ftk.new_stats(DEV)
    Cn, counts = ftk.kmeans_update(Xd, Ld, Cd, ft_mode=mode, faults=faults, stats=stats)
    torch.cuda.synchronize()
    return Cn.cpu().numpy(), counts.cpu().numpy(), ftk.stats_dict(stats)


def _faults(X, N, D, K, dtype, n, seed, bits):
    code = ftk.F32 if dtype == "f32" else ftk.F64
    esz = 4 if dtype == "f32" else 8
    geom = ftk.update_geometry(code, N, D, K, (D * esz) % 16 == 0)
    rng = np.random.default_rng(seed)
    wgs = rng.choice(geom.workgroups, size=min(n, geom.workgroups), replace=False)
    # early steps only, so that the addressed lane still has rows to walk
    steps = max(1, geom.tiles_per_wave // 4)
    return [(int(g), int(rng.integers(geom.waves_per_workgroup)), int(rng.integers(steps)),
             int(rng.integers(geom.regs_per_tile)), int(rng.integers(64)), int(rng.choice(bits))) for g in wgs]


@pytest.mark.parametrize("name,N,D,K,dtype", SHAPES)
def test_dmr_on_clean_input_changes_nothing(name, N, D, K, dtype):
    X, C, labels = _problem(N, D, K, dtype)
    print("dmr clean", name, flush=True)
    C_off, n_off, _ = _update(X, C, labels, ftk.FT_OFF)
    C_on, n_on, st = _update(X, C, labels, ftk.FT_CORRECT)
    assert np.array_equal(C_on, C_off) and np.array_equal(n_on, n_off)
    assert st["detected"] == 0 and st["recomputed"] == 0 and st["uncorrectable"] == 0
    C_o, n_o = oracle.update(X, labels, C)
    assert np.array_equal(n_on, n_o)
    check_centroids(C_on, C_o)


@pytest.mark.parametrize("name,N,D,K,dtype", SHAPES)
def test_injected_flips_are_detected_and_recomputed(name, N, D, K, dtype):
    X, C, labels = _problem(N, D, K, dtype)
    rows = _faults(X, N, D, K, dtype, 24, seed=3, bits=np.arange(64))
    faults = ftk.make_faults(rows, DEV)
    print("dmr inject", name, "faults", len(rows), flush=True)
    C_clean, n_clean, _ = _update(X, C, labels, ftk.FT_CORRECT)
    C_inj, n_inj, st = _update(X, C, labels, ftk.FT_CORRECT, faults)
    assert st["injected"] >= 1, st
    assert st["detected"] == st["injected"] and st["recomputed"] == st["detected"], st
    assert st["uncorrectable"] == 0
    assert np.array_equal(C_inj, C_clean) and np.array_equal(n_inj, n_clean)


@pytest.mark.parametrize("name,N,D,K,dtype", [SHAPES[0], SHAPES[5], SHAPES[7]])
def test_high_bit_flips_corrupt_centroids_without_dmr(name, N, D, K, dtype):
    X, C, labels = _problem(N, D, K, dtype)
    faults = ftk.make_faults(_faults(X, N, D, K, dtype, 24, seed=5, bits=np.arange(50, 61)), DEV)
    C_clean, _, _ = _update(X, C, labels, ftk.FT_OFF)
    C_bad, _, st = _update(X, C, labels, ftk.FT_OFF, faults)
    assert st["injected"] >= 1 and st["detected"] == 0
    assert not np.array_equal(C_bad, C_clean), "injection had no visible effect with DMR off"
    C_dmr, _, st2 = _update(X, C, labels, ftk.FT_CORRECT, faults)
    assert np.array_equal(C_dmr, C_clean) and st2["detected"] == st2["injected"] >= 1


def test_detect_mode_only_counts():
    name, N, D, K, dtype = SHAPES[5]
    X, C, labels = _problem(N, D, K, dtype)
    faults = ftk.make_faults(_faults(X, N, D, K, dtype, 8, seed=9, bits=np.arange(50, 61)), DEV)
    _, _, st = _update(X, C, labels, ftk.FT_DETECT, faults)
    assert st["injected"] >= 1 and st["detected"] == st["injected"]
    assert st["recomputed"] == 0 and st["corrected"] == 0


def test_fit_with_ft_runs_the_update_under_dmr_and_matches_plain_fit():
    w = synth.WORKLOADS["c1"]
    X, _ = synth.make_points(w)
    C0 = X[synth.init_indices(w, w.N)]
    Xd = to_dev(X)
    plain = ftk.kmeans_fit(Xd, w.K, 5, C_init=to_dev(C0), ft_mode=ftk.FT_OFF)
    prot = ftk.kmeans_fit(Xd, w.K, 5, C_init=to_dev(C0), ft_mode=ftk.FT_CORRECT)
    assert torch.equal(plain["C"], prot["C"]) and torch.equal(plain["labels"], prot["labels"])

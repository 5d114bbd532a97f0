"""GPU parity: the HIP path, called through the C-ABI binding, against the CPU oracle on the same
seeded inputs.  Labels must be identical except inside the tie band (1e-5 relative for fp32,
1e-12 for fp64, relative to the best distance); centroids within 1e-4 / 1e-10 relative."""
import numpy as np
import pytest
import torch

from oracle import cpu as oracle
from paper_2408_01391_amd import binding as ftk, synth
from tests.gpu_util import (DEV, check_assign, check_centroids, gpu_assign, gpu_update, to_dev)

pytestmark = pytest.mark.gpu

SHAPES = [
    (1, 1, 1), (5, 3, 2), (64, 4, 64), (100, 7, 5), (300, 8, 33), (1000, 16, 8), (257, 2, 600),
    (777, 33, 130), (2048, 128, 256), (513, 200, 70), (100, 1, 300), (1500, 64, 129), (640, 24, 1025),
    (3000, 8, 3000), (1111, 32, 900), (450000, 8, 40), (2500, 12, 77), (9000, 20, 2049),
    # few centroids, many features: the one- and two-tile blockings of the generic kernel
    (4000, 72, 40), (3000, 40, 20), (2000, 100, 64), (70000, 256, 12),
    # long rows with several chunks of centroids (fp64: eight centroid tiles of one point tile)
    (1500, 512, 130), (700, 640, 300),
]


@pytest.mark.parametrize("dtype", ["f32", "f64"])
@pytest.mark.parametrize("N,D,K", SHAPES)
def test_assign_matches_oracle_on_ragged_shapes(dtype, N, D, K):
    X, C = synth.random_problem(N * 7 + D * 3 + K, N, D, K, dtype)
    print("assign", dtype, N, D, K, flush=True)
    labels, mind = gpu_assign(X, C)
    check_assign(X, C, labels, mind)


@pytest.mark.parametrize("dtype", ["f32", "f64"])
def test_assign_exact_on_integers_with_duplicate_centroids(dtype):
    X, C = synth.random_problem(5, 3000, 12, 40, dtype, integer=True)
    C[17] = C[3]
    C[39] = C[3]
    C[8] = C[30]
    labels, mind = gpu_assign(X, C)
    lab_o, d1, _ = oracle.assign(X, C)
    assert np.array_equal(labels, lab_o)          # every tie to the lowest index
    assert not np.isin(labels, [17, 39, 30]).any()
    assert np.allclose(mind, d1, rtol=1e-6, atol=1e-3)


def test_assign_offset_data_needs_the_exact_tie_break():
    """Large common offset: ||x||^2 is ~1e8 while cluster gaps are ~1; the expanded form alone
    cannot order the two nearest centroids in fp32."""
    rng = np.random.default_rng(3)
    X = (rng.normal(size=(4000, 8)) + 3000.0).astype(np.float32)
    C = X[rng.choice(4000, 50, replace=False)].copy()
    labels, mind = gpu_assign(X, C)
    check_assign(X, C, labels)


@pytest.mark.parametrize("dtype", ["f32", "f64"])
@pytest.mark.parametrize("N,D,K", [(1, 1, 1), (1000, 8, 16), (5000, 128, 256), (3001, 17, 700),
                                   (4096, 512, 64), (20000, 32, 4096), (999, 3, 5),
                                   # N >= 65536 with rows of a cache line or more: LDS tables while K*D
                                   # fits four of them, the label-sorted path beyond
                                   (70000, 64, 100), (70000, 64, 600), (66000, 40, 900)])
def test_update_matches_oracle(dtype, N, D, K):
    X, C = synth.random_problem(N + D + K, N, D, K, dtype)
    rng = np.random.default_rng(N)
    labels = rng.integers(0, max(1, K - 1), size=N).astype(np.int32)   # last cluster stays empty
    print("update", dtype, N, D, K, flush=True)
    C_g, counts_g = gpu_update(X, labels, C)
    C_o, counts_o = oracle.update(X, labels, C)
    assert np.array_equal(counts_g, counts_o)
    check_centroids(C_g, C_o)
    if K > 1:
        assert np.array_equal(C_g[K - 1], C[K - 1])       # empty cluster keeps its centroid


@pytest.mark.parametrize("dtype", ["f32", "f64"])
def test_update_with_feature_scales_spanning_six_orders_of_magnitude(dtype):
    """One fixed-point scale serves all features: a feature far below the largest |x| keeps
    fewer bits.  The documented bound - half a quantum of max|x| 2^-(61 - ceil(log2 N)) (fp32) or
    max|x| 2^-50 (fp64) plus the final rounding - must hold for every coordinate, and the
    centroid tolerance of the workloads with it."""
    N, D, K = 200000, 16, 37
    X, C = synth.random_problem(99, N, D, K, dtype)
    scales = np.logspace(-3, 3, D).astype(X.dtype)
    X = np.ascontiguousarray(X * scales)
    C = np.ascontiguousarray(C * scales)
    labels = np.random.default_rng(4).integers(0, K, size=N).astype(np.int32)
    C_g, counts_g = gpu_update(X, labels, C)
    C_o, counts_o = oracle.update(X, labels, C)
    assert np.array_equal(counts_g, counts_o)
    check_centroids(C_g, C_o)
    absmax = np.abs(X).max()
    q = absmax * (2.0 ** -(61 - 18) if dtype == "f32" else 2.0 ** -50)
    u = 2.0 ** -24 if dtype == "f32" else 2.0 ** -53
    err = np.abs(C_g.astype(np.float64) - C_o.astype(np.float64))
    assert np.all(err <= 0.5 * q + 2 * u * np.abs(C_o)), (err / (0.5 * q + 2 * u * np.abs(C_o))).max()
    # per-feature relative accuracy actually reached (smallest features are 10^6 below the largest)
    rel = np.median(err / np.maximum(np.abs(C_o), np.finfo(np.float64).tiny), axis=0)
    print("update, feature scales 1e-3..1e3,", dtype, "median relative error per feature:", rel)


@pytest.mark.parametrize("dtype", ["f32", "f64"])
def test_nonfinite_points_only_spoil_their_own_cluster(dtype):
    """Inputs are required to be finite; a NaN or Inf coordinate must not fault, must leave the
    labels in range, and must not disturb points and clusters it does not belong to."""
    N, D, K = 20000, 12, 30
    X, C = synth.random_problem(123, N, D, K, dtype)
    bad_rows = np.array([5, 777, 19999])
    Xb = X.copy()
    Xb[5, 3] = np.nan
    Xb[777, 0] = np.inf
    Xb[19999, 11] = -np.inf
    for mode in (ftk.FT_OFF, ftk.FT_STRICT):
        lab_clean, _ = gpu_assign(X, C, ft_mode=mode)
        lab, _ = gpu_assign(Xb, C, ft_mode=mode)
        assert lab.min() >= 0 and lab.max() < K
        keep = np.ones(N, dtype=bool)
        keep[bad_rows] = False
        assert np.array_equal(lab[keep], lab_clean[keep])
    assert float(ftk.absmax(to_dev(Xb)).cpu()[0]) == np.abs(Xb[np.isfinite(Xb)]).max()
    labels = lab_clean.astype(np.int32)
    C_g, counts_g = gpu_update(Xb, labels, C)
    C_o, _ = oracle.update(X, labels, C)
    spoiled = np.unique(labels[bad_rows])
    fine = np.setdiff1d(np.arange(K), spoiled)
    check_centroids(C_g[fine], C_o[fine])
    assert np.array_equal(counts_g, np.bincount(labels, minlength=K))


def test_update_is_bitwise_reproducible():
    X, C = synth.random_problem(77, 50000, 24, 300, "f32")
    labels = np.random.default_rng(0).integers(0, 300, size=50000).astype(np.int32)
    a, _ = gpu_update(X, labels, C)
    for _ in range(3):
        b, _ = gpu_update(X, labels, C)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_absmax():
    x = np.random.default_rng(1).normal(size=100003).astype(np.float32)
    x[4711] = -77.5
    assert float(ftk.absmax(to_dev(x.reshape(1, -1))).cpu()[0]) == 77.5


@pytest.mark.parametrize("name,N,iters", [("c1", 4096, 10), ("c2", 1 << 15, 6), ("c3", 1 << 13, 5),
                                          ("c4", 1 << 12, 4), ("c5", 1 << 14, 4)])
def test_teacher_forced_lloyd_iterations(name, N, iters):
    """Per iteration: assign against the oracle's previous centroids, update from the oracle's
    labels (a free-running comparison would amplify a single tie flip)."""
    w = synth.WORKLOADS[name]
    K = min(w.K, N // 4)
    X, _ = synth.make_points(w, N)
    C0 = X[synth.init_indices(w, N, K)].copy()
    ref = oracle.fit(X, C0, iters, history=True)
    Xd = to_dev(X)
    C_prev = C0
    in_band = 0
    for t in range(iters):
        print("teacher", name, "iter", t, flush=True)
        labels, mind = ftk.kmeans_assign(Xd, to_dev(C_prev))
        torch.cuda.synchronize()
        nb, _ = check_assign(X, C_prev, labels.cpu().numpy(), mind.cpu().numpy())
        in_band += nb
        C_g, counts_g = gpu_update(X, ref["labels_hist"][t], C_prev)
        check_centroids(C_g, ref["C_hist"][t])
        C_prev = ref["C_hist"][t]
    print(name, "labels inside the tie band:", in_band)


def test_fit_free_running_matches_oracle_on_c1():
    w = synth.WORKLOADS["c1"]
    X, _ = synth.make_points(w)
    C0 = X[synth.init_indices(w, w.N)].copy()
    ref = oracle.fit(X, C0, w.iters)
    out = ftk.kmeans_fit(to_dev(X), w.K, w.iters, C_init=to_dev(C0))
    assert np.array_equal(out["labels"].cpu().numpy(), ref["labels"])
    assert np.array_equal(out["counts"].cpu().numpy(), ref["counts"])
    check_centroids(out["C"].cpu().numpy(), ref["C"])
    assert np.allclose(out["inertia"], ref["inertia"], rtol=1e-4)
    assert np.all(np.diff(out["inertia"]) <= 1e-6 * out["inertia"][:-1])


def test_fit_seeded_init_uses_the_documented_index_choice():
    X, _ = synth.random_problem(9, 5000, 6, 10, "f64")
    idx_o = oracle.seeded_indices(2024, 5000, 10)
    assert np.array_equal(ftk.seeded_indices(2024, 5000, 10), idx_o)
    ref = oracle.fit(X, X[idx_o].copy(), 5)
    out = ftk.kmeans_fit(to_dev(X), 10, 5, seed=2024)
    assert np.array_equal(out["labels"].cpu().numpy(), ref["labels"])
    check_centroids(out["C"].cpu().numpy(), ref["C"])


def test_error_paths_return_codes_without_touching_the_gpu_state():
    X = torch.zeros(16, 4, device=DEV)
    C = torch.zeros(2, 4, device=DEV)
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(ftk.FtkError) as e:
        ftk.kmeans_assign(X, C, workspace=small)
    assert e.value.code == 3
    with pytest.raises(ftk.FtkError) as e:
        ftk.kmeans_fit(X, 32, 1, seed=1)            # K > N with seeded init
    assert e.value.code == 1
    with pytest.raises(ValueError):
        ftk.kmeans_assign(X, torch.zeros(2, 5, device=DEV))
    labels, _ = ftk.kmeans_assign(X, C)             # still usable afterwards
    torch.cuda.synchronize()
    assert labels.cpu().tolist() == [0] * 16


@pytest.mark.parametrize("N,D,K", [(600_000, 8, 64), (300_000, 64, 64)])
def test_every_point_ambiguous_overflows_the_workgroup_lists_and_is_still_exact(N, D, K):
    """Centroids that differ by a few units in the last place: every score lies inside the rounding
    bound of every other, so every point needs the exact recomputation.  The register-resident
    kernels collect such points in a list of 512 entries per workgroup before handing them over;
    a workgroup here sees more than a thousand of them, so most go to the device-wide list
    directly.  Labels as the oracle's, and the same with checksums on (other tile layout, for the
    wider rows another kernel)."""
    rng = np.random.default_rng(N + D)
    X = rng.normal(size=(N, D)).astype(np.float32)
    base = rng.normal(size=(1, D)).astype(np.float32)
    C = (base * (1.0 + 2.0e-7 * rng.integers(-3, 4, size=(K, D)))).astype(np.float32)
    C[K - 1] = C[5]  # and an exact duplicate: lowest index wins
    stats = ftk.new_stats(torch.device("cuda:0"))
    labels, mind = gpu_assign(X, C, stats=stats)
    st = ftk.stats_dict(stats)
    assert st["refined"] > 0.9 * N, st
    check_assign(X, C, labels, mind)
    assert not np.any(labels == K - 1)
    labels_ft, mind_ft = gpu_assign(X, C, ft_mode=ftk.FT_CORRECT)
    assert np.array_equal(labels, labels_ft)
    assert np.array_equal(mind, mind_ft)

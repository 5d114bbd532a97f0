"""Every kernel choice the tuning hook can force computes the same results: assignment and update
parity against the oracle under each override (these are the candidates the shape sweep times)."""
import numpy as np
import pytest
import torch

from oracle import cpu as oracle
from paper_2408_01391_amd import binding as ftk, synth
from tests.gpu_util import check_assign, check_centroids, gpu_assign, gpu_update

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _restore_rules():
    yield
    ftk.tuning_override(-1, -1, -1)


@pytest.mark.parametrize("dtype", ["f32", "f64"])
@pytest.mark.parametrize("variant,tiles", [(0, 1), (0, 2), (0, 4), (0, 8), (1, -1)])
@pytest.mark.parametrize("N,D,K", [(3000, 8, 70), (2500, 32, 300), (1500, 64, 129), (70000, 16, 20)])
def test_assign_parity_under_every_forced_kernel(dtype, variant, tiles, N, D, K):
    X, C = synth.random_problem(N + 3 * D + K, N, D, K, dtype)
    ftk.tuning_override(variant, tiles, -1)
    print("forced assign", dtype, variant, tiles, N, D, K, flush=True)
    for mode in (ftk.FT_OFF, ftk.FT_CORRECT):
        labels, mind = gpu_assign(X, C, ft_mode=mode)
        check_assign(X, C, labels, mind)


@pytest.mark.parametrize("dtype", ["f32", "f64"])
@pytest.mark.parametrize("path", [0, 1])
@pytest.mark.parametrize("N,D,K", [(3000, 8, 70), (70000, 64, 100), (66000, 40, 900), (5000, 128, 256), (999, 4, 5)])
def test_update_parity_under_both_forced_paths(dtype, path, N, D, K):
    X, C = synth.random_problem(N + D + K, N, D, K, dtype)
    labels = np.random.default_rng(N).integers(0, K, size=N).astype(np.int32)
    labels[labels == 3] = 0  # leaves cluster 3 empty when K > 3
    ftk.tuning_override(-1, -1, path)
    print("forced update", dtype, path, N, D, K, flush=True)
    C_g, counts = gpu_update(X, labels, C)
    C_o, n_o = oracle.update(X, labels, C)
    assert np.array_equal(counts, n_o)
    check_centroids(C_g, C_o)
    # and under dual modular redundancy the result is bit-identical
    Cd = torch.from_numpy(C.copy()).cuda()
    ftk.kmeans_update(torch.from_numpy(X).cuda(), torch.from_numpy(labels).cuda(), Cd, ft_mode=ftk.FT_CORRECT)
    assert np.array_equal(Cd.cpu().numpy(), C_g)


def test_tuning_override_rejects_unknown_values():
    with pytest.raises(ftk.FtkError):
        ftk.tuning_override(2, -1, -1)
    with pytest.raises(ftk.FtkError):
        ftk.tuning_override(-1, 3, -1)
    with pytest.raises(ftk.FtkError):
        ftk.tuning_override(-1, -1, 5)

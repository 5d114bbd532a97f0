"""The batched Lloyd step (assign a batch of rows, add it to the running sums while it is
cache-resident; paper Section 2.2, single-pass processing) against the two-call step and the
oracle: labels, distances and counts identical to ftk_kmeans_assign / ftk_kmeans_update on the
same inputs, centroids within the update's tolerance of the oracle's."""
import numpy as np
import pytest
import torch

from oracle import cpu as oracle
from paper_2408_01391_amd import binding as ftk, synth
from tests.gpu_util import DEV, check_assign, check_centroids, to_dev

pytestmark = pytest.mark.gpu

# (N, D, K, dtype, batch_rows): uneven last batch, a single batch, many batches, every kernel family
CASES = [
    (50000, 8, 300, "f32", 16384),
    (50000, 8, 300, "f32", 50000),
    (20000, 32, 1500, "f32", 7000),
    (30000, 128, 256, "f32", 8192),
    (9000, 33, 130, "f32", 1000),
    (12000, 512, 64, "f64", 4096),
    (5000, 64, 100, "f64", 777),
]


@pytest.mark.parametrize("N,D,K,dtype,batch", CASES)
def test_batched_step_matches_two_call_step_and_oracle(N, D, K, dtype, batch):
    X, C = synth.random_problem(N + D + K + batch, N, D, K, dtype, spread=5.0)
    print("batched step", N, D, K, dtype, batch, flush=True)
    Xd = to_dev(X)
    lab_ref, md_ref = ftk.kmeans_assign(Xd, to_dev(C))
    C_ref = to_dev(C).clone()
    _, counts_ref = ftk.kmeans_update(Xd, lab_ref, C_ref)
    C_b = to_dev(C).clone()
    labels, mind, counts = ftk.kmeans_step_batched(Xd, C_b, batch)
    torch.cuda.synchronize()
    assert torch.equal(labels, lab_ref)
    assert torch.equal(mind, md_ref)
    assert torch.equal(counts, counts_ref)
    lab = labels.cpu().numpy()
    check_assign(X, C, lab, mind.cpu().numpy())
    C_o, counts_o = oracle.update(X, lab, C)
    assert np.array_equal(counts.cpu().numpy(), counts_o)
    check_centroids(C_b.cpu().numpy(), C_o)
    check_centroids(C_b.cpu().numpy(), C_ref.cpu().numpy())


def test_batched_step_keeps_empty_clusters_and_rejects_bad_batch_sizes():
    X, C = synth.random_problem(3, 4000, 16, 20, "f32")
    C[7] = 1e6          # nobody is nearest to it
    Xd, Cd = to_dev(X), to_dev(C)
    _, _, counts = ftk.kmeans_step_batched(Xd, Cd, 1500)
    torch.cuda.synchronize()
    assert int(counts[7]) == 0 and np.array_equal(Cd[7].cpu().numpy(), C[7])
    with pytest.raises(ftk.FtkError):
        ftk.kmeans_step_batched(Xd, Cd, 0)
    with pytest.raises(ftk.FtkError):
        ftk.kmeans_step_batched(to_dev(np.zeros((10000, 4), np.float32)), to_dev(np.zeros((2, 4), np.float32)), 2)


def test_batched_step_whose_last_batch_is_planned_for_another_kernel():
    """A first batch of 2^17 rows and more goes to the mid-D kernel, the shorter last batch to the
    generic one, whose padded norm vector differs: the norms are then written again for it."""
    N, D, K, batch = 200_000, 64, 300, 140_000
    first = ftk.assign_geometry(ftk.F32, batch, D, K, ftk.FT_OFF)
    last = ftk.assign_geometry(ftk.F32, N - batch, D, K, ftk.FT_OFF)
    assert first.waves_per_workgroup != last.waves_per_workgroup, "the two batches no longer plan different kernels"
    X, C = synth.random_problem(17, N, D, K, "f32", spread=5.0)
    Xd, C_b = to_dev(X), to_dev(C).clone()
    labels, mind, counts = ftk.kmeans_step_batched(Xd, C_b, batch)
    torch.cuda.synchronize()
    lab = labels.cpu().numpy()
    check_assign(X, C, lab, mind.cpu().numpy())
    C_o, counts_o = oracle.update(X, lab, C)
    assert np.array_equal(counts.cpu().numpy(), counts_o)
    check_centroids(C_b.cpu().numpy(), C_o)

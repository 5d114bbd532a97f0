"""The entry point that allocates nothing (ftk_kmeans_assign_static) against ftk_kmeans_assign.

Both run the same kernels, one on the library's static device scratch, the other on a caller
workspace, so labels and distances must be identical bit for bit - on two calls in a row, the
second on a smaller problem (the static buffer then still holds the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2408_01391_amd import binding as ftk, synth
from tests.gpu_util import DEV, check_assign, to_dev

pytestmark = pytest.mark.gpu

# (N, D, K, dtype, ft): first a large problem, then a smaller one of another shape and kernel
SEQUENCES = [
    [(150000, 8, 1000, "f32", ftk.FT_OFF), (7001, 8, 77, "f32", ftk.FT_OFF)],
    [(60000, 32, 1500, "f32", ftk.FT_STRICT), (5000, 12, 77, "f32", ftk.FT_STRICT)],
    [(20000, 128, 256, "f32", ftk.FT_CORRECT), (3000, 33, 130, "f32", ftk.FT_CORRECT)],
    [(6000, 512, 64, "f64", ftk.FT_CORRECT), (1500, 64, 100, "f64", ftk.FT_OFF)],
]


@pytest.mark.parametrize("seq", SEQUENCES, ids=lambda s: "%dx%d_K%d_%s" % s[0][:4])
def test_static_entry_point_matches_workspace_entry_point(seq):
    before = torch.cuda.memory_allocated()
    for N, D, K, dtype, ft in seq:
        print("no-alloc case", N, D, K, dtype, "ft", ft, flush=True)
        X, C = synth.random_problem(7 + N + D + K, N, D, K, dtype, spread=6.0)
        Xd, Cd = to_dev(X), to_dev(C)
        lab_ref, md_ref = ftk.kmeans_assign(Xd, Cd, ft_mode=ft)
        labels = torch.full((N,), -1, dtype=torch.int32, device=DEV)
        mind = torch.full((N,), -1.0, dtype=Xd.dtype, device=DEV)
        stats = ftk.new_stats(DEV)
        torch.cuda.synchronize()
        held = torch.cuda.memory_allocated()
        ftk.kmeans_assign_static(Xd, Cd, labels, mind, ft_mode=ft, stats=stats)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == held   # the binding allocated no tensor either
        assert torch.equal(labels, lab_ref)
        assert torch.equal(mind, md_ref)
        check_assign(X, C, labels.cpu().numpy(), mind.cpu().numpy())
        if ft != ftk.FT_OFF:
            st = ftk.stats_dict(stats)
            assert st["tiles_checked"] > 0 and st["detected"] == 0
        del Xd, Cd, labels, mind, lab_ref, md_ref
    assert torch.cuda.memory_allocated() <= before + (1 << 20)


def test_static_entry_point_repairs_injected_faults():
    N, D, K = 40000, 8, 1000
    X, C = synth.random_problem(3, N, D, K, "f32", spread=6.0)
    Xd, Cd = to_dev(X), to_dev(C)
    geom = ftk.assign_geometry(ftk.F32, N, D, K, ftk.FT_STRICT)
    faults = ftk.make_faults([(0, 1, 9, 3, 37, 30), (2, 0, 40, 15, 5, 29)], DEV)
    clean, _ = ftk.kmeans_assign(Xd, Cd, ft_mode=ftk.FT_STRICT)
    labels = torch.empty(N, dtype=torch.int32, device=DEV)
    stats = ftk.new_stats(DEV)
    ftk.kmeans_assign_static(Xd, Cd, labels, None, ft_mode=ftk.FT_STRICT, faults=faults, stats=stats)
    torch.cuda.synchronize()
    st = ftk.stats_dict(stats)
    assert geom.workgroups > 2 and st["injected"] == 2 and st["detected"] == 2
    assert torch.equal(labels, clean)


def test_static_entry_point_rejects_what_does_not_fit():
    cap = ftk.static_scratch_bytes()
    assert cap == 16 << 20
    N = cap // 4 + 1024           # the refine work-list alone (4 bytes per point) exceeds the array
    Xd = torch.zeros(N, 4, dtype=torch.float32, device=DEV)
    Cd = torch.zeros(3, 4, dtype=torch.float32, device=DEV)
    labels = torch.full((N,), -7, dtype=torch.int32, device=DEV)
    with pytest.raises(ftk.FtkError) as e:
        ftk.kmeans_assign_static(Xd, Cd, labels)
    assert e.value.code == 3 and "static buffer" in str(e.value)
    torch.cuda.synchronize()
    assert int(labels.min()) == -7 and int(labels.max()) == -7   # nothing was enqueued

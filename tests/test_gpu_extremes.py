"""Extreme shapes through the C-ABI: very many points, very many centroids, very long and very
short rows.  The oracle checks a seeded sample of rows for the assignment (its cost is
rows x K x D) and the whole update."""
import numpy as np
import pytest
import torch

from oracle import cpu as oracle
from paper_2408_01391_amd import binding as ftk
from tests.gpu_util import DEV, check_assign, check_centroids, to_dev

pytestmark = pytest.mark.gpu

CASES = [
    (1 << 24, 4, 50, "f32"),        # 16.8 M points
    (500000, 8, 100000, "f32"),     # 100 k centroids, streamed through LDS in chunks
    (100000, 2048, 300, "f32"),     # long rows, generic kernel, three K-chunks
    (50000, 4096, 64, "f64"),
    (300000, 1, 7, "f64"),          # one feature
    (70000, 3, 65537, "f32"),       # more centroids than points per workgroup sweep, odd D
    (60000, 1024, 1024, "f32"),     # whole stages and chunks: the generic kernel's condition-free loop, 4 MB of C
    (200000, 128, 8192, "f32"),     # the same with 64 K-chunks
    (300000, 100, 5000, "f32"),     # mid-D kernel: ragged width, centroids staged in 19 chunks
]


@pytest.mark.parametrize("N,D,K,dtype", CASES)
def test_extreme_shape_matches_oracle(N, D, K, dtype):
    rng = np.random.default_rng(N % 1000 + D + K)
    X = (rng.normal(size=(N, D)) * 3).astype(np.float32 if dtype == "f32" else np.float64)
    C = X[rng.choice(N, K, replace=False)].copy()
    rows = rng.choice(N, 1024, replace=False)
    print("extreme", N, D, K, dtype, flush=True)
    Xd, Cd = to_dev(X), to_dev(C)
    labels = None
    for mode in (ftk.FT_OFF, ftk.FT_STRICT):
        stats = ftk.new_stats(DEV)
        lab, md = ftk.kmeans_assign(Xd, Cd, ft_mode=mode, stats=stats)
        torch.cuda.synchronize()
        labels = lab.cpu().numpy()
        check_assign(X, C, labels, md.cpu().numpy(), rows=rows)
        st = ftk.stats_dict(stats)
        assert st["detected"] == 0 and st["uncorrectable"] == 0, st
    Cn, counts = ftk.kmeans_update(Xd, lab, Cd.clone(), ft_mode=ftk.FT_CORRECT)
    torch.cuda.synchronize()
    C_o, n_o = oracle.update(X, labels, C)
    assert np.array_equal(counts.cpu().numpy(), n_o)
    check_centroids(Cn.cpu().numpy(), C_o)

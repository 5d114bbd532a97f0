"""Seeded synthetic inputs for the K-means hot path.

This module holds no K-means arithmetic.  It only draws the point clouds and
initial-centroid index sets that both the CPU oracle and the HIP path are fed,
so that the two sides never exchange computed values.

The paper names no dataset: its evaluation (Section 5) sweeps problem shapes
with unspecified values.  The five workloads below stand in for those sweeps;
each is fully determined by its name, an optional point count override and a
seed (numpy ``Generator(PCG64(seed))``; values are drawn in float64 and cast
once to the working dtype).

Blob membership is scattered through memory (the blob id of every point is a
seeded permutation of a balanced id list) so that neither the assignment nor
the update step sees points of one cluster stored contiguously.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    D: int
    K: int
    dtype: str          # "f32" | "f64"
    iters: int
    seed: int
    kind: str           # "blobs_uniform" | "blobs_normal" | "blobs_noise" | "uniform"
    centre_scale: float  # half-width of the uniform box / std of the normal draw
    std: float           # blob standard deviation
    noise_frac: float = 0.0
    noise_half_width: float = 0.0
    ft: bool = False
    flips_per_s: float = 0.0


WORKLOADS = {
    # small, well separated, launch-latency bound
    "c1": Workload("c1", 4096, 16, 8, "f32", 10, 1001, "blobs_uniform", 10.0, 1.0),
    # tiny D, large K
    "c2": Workload("c2", 1 << 20, 8, 1024, "f32", 20, 1002, "blobs_uniform", 100.0, 1.0, ft=True),
    # compute-bound fp32 contraction
    "c3": Workload("c3", 1 << 18, 128, 256, "f32", 20, 1003, "blobs_normal", 5.0, 1.0,
                   ft=True, flips_per_s=50.0),
    # fp64, large D, small K, 5% uniform noise points
    "c4": Workload("c4", 1 << 20, 512, 64, "f64", 10, 1004, "blobs_noise", 5.0, 0.5,
                   noise_frac=0.05, noise_half_width=10.0, ft=True),
    # no cluster structure: dense near-ties
    "c5": Workload("c5", 1 << 21, 32, 4096, "f32", 10, 1005, "uniform", 1.0, 0.0,
                   ft=True, flips_per_s=20.0),
}


def np_dtype(dtype: str):
    return np.float32 if dtype == "f32" else np.float64


def make_points(w: Workload, N: int | None = None, chunk_rows: int = 1 << 16):
    """Draw the point matrix X [N, D] (row-major, C-contiguous) of workload ``w``.

    Returns (X, blob_id) where blob_id[i] is the generating blob of point i
    (-1 for uniform-noise points, all -1 for the structureless workload).
    ``N`` overrides the point count (parity tests use reduced sizes); blob sizes
    stay balanced to within one point.
    """
    N = int(w.N if N is None else N)
    rng = np.random.default_rng(np.random.PCG64(w.seed))
    dt = np_dtype(w.dtype)
    X = np.empty((N, w.D), dtype=dt)
    if w.kind == "uniform":
        for r0 in range(0, N, chunk_rows):
            r1 = min(N, r0 + chunk_rows)
            X[r0:r1] = rng.random((r1 - r0, w.D))
        return X, np.full(N, -1, dtype=np.int32)

    if w.kind == "blobs_normal":
        centres = rng.normal(0.0, w.centre_scale, size=(w.K, w.D))
    else:
        centres = rng.uniform(-w.centre_scale, w.centre_scale, size=(w.K, w.D))
    n_noise = int(round(w.noise_frac * N))
    n_blob = N - n_noise
    ids = np.concatenate([
        np.arange(n_blob, dtype=np.int64) % w.K,
        np.full(n_noise, -1, dtype=np.int64),
    ])
    rng.shuffle(ids)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        cid = ids[r0:r1]
        block = rng.normal(0.0, w.std, size=(r1 - r0, w.D))
        blob = cid >= 0
        block[blob] += centres[cid[blob]]
        n_here = int((~blob).sum())
        if n_here:
            block[~blob] = rng.uniform(-w.noise_half_width, w.noise_half_width,
                                       size=(n_here, w.D))
        X[r0:r1] = block
    return X, ids.astype(np.int32)


def init_indices(w: Workload, N: int, K: int | None = None) -> np.ndarray:
    """K distinct seeded point indices used as the initial centroids."""
    K = int(w.K if K is None else K)
    rng = np.random.default_rng(np.random.PCG64(w.seed + 7919))
    return np.sort(rng.choice(N, size=K, replace=False)).astype(np.int64)


def random_problem(seed: int, N: int, D: int, K: int, dtype: str = "f32",
                   spread: float = 4.0, integer: bool = False):
    """A small generic problem for shape fuzzing: K loose blobs, or small integers.

    With ``integer=True`` every coordinate is an integer in [-8, 8], which makes
    every sum in the distance expansion and in the checksums exactly
    representable (all partial sums stay far below 2^24).
    """
    rng = np.random.default_rng(np.random.PCG64(seed))
    dt = np_dtype(dtype)
    if integer:
        X = rng.integers(-8, 9, size=(N, D)).astype(dt)
        C = rng.integers(-8, 9, size=(K, D)).astype(dt)
        return X, C
    centres = rng.normal(0.0, spread, size=(K, D))
    ids = rng.integers(0, K, size=N)
    X = (centres[ids] + rng.normal(0.0, 1.0, size=(N, D))).astype(dt)
    pick = rng.choice(N, size=K, replace=(K > N))
    C = X[pick].copy()
    return X, C

"""Helpers shared by the GPU parity tests: run the HIP path through the C-ABI binding and
compare with the CPU oracle under the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

from oracle import cpu as oracle
from paper_2408_01391_amd import binding as ftk

DEV = torch.device("cuda:0")

# labels may differ from the oracle only where the oracle's best and the GPU's choice differ by
# at most this much relative to the best distance
LABEL_RTOL = {np.dtype(np.float32): 1e-5, np.dtype(np.float64): 1e-12}
# centroids: relative to max(|c|, 1e-3 * ||C_j||_inf)
CENTROID_RTOL = {np.dtype(np.float32): 1e-4, np.dtype(np.float64): 1e-10}


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def exact_dist_to(X, C, rows, labels):
    """float64 direct-form squared distance of X[rows] to C[labels] (numpy, test side)."""
    diff = X[rows].astype(np.float64) - C[labels].astype(np.float64)
    return (diff * diff).sum(1)


def check_assign(X: np.ndarray, C: np.ndarray, labels_g: np.ndarray, mindist_g=None, rows=None, ref=None):
    """Compare GPU labels (for all points, or for the listed rows) with the oracle.

    ``ref`` = (labels, best, second) of an earlier oracle.assign over the same rows, to compare
    several GPU runs against one oracle pass.
    Returns (number of label differences inside the tie band, number of points checked).
    Raises AssertionError on any difference outside the band.
    """
    lab_o, d1, d2 = oracle.assign(X, C, rows) if ref is None else ref
    idx = np.arange(X.shape[0]) if rows is None else np.asarray(rows)
    lab_g = labels_g[idx]
    assert lab_g.min() >= 0 and lab_g.max() < C.shape[0], "label out of range"
    diff = np.flatnonzero(lab_g != lab_o)
    rtol = LABEL_RTOL[X.dtype]
    if diff.size:
        dg = exact_dist_to(X, C, idx[diff], lab_g[diff])
        gap = dg - d1[diff]
        bad = gap > rtol * np.maximum(d1[diff], np.finfo(np.float64).tiny)
        assert not bad.any(), (
            "%d labels differ outside the tie band; first: point %d gpu %d (d=%.17g) oracle %d (d=%.17g)"
            % (bad.sum(), idx[diff][bad][0], lab_g[diff][bad][0], dg[bad][0], lab_o[diff][bad][0],
               d1[diff][bad][0]))
        # an exact tie must go to the lowest index, which is the oracle's label
        assert not (gap == 0).any(), "exact tie not given to the lowest index"
    if mindist_g is not None:
        md = mindist_g[idx].astype(np.float64)
        assert np.all(md >= 0)
        xn = (X[idx].astype(np.float64) ** 2).sum(1)
        cn = (C.astype(np.float64) ** 2).sum(1).max()
        # the expanded form cancels: absolute error scales with the norms, not with the distance;
        # the bound is the one the header documents, from the library's own rounding band
        code = ftk.F32 if X.dtype == np.float32 else ftk.F64
        _, band = ftk.ft_thresholds(code, X.shape[0], X.shape[1], C.shape[0], ftk.FT_OFF)
        atol = 1.5 * band * (np.sqrt(xn * cn) + 0.5 * cn)
        err = np.abs(md - d1)
        assert np.all(err <= 1e-5 * d1 + atol), "mindist off: max err %g" % err.max()
    return int(diff.size), int(idx.size)


def check_moved_labels_within_detection_threshold(X, C, lab, lab_clean, ft_mode, coefs=None):
    """Labels under injected faults against the fault-free labels of the same mode.

    STRICT: identical.  CORRECT (the paper's scheme): an error below the detection threshold of
    Section 2.3 passes unnoticed and may move the point whose score it hit, but only to a centroid
    whose exact squared distance exceeds the oracle's best by less than twice (scores are half
    distances) the threshold plus the settlement band of THAT point, as the library reports them
    (``coefs`` = (detect_coef, band_coef) for a path other than the one ftk_ft_thresholds describes).
    Returns the number of moved labels."""
    diff = np.flatnonzero(lab != lab_clean)
    if ft_mode == ftk.FT_STRICT:
        assert diff.size == 0, "%d labels changed under injection in strict mode" % diff.size
        return 0
    if diff.size == 0:
        return 0
    code = ftk.F32 if X.dtype == np.float32 else ftk.F64
    detect, band = coefs if coefs is not None else ftk.ft_thresholds(code, X.shape[0], X.shape[1], C.shape[0], ft_mode)
    _, d1, _ = oracle.assign(X, C, diff)
    d_new = exact_dist_to(X, C, diff, lab[diff])
    cmax2 = (C.astype(np.float64) ** 2).sum(1).max()
    B = np.sqrt((X[diff].astype(np.float64) ** 2).sum(1) * cmax2) + 0.5 * cmax2
    tol = 2.0 * (detect + band) * B
    worst = ((d_new - d1) / tol).max()
    assert worst <= 1.0, ("%d labels moved, the worst by %.3g of the detection threshold of its point"
                          % (diff.size, worst))
    return int(diff.size)


def check_centroids(C_g: np.ndarray, C_o: np.ndarray):
    rtol = CENTROID_RTOL[C_o.dtype]
    scale = np.maximum(np.abs(C_o.astype(np.float64)),
                       1e-3 * np.abs(C_o.astype(np.float64)).max(axis=1, keepdims=True))
    err = np.abs(C_g.astype(np.float64) - C_o.astype(np.float64))
    worst = (err / np.maximum(scale, np.finfo(np.float64).tiny)).max() if err.size else 0.0
    assert worst <= rtol, "centroids differ: worst relative error %g > %g" % (worst, rtol)
    return worst


def gpu_assign(X, C, **kw):
    labels, mind = ftk.kmeans_assign(to_dev(X), to_dev(C), **kw)
    torch.cuda.synchronize()
    return labels.cpu().numpy(), (None if mind is None else mind.cpu().numpy())


def gpu_update(X, labels, C_prev):
    Cd = to_dev(C_prev).clone()
    _, counts = ftk.kmeans_update(to_dev(X), to_dev(labels.astype(np.int32)), Cd)
    torch.cuda.synchronize()
    return Cd.cpu().numpy(), counts.cpu().numpy()

"""Checksum (ABFT) oracle in float64 numpy -- TEST INFRASTRUCTURE.

Plain statements of the identities the fault-tolerant contraction relies on.
Notation follows the paper: X is the m x k sample block, Y the k x n centroid
block (centroids as columns), D = X Y the product the distance step needs.

  * classic encoding, Section 2.3, Eq. (3)-(5):   X' = [X; e^T X],  Y' = [Y, Y e],
    D' = X' Y' = [[D, D e], [e^T D, .]]
  * online (outer-product) form, Section 2.3, Eq. (6): the same relation holds
    after every rank-one update of the accumulation.
  * location encoding, Section 4.1: a second weight vector e2 = [1, 2, ...]
    next to e1 = [1, ..., 1]; the three scalars e1^T X Y e1, e1^T X Y e2 and
    e2^T X Y e1 locate one corrupted element of the tile and give its error.
  * per-sample (row) form: Eq. (5)'s column D e = X (Y e) taken with both weight
    vectors; it locates the corrupted column within a row.
  * cost model, Section 4.2: three extra matrix instructions per warp tile of
    m_w x n_w instructions.

Where the paper leaves a choice: the weights of e2 count positions inside the
tile (1..rows, 1..cols), and the detection threshold is an argument.
"""
from __future__ import annotations

import numpy as np


def e1(n: int) -> np.ndarray:
    return np.ones(n, dtype=np.float64)


def e2(n: int) -> np.ndarray:
    return np.arange(1, n + 1, dtype=np.float64)


def encode(X: np.ndarray, Y: np.ndarray):
    """Eq. (3)-(5): returns (X', Y', D') with the checksum row / column appended."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    Xc = e1(X.shape[0]) @ X            # e^T X, Eq. (3)
    Yr = Y @ e1(Y.shape[1])            # Y e,   Eq. (4)
    Xp = np.vstack([X, Xc[None, :]])
    Yp = np.hstack([Y, Yr[:, None]])
    return Xp, Yp, Xp @ Yp             # Eq. (5)


def online_outer_product(X: np.ndarray, Y: np.ndarray):
    """Eq. (6): accumulate D' one rank-one update at a time.

    Yields, after every step s, the running D'_s; the caller checks that its last
    column equals the row sums of its data block and its last row the column sums.
    """
    Xp, Yp, _ = encode(X, Y)
    acc = np.zeros((Xp.shape[0], Yp.shape[1]), dtype=np.float64)
    for s in range(Xp.shape[1]):
        acc = acc + np.outer(Xp[:, s], Yp[s, :])
        yield acc.copy()


def tile_checksums(X: np.ndarray, Y: np.ndarray):
    """Section 4.1: the three scalars carried with a tile, from operand checksums.

    Returns (c11, c12, c21) = (e1^T X Y e1, e1^T X Y e2, e2^T X Y e1), each formed
    as (weights^T X) (Y weights) so that the product D itself is never used.
    """
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    m, n = X.shape[0], Y.shape[1]
    x1, x2 = e1(m) @ X, e2(m) @ X
    y1, y2 = Y @ e1(n), Y @ e2(n)
    return float(x1 @ y1), float(x1 @ y2), float(x2 @ y1)


def tile_sums(S: np.ndarray):
    """The same three scalars taken from a computed (possibly corrupted) tile S."""
    S = np.asarray(S, dtype=np.float64)
    m, n = S.shape
    return float(e1(m) @ S @ e1(n)), float(e1(m) @ S @ e2(n)), float(e2(m) @ S @ e1(n))


def locate_and_correct(S: np.ndarray, carried, threshold: float):
    """Detect, locate and correct one corrupted element of tile S.

    ``carried`` = tile_checksums of the operands.  Returns (S_fixed, info) where
    info is None when the checksums agree within ``threshold`` and otherwise a
    dict with delta, row, col (0-based) and ``ok`` = whether the decoded location
    is integral and inside the tile (if not, S is returned unchanged).
    """
    S = np.array(S, dtype=np.float64, copy=True)
    s11, s12, s21 = tile_sums(S)
    c11, c12, c21 = carried
    delta = s11 - c11
    if not (abs(delta) > threshold):
        return S, None
    m, n = S.shape
    if not np.isfinite(delta):
        return S, dict(delta=delta, row=-1, col=-1, ok=False)
    fi = (s21 - c21) / delta          # = weight of the corrupted row    (1-based)
    fj = (s12 - c12) / delta          # = weight of the corrupted column (1-based)
    i, j = int(round(fi)) - 1, int(round(fj)) - 1
    ok = (abs(fi - round(fi)) < 0.1 and abs(fj - round(fj)) < 0.1
          and 0 <= i < m and 0 <= j < n)
    if ok:
        S[i, j] -= delta
    return S, dict(delta=delta, row=i, col=j, ok=ok)


def row_checksums(X: np.ndarray, Y: np.ndarray):
    """Per-sample form: (X (Y e1), X (Y e2)), one pair of checksums per row of D."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    n = Y.shape[1]
    return X @ (Y @ e1(n)), X @ (Y @ e2(n))


def row_locate_and_correct(S: np.ndarray, carried, threshold: float):
    """Row form of detect / locate / correct: at most one bad element per row."""
    S = np.array(S, dtype=np.float64, copy=True)
    n = S.shape[1]
    r1, r2 = carried
    found = []
    for i in range(S.shape[0]):
        delta = S[i] @ e1(n) - r1[i]
        if not (abs(delta) > threshold):
            continue
        fj = (S[i] @ e2(n) - r2[i]) / delta if np.isfinite(delta) else np.nan
        ok = bool(np.isfinite(fj) and abs(fj - round(fj)) < 0.1 and 1 <= round(fj) <= n)
        j = int(round(fj)) - 1 if ok else -1
        if ok:
            S[i, j] -= delta
        found.append(dict(row=i, col=j, delta=float(delta), ok=ok))
    return S, found


def flip_bit(value, bit: int, dtype):
    """Fault model of Section 2.1: flip one bit of the float32 / float64 pattern."""
    dtype = np.dtype(dtype)
    itype = np.uint32 if dtype == np.float32 else np.uint64
    a = np.array([value], dtype=dtype)
    a.view(itype)[0] ^= itype(1) << itype(bit)
    return a[0]


def mma_overhead(m_w: int, n_w: int) -> float:
    """Section 4.2: three extra matrix instructions per m_w x n_w warp tile."""
    return 3.0 / (m_w * n_w)

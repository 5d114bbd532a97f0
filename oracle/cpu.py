"""ctypes front-end of the C oracle (``ftk_oracle.c``) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
It never touches the HIP library and the HIP path never touches it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "ftk_oracle.c"
_LIB = _HERE / "libftk_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP, no fused contraction)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
             "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"],
            check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(str(_LIB))
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.oracle_assign_rows.argtypes = [i32, vp, vp, vp, i64, i32, i32, vp, vp, vp]
        L.oracle_assign_rows.restype = i32
        L.oracle_update.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp]
        L.oracle_update.restype = i32
        L.oracle_fit.argtypes = [i32, vp, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp]
        L.oracle_fit.restype = i32
        L.oracle_seeded_indices.argtypes = [ctypes.c_uint64, i64, i32, vp]
        L.oracle_seeded_indices.restype = i32
        L.oracle_splitmix64.argtypes = [ctypes.c_uint64, i32, vp]
        L.oracle_splitmix64.restype = None
        _lib = L
    return _lib


def _code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.float64:
        return 1
    raise TypeError("oracle takes float32 or float64 storage, got %s" % a.dtype)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(X, C):
    if X.ndim != 2 or C.ndim != 2 or X.shape[1] != C.shape[1]:
        raise ValueError("X [N,D] and C [K,D] expected")
    if X.dtype != C.dtype:
        raise TypeError("X and C must share a dtype")
    if not (X.flags.c_contiguous and C.flags.c_contiguous):
        raise ValueError("row-major contiguous arrays expected")


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    return os.cpu_count() or 1


def assign(X: np.ndarray, C: np.ndarray, rows: np.ndarray | None = None):
    """Eq. (1): (labels int32, best squared distance f64, second-best f64).

    ``rows`` restricts the computation to the listed point indices.
    """
    _check(X, C)
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        if rows.size and (rows.min() < 0 or rows.max() >= X.shape[0]):
            raise IndexError("row index out of range")
        n = rows.size
    else:
        n = X.shape[0]
    labels = np.empty(n, dtype=np.int32)
    best = np.empty(n, dtype=np.float64)
    second = np.empty(n, dtype=np.float64)
    rc = _load().oracle_assign_rows(_code(X), _p(X), _p(C), _p(rows), n, X.shape[1], C.shape[0],
                                    _p(labels), _p(best), _p(second))
    if rc:
        raise RuntimeError("oracle_assign_rows failed: %d" % rc)
    return labels, best, second


def update(X: np.ndarray, labels: np.ndarray, C_prev: np.ndarray):
    """Eq. (2): (new centroids in X's dtype, counts int64); empty clusters keep C_prev."""
    _check(X, C_prev)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    if labels.shape != (X.shape[0],):
        raise ValueError("labels must have one entry per point")
    C = np.array(C_prev, copy=True, order="C")
    counts = np.zeros(C.shape[0], dtype=np.int64)
    rc = _load().oracle_update(_code(X), _p(X), _p(labels), X.shape[0], X.shape[1], C.shape[0],
                               _p(C), _p(counts))
    if rc:
        raise RuntimeError("oracle_update failed: %d" % rc)
    return C, counts


def fit(X: np.ndarray, C0: np.ndarray, iters: int, history: bool = False):
    """Lloyd iterations from C0.  Returns dict(C, labels, counts, inertia[, C_hist, labels_hist])."""
    _check(X, C0)
    N, D = X.shape
    K = C0.shape[0]
    C = np.array(C0, copy=True, order="C")
    labels = np.zeros(N, dtype=np.int32)
    counts = np.zeros(K, dtype=np.int64)
    inertia = np.zeros(max(iters, 0), dtype=np.float64)
    C_hist = np.zeros((iters, K, D), dtype=X.dtype) if history else None
    labels_hist = np.zeros((iters, N), dtype=np.int32) if history else None
    rc = _load().oracle_fit(_code(X), _p(X), N, D, K, iters, _p(C), _p(labels), _p(counts),
                            _p(inertia), _p(C_hist), _p(labels_hist))
    if rc:
        raise RuntimeError("oracle_fit failed: %d" % rc)
    out = dict(C=C, labels=labels, counts=counts, inertia=inertia)
    if history:
        out.update(C_hist=C_hist, labels_hist=labels_hist)
    return out


def seeded_indices(seed: int, N: int, K: int) -> np.ndarray:
    """K distinct indices in [0,N): Floyd sampling driven by SplitMix64(seed)."""
    idx = np.empty(K, dtype=np.int64)
    rc = _load().oracle_seeded_indices(ctypes.c_uint64(seed & (2**64 - 1)), N, K, _p(idx))
    if rc:
        raise ValueError("need 1 <= K <= N")
    return idx


def splitmix64(seed: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.uint64)
    _load().oracle_splitmix64(ctypes.c_uint64(seed & (2**64 - 1)), n, _p(out))
    return out

"""Thin ctypes binding of libftkmeans (argument marshalling only).

PyTorch provides device memory and the current stream; every step of the hot path runs
inside the HIP library.  There is no CPU fallback: if the library is missing or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

FT_OFF, FT_DETECT, FT_CORRECT, FT_STRICT = 0, 1, 2, 3
F32, F64 = 0, 1

_LIB_PATH = Path(__file__).resolve().parent / "libftkmeans.so"
_lib = None

STAT_FIELDS = ("tiles_checked", "injected", "detected", "corrected", "recomputed",
               "uncorrectable", "refined", "max_residual_ppm")


class Geometry(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in
                ("workgroups", "waves_per_workgroup", "tiles_per_wave", "regs_per_tile", "lanes", "bits")]


class FtkError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("ftkmeans error %d: %s" % (code, text))
        self.code = code


def load():
    """Load the shared library (built by ``__graft_entry__.build()``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not _LIB_PATH.exists():
        raise FileNotFoundError(
            "%s not found: build it with `python __graft_entry__.py` (hipcc, gfx950)" % _LIB_PATH)
    L = ctypes.CDLL(str(_LIB_PATH))
    vp, i64, i32, u64, sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                             ctypes.c_size_t)
    L.ftk_workspace_bytes.argtypes = [i32, i64, i32, i32, i32]
    L.ftk_workspace_bytes.restype = sz
    L.ftk_assign_geometry.argtypes = [i32, i64, i32, i32, i32, ctypes.POINTER(Geometry)]
    L.ftk_assign_geometry.restype = i32
    L.ftk_ft_thresholds.argtypes = [i32, i64, i32, i32, i32, ctypes.POINTER(ctypes.c_double),
                                    ctypes.POINTER(ctypes.c_double)]
    L.ftk_ft_thresholds.restype = i32
    L.ftk_plan_padded_rows.argtypes = [i32, i64, i32, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.ftk_plan_padded_rows.restype = i32
    L.ftk_kmeans_assign.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp, i32, vp, i32, vp, vp, sz, vp]
    L.ftk_kmeans_assign.restype = i32
    L.ftk_kmeans_assign_static.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp, i32, vp, i32, vp, vp]
    L.ftk_kmeans_assign_static.restype = i32
    L.ftk_static_scratch_bytes.argtypes = []
    L.ftk_static_scratch_bytes.restype = sz
    L.ftk_kmeans_assign_fast.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp, i32, vp, i32, vp, vp, sz, vp]
    L.ftk_kmeans_assign_fast.restype = i32
    L.ftk_fast_plan.argtypes = [i32, i64, i32, i32, i32, vp, vp, vp]
    L.ftk_fast_plan.restype = i32
    L.ftk_absmax.argtypes = [i32, vp, i64, vp, vp]
    L.ftk_absmax.restype = i32
    L.ftk_kmeans_update.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp, vp, vp, sz, vp]
    L.ftk_kmeans_update.restype = i32
    L.ftk_kmeans_step_batched.argtypes = [i32, vp, i64, i32, i32, vp, vp, vp, vp, vp, i64, vp, sz, vp]
    L.ftk_kmeans_step_batched.restype = i32
    L.ftk_kmeans_update_ft.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp, vp, i32, vp, i32, vp, vp, sz, vp]
    L.ftk_kmeans_update_ft.restype = i32
    L.ftk_update_geometry.argtypes = [i32, i64, i32, i32, i32, ctypes.POINTER(Geometry)]
    L.ftk_update_geometry.restype = i32
    L.ftk_kmeans_fit.argtypes = [i32, vp, i64, i32, i32, i32, u64, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    L.ftk_kmeans_fit.restype = i32
    L.ftk_kmeans_fit_fast.argtypes = [i32, vp, i64, i32, i32, i32, u64, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    L.ftk_kmeans_fit_fast.restype = i32
    L.ftk_seeded_indices.argtypes = [u64, i64, i32, vp]
    L.ftk_seeded_indices.restype = i32
    L.ftk_profile_enable.argtypes = [i32]
    L.ftk_profile_enable.restype = i32
    L.ftk_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    L.ftk_profile_read.restype = i32
    L.ftk_tuning_override.argtypes = [i32, i32, i32]
    L.ftk_tuning_override.restype = i32
    L.ftk_last_error.restype = ctypes.c_char_p
    L.ftk_version.restype = ctypes.c_char_p
    _lib = L
    return L


EXPORTS = ("ftk_workspace_bytes", "ftk_assign_geometry", "ftk_plan_padded_rows", "ftk_ft_thresholds", "ftk_kmeans_assign_static", "ftk_static_scratch_bytes", "ftk_kmeans_assign", "ftk_kmeans_assign_fast", "ftk_fast_plan", "ftk_absmax",
           "ftk_kmeans_update", "ftk_kmeans_update_ft", "ftk_kmeans_step_batched", "ftk_update_geometry", "ftk_kmeans_fit", "ftk_kmeans_fit_fast", "ftk_seeded_indices", "ftk_profile_enable",
           "ftk_profile_read", "ftk_tuning_override", "ftk_last_error", "ftk_version")


def _check(rc):
    if rc != 0:
        raise FtkError(rc, load().ftk_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.float64:
        return F64
    raise TypeError("float32 or float64 tensor expected, got %s" % t.dtype)


def _dev2d(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if t.dim() != 2 or not t.is_contiguous():
        raise ValueError("%s must be a contiguous 2-D tensor" % name)
    return t


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def ft_thresholds(dtype_code: int, N: int, D: int, K: int, ft_mode: int = FT_CORRECT):
    """(detect_coef, band_coef): detection threshold and exact-settlement band of point i are these
    times ||x_i|| max||c|| + max||c||^2/2, in score units (half a squared distance)."""
    a, b = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(load().ftk_ft_thresholds(dtype_code, N, D, K, ft_mode, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def plan_padded_rows(dtype_code: int, N: int, D: int, K: int):
    """(largest padded centroid-row count over all kernel variants, rows the workspace reserves)"""
    a, b = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(load().ftk_plan_padded_rows(dtype_code, N, D, K, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def workspace_bytes(dtype_code: int, N: int, D: int, K: int, ft_mode: int = FT_OFF) -> int:
    n = load().ftk_workspace_bytes(dtype_code, N, D, K, ft_mode)
    if n == 0:
        raise FtkError(1, load().ftk_last_error().decode())
    return n


def new_workspace(X: torch.Tensor, K: int, ft_mode: int = FT_CORRECT) -> torch.Tensor:
    n = workspace_bytes(_dtype_code(X), X.shape[0], X.shape[1], K, ft_mode)
    return torch.empty(n + 256, dtype=torch.uint8, device=X.device)


def _ws_args(ws: torch.Tensor):
    base = ws.data_ptr()
    aligned = (base + 255) // 256 * 256
    return aligned, ws.numel() - (aligned - base)


def assign_geometry(dtype_code: int, N: int, D: int, K: int, ft_mode: int = FT_OFF) -> Geometry:
    g = Geometry()
    _check(load().ftk_assign_geometry(dtype_code, N, D, K, ft_mode, ctypes.byref(g)))
    return g


def new_stats(device) -> torch.Tensor:
    return torch.zeros(len(STAT_FIELDS), dtype=torch.int64, device=device)


def stats_dict(stats: torch.Tensor) -> dict:
    return dict(zip(STAT_FIELDS, (int(v) for v in stats.cpu().tolist())))


def make_faults(rows, device) -> torch.Tensor:
    """rows: iterable of (workgroup, wave, tile, reg, lane, bit) -> device tensor [n, 6] uint32-as-int32."""
    t = torch.tensor(list(rows), dtype=torch.int64).reshape(-1, 6)
    return t.to(torch.int32).contiguous().to(device)


def kmeans_assign(X, C, labels=None, mindist=None, ft_mode=FT_OFF, faults=None, stats=None,
                  workspace=None, want_mindist=True):
    """Assignment step (Eq. 1).  Returns (labels int32 [N], mindist [N] or None)."""
    _dev2d(X, "X"), _dev2d(C, "C")
    if X.dtype != C.dtype or X.shape[1] != C.shape[1]:
        raise ValueError("X [N,D] and C [K,D] must share dtype and D")
    N, D = X.shape
    K = C.shape[0]
    if labels is None:
        labels = torch.empty(N, dtype=torch.int32, device=X.device)
    if mindist is None and want_mindist:
        mindist = torch.empty(N, dtype=X.dtype, device=X.device)
    if workspace is None:
        workspace = new_workspace(X, K, ft_mode)
    wp, wn = _ws_args(workspace)
    nf = 0 if faults is None else faults.shape[0]
    _check(load().ftk_kmeans_assign(_dtype_code(X), X.data_ptr(), C.data_ptr(), N, D, K,
                                    labels.data_ptr(), _ptr(mindist), ft_mode, _ptr(faults), nf,
                                    _ptr(stats), wp, wn, _stream()))
    return labels, mindist


def static_scratch_bytes() -> int:
    return load().ftk_static_scratch_bytes()


def kmeans_assign_static(X, C, labels, mindist=None, ft_mode=FT_OFF, faults=None, stats=None):
    """Assignment step through the entry point that allocates nothing: outputs are the caller's
    tensors, scratch is the library's static device array.  Returns (labels, mindist)."""
    _dev2d(X, "X"), _dev2d(C, "C")
    if X.dtype != C.dtype or X.shape[1] != C.shape[1]:
        raise ValueError("X [N,D] and C [K,D] must share dtype and D")
    N, D = X.shape
    K = C.shape[0]
    nf = 0 if faults is None else faults.shape[0]
    _check(load().ftk_kmeans_assign_static(_dtype_code(X), X.data_ptr(), C.data_ptr(), N, D, K,
                                           labels.data_ptr(), _ptr(mindist), ft_mode, _ptr(faults), nf,
                                           _ptr(stats), _stream()))
    return labels, mindist


def fast_plan(dtype_code: int, N: int, D: int, K: int, ft_mode: int = FT_OFF):
    """(geometry, detect_coef, band_coef) of the split-bf16 path: what assign_geometry and
    ft_thresholds report for the fp32 path."""
    g = Geometry()
    a, b = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(load().ftk_fast_plan(dtype_code, N, D, K, ft_mode, ctypes.byref(g), ctypes.byref(a), ctypes.byref(b)))
    return g, a.value, b.value


def kmeans_assign_fast(X, C, labels=None, mindist=None, workspace=None, want_mindist=True, ft_mode=FT_OFF,
                       faults=None, stats=None):
    """Assignment step on the split-bf16 matrix path (fp32 data, D <= 128).  Returns (labels, mindist)."""
    _dev2d(X, "X"), _dev2d(C, "C")
    if X.dtype != C.dtype or X.shape[1] != C.shape[1]:
        raise ValueError("X [N,D] and C [K,D] must share dtype and D")
    N, D = X.shape
    K = C.shape[0]
    if labels is None:
        labels = torch.empty(N, dtype=torch.int32, device=X.device)
    if mindist is None and want_mindist:
        mindist = torch.empty(N, dtype=X.dtype, device=X.device)
    if workspace is None:
        workspace = new_workspace(X, K, ft_mode)
    wp, wn = _ws_args(workspace)
    nf = 0 if faults is None else faults.shape[0]
    _check(load().ftk_kmeans_assign_fast(_dtype_code(X), X.data_ptr(), C.data_ptr(), N, D, K,
                                         labels.data_ptr(), _ptr(mindist), ft_mode, _ptr(faults), nf,
                                         _ptr(stats), wp, wn, _stream()))
    return labels, mindist


def tuning_override(assign_variant: int = -1, generic_tiles: int = -1, update_path: int = -1):
    """Force kernel choices for later calls (-1 = built-in rule); for the shape-sweep tool and tests."""
    _check(load().ftk_tuning_override(assign_variant, generic_tiles, update_path))


def absmax(X: torch.Tensor) -> torch.Tensor:
    out = torch.empty(1, dtype=torch.float64, device=X.device)
    _check(load().ftk_absmax(_dtype_code(X), X.data_ptr(), X.numel(), out.data_ptr(), _stream()))
    return out


def update_geometry(dtype_code: int, N: int, D: int, K: int, rows_aligned16: bool = True) -> Geometry:
    g = Geometry()
    _check(load().ftk_update_geometry(dtype_code, N, D, K, 1 if rows_aligned16 else 0, ctypes.byref(g)))
    return g


def kmeans_update(X, labels, C, counts=None, x_absmax=None, workspace=None, ft_mode=FT_OFF, faults=None,
                  stats=None):
    """Update step (Eq. 2), in place on C; with ft_mode on, under dual modular redundancy.
    Returns (C, counts int32 [K])."""
    _dev2d(X, "X"), _dev2d(C, "C")
    N, D = X.shape
    K = C.shape[0]
    if labels.dtype != torch.int32 or labels.shape != (N,) or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 vector of length N")
    if counts is None:
        counts = torch.empty(K, dtype=torch.int32, device=X.device)
    if workspace is None:
        workspace = new_workspace(X, K, FT_OFF)
    wp, wn = _ws_args(workspace)
    if ft_mode == FT_OFF and faults is None and stats is None:
        _check(load().ftk_kmeans_update(_dtype_code(X), X.data_ptr(), labels.data_ptr(), N, D, K,
                                        C.data_ptr(), counts.data_ptr(), _ptr(x_absmax), wp, wn, _stream()))
    else:
        nf = 0 if faults is None else int(faults.shape[0])
        _check(load().ftk_kmeans_update_ft(_dtype_code(X), X.data_ptr(), labels.data_ptr(), N, D, K,
                                           C.data_ptr(), counts.data_ptr(), _ptr(x_absmax), ft_mode,
                                           _ptr(faults), nf, _ptr(stats), wp, wn, _stream()))
    return C, counts


def kmeans_step_batched(X, C, batch_rows, labels=None, mindist=None, counts=None, x_absmax=None, workspace=None):
    """One Lloyd iteration in batches of `batch_rows` points (assign a batch, add it to the sums while
    it is cache-resident); C is updated in place.  Returns (labels, mindist, counts)."""
    _dev2d(X, "X"), _dev2d(C, "C")
    N, D = X.shape
    K = C.shape[0]
    if labels is None:
        labels = torch.empty(N, dtype=torch.int32, device=X.device)
    if mindist is None:
        mindist = torch.empty(N, dtype=X.dtype, device=X.device)
    if counts is None:
        counts = torch.empty(K, dtype=torch.int32, device=X.device)
    if x_absmax is None:
        x_absmax = absmax(X)
    if workspace is None:
        workspace = new_workspace(X, K, FT_OFF)
    wp, wn = _ws_args(workspace)
    _check(load().ftk_kmeans_step_batched(_dtype_code(X), X.data_ptr(), N, D, K, C.data_ptr(), labels.data_ptr(),
                                          _ptr(mindist), counts.data_ptr(), x_absmax.data_ptr(), int(batch_rows),
                                          wp, wn, _stream()))
    return labels, mindist, counts


def seeded_indices(seed: int, N: int, K: int):
    import numpy as np
    idx = np.empty(K, dtype=np.int64)
    _check(load().ftk_seeded_indices(seed & (2**64 - 1), N, K, idx.ctypes.data))
    return idx


def profile_enable(on: bool) -> None:
    _check(load().ftk_profile_enable(1 if on else 0))


def profile_read():
    """(total milliseconds, launches) of the main assignment kernel since the last read."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(load().ftk_profile_read(ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


def kmeans_fit(X, K, iters, seed=0, C_init=None, ft_mode=FT_OFF, stats=None, workspace=None,
               want_inertia=True, fast=False):
    """Lloyd loop.  Returns dict(C, labels, counts, inertia (numpy, host) or None).
    fast=True runs the assignment on the split-bf16 matrix path (fp32, D <= 128)."""
    import numpy as np
    _dev2d(X, "X")
    N, D = X.shape
    if C_init is not None:
        _dev2d(C_init, "C_init")
        if C_init.shape != (K, D) or C_init.dtype != X.dtype:
            raise ValueError("C_init must be [K,D] of X's dtype")
    C = torch.empty(K, D, dtype=X.dtype, device=X.device)
    labels = torch.empty(N, dtype=torch.int32, device=X.device)
    counts = torch.empty(K, dtype=torch.int32, device=X.device)
    inertia = np.zeros(iters, dtype=np.float64) if want_inertia else None
    if workspace is None:
        workspace = new_workspace(X, K, ft_mode)
    wp, wn = _ws_args(workspace)
    if fast:
        _check(load().ftk_kmeans_fit_fast(_dtype_code(X), X.data_ptr(), N, D, K, iters, seed & (2**64 - 1),
                                          _ptr(C_init), C.data_ptr(), labels.data_ptr(), counts.data_ptr(),
                                          None if inertia is None else inertia.ctypes.data, ft_mode,
                                          _ptr(stats), wp, wn, _stream()))
        return dict(C=C, labels=labels, counts=counts, inertia=inertia)
    _check(load().ftk_kmeans_fit(_dtype_code(X), X.data_ptr(), N, D, K, iters, seed & (2**64 - 1),
                                 _ptr(C_init), C.data_ptr(), labels.data_ptr(), counts.data_ptr(),
                                 None if inertia is None else inertia.ctypes.data, ft_mode,
                                 _ptr(stats), wp, wn, _stream()))
    return dict(C=C, labels=labels, counts=counts, inertia=inertia)

"""ctypes binding of libftk_ablation (measurement-only kernels: the naive kernel, the
unfused GEMM + arg-min variant and the plain-ALU fused variants that precede the fused kernel in the paper's Section 3.1).

Not part of the product path: nothing in ``binding.py`` imports this module.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_LIB_PATH = Path(__file__).resolve().parent / "libftk_ablation.so"
_lib = None

EXPORTS = ("ftk_abl_naive_assign", "ftk_abl_gemm_workspace_bytes", "ftk_abl_gemm_assign",
           "ftk_abl_fused_alu_workspace_bytes", "ftk_abl_fused_alu_assign", "ftk_abl_mfma_bf16",
           "ftk_abl_mfma_f32", "ftk_abl_mfma_f64", "ftk_abl_last_error")


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not _LIB_PATH.exists():
        raise FileNotFoundError(
            "%s not found: build it with `python __graft_entry__.py` (hipcc, gfx950)" % _LIB_PATH)
    L = ctypes.CDLL(str(_LIB_PATH))
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    L.ftk_abl_naive_assign.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp, vp]
    L.ftk_abl_naive_assign.restype = i32
    L.ftk_abl_gemm_workspace_bytes.argtypes = [i32, i64, i32]
    L.ftk_abl_gemm_workspace_bytes.restype = sz
    L.ftk_abl_gemm_assign.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp, vp, sz, vp]
    L.ftk_abl_gemm_assign.restype = i32
    L.ftk_abl_fused_alu_workspace_bytes.argtypes = [i32, i64, i32, i32]
    L.ftk_abl_fused_alu_workspace_bytes.restype = sz
    L.ftk_abl_fused_alu_assign.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp, i32, vp, sz, vp]
    L.ftk_abl_fused_alu_assign.restype = i32
    L.ftk_abl_mfma_bf16.argtypes = [vp, vp, vp, vp, i32, vp]
    L.ftk_abl_mfma_bf16.restype = i32
    for fn in (L.ftk_abl_mfma_f32, L.ftk_abl_mfma_f64):
        fn.argtypes = [vp, vp, vp, vp, i32, vp]
        fn.restype = i32
    L.ftk_abl_last_error.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise RuntimeError("ftk_ablation error %d: %s" % (rc, load().ftk_abl_last_error().decode()))


def _prep(X, C):
    assert X.is_cuda and C.is_cuda and X.dtype == C.dtype and X.is_contiguous() and C.is_contiguous()
    assert X.dtype in (torch.float32, torch.float64) and X.shape[1] == C.shape[1]
    return 0 if X.dtype == torch.float32 else 1


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def naive_assign(X, C, labels=None, mindist=None):
    code = _prep(X, C)
    N, D = X.shape
    K = C.shape[0]
    labels = labels if labels is not None else torch.empty(N, dtype=torch.int32, device=X.device)
    mindist = mindist if mindist is not None else torch.empty(N, dtype=X.dtype, device=X.device)
    _check(load().ftk_abl_naive_assign(code, X.data_ptr(), C.data_ptr(), N, D, K, labels.data_ptr(),
                                       mindist.data_ptr(), _stream()))
    return labels, mindist


def gemm_workspace(X, K):
    code = 0 if X.dtype == torch.float32 else 1
    nbytes = load().ftk_abl_gemm_workspace_bytes(code, X.shape[0], K)
    return torch.empty(nbytes, dtype=torch.uint8, device=X.device)


def gemm_assign(X, C, labels=None, mindist=None, workspace=None):
    code = _prep(X, C)
    N, D = X.shape
    K = C.shape[0]
    labels = labels if labels is not None else torch.empty(N, dtype=torch.int32, device=X.device)
    mindist = mindist if mindist is not None else torch.empty(N, dtype=X.dtype, device=X.device)
    workspace = workspace if workspace is not None else gemm_workspace(X, K)
    _check(load().ftk_abl_gemm_assign(code, X.data_ptr(), C.data_ptr(), N, D, K, labels.data_ptr(),
                                      mindist.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()))
    return labels, mindist


def fused_alu_workspace(X, K, variant):
    code = 0 if X.dtype == torch.float32 else 1
    nbytes = load().ftk_abl_fused_alu_workspace_bytes(code, X.shape[0], K, variant)
    return torch.empty(nbytes, dtype=torch.uint8, device=X.device)


def fused_alu_assign(X, C, variant, labels=None, mindist=None, workspace=None):
    code = _prep(X, C)
    N, D = X.shape
    K = C.shape[0]
    labels = labels if labels is not None else torch.empty(N, dtype=torch.int32, device=X.device)
    mindist = mindist if mindist is not None else torch.empty(N, dtype=X.dtype, device=X.device)
    workspace = workspace if workspace is not None else fused_alu_workspace(X, K, variant)
    _check(load().ftk_abl_fused_alu_assign(code, X.data_ptr(), C.data_ptr(), N, D, K, labels.data_ptr(),
                                           mindist.data_ptr(), variant, workspace.data_ptr(),
                                           workspace.numel(), _stream()))
    return labels, mindist


def mfma_bf16(A_bits, B_bits, C):
    """D = A B + C by one bf16 matrix instruction per 32x32x16 problem.  A_bits [T,32,16] and B_bits
    [T,16,32] are int16 tensors holding bf16 bit patterns, C [T,32,32] float32."""
    assert A_bits.is_cuda and A_bits.dtype == torch.int16 and A_bits.is_contiguous() and A_bits.shape[1:] == (32, 16)
    assert B_bits.dtype == torch.int16 and B_bits.is_contiguous() and B_bits.shape[1:] == (16, 32)
    assert C.dtype == torch.float32 and C.is_contiguous() and C.shape[1:] == (32, 32)
    T = A_bits.shape[0]
    assert B_bits.shape[0] == T and C.shape[0] == T
    D = torch.empty_like(C)
    _check(load().ftk_abl_mfma_bf16(A_bits.data_ptr(), B_bits.data_ptr(), C.data_ptr(), D.data_ptr(), T, _stream()))
    return D


def mfma_plain(A, B, C):
    """D = A B + C by one fp32 (A [T,32,2], B [T,2,32], C [T,32,32]) or fp64 (A [T,16,4],
    B [T,4,16], C [T,16,16]) matrix instruction per problem."""
    assert A.is_cuda and A.dtype == B.dtype == C.dtype and A.is_contiguous() and B.is_contiguous() and C.is_contiguous()
    T = A.shape[0]
    if A.dtype == torch.float32:
        assert A.shape == (T, 32, 2) and B.shape == (T, 2, 32) and C.shape == (T, 32, 32)
        fn = load().ftk_abl_mfma_f32
    else:
        assert A.dtype == torch.float64 and A.shape == (T, 16, 4) and B.shape == (T, 4, 16) and C.shape == (T, 16, 16)
        fn = load().ftk_abl_mfma_f64
    D = torch.empty_like(C)
    _check(fn(A.data_ptr(), B.data_ptr(), C.data_ptr(), D.data_ptr(), T, _stream()))
    return D

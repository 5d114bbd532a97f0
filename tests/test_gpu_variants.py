"""The measurement-only variants (naive kernel of Section 3.1.1, unfused GEMM + arg-min of
Section 3.1.2, plain-ALU GEMM with the minimum fused in of Sections 3.1.3 and 3.1.4) against the oracle, through their own C boundary (include/ftk_ablation.h)."""
import ctypes
import re
from pathlib import Path

import numpy as np
import pytest

from paper_2408_01391_amd import ablation

ROOT = Path(__file__).resolve().parent.parent


def _declared():
    text = (ROOT / "include" / "ftk_ablation.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ftk_abl_[a-z_0-9]+)\s*\(", text)))


def test_ablation_header_and_binding_agree():
    assert _declared() == sorted(ablation.EXPORTS)


def test_ablation_sources_stay_out_of_the_product_library():
    # the product library is built from csrc/ only and its binding never imports the ablation module
    assert not list((ROOT / "paper_2408_01391_amd" / "csrc").glob("*ablation*"))
    assert "ablation" not in (ROOT / "paper_2408_01391_amd" / "binding.py").read_text()


SHAPES = [  # N, D, K, dtype, spread of the blob centres
    (1000, 8, 37, np.float32, 10.0),
    (4099, 16, 8, np.float32, 10.0),
    (3001, 33, 130, np.float32, 3.0),
    (2050, 128, 64, np.float64, 5.0),
    (777, 5, 3, np.float64, 1.0),
]


def _data(N, D, K, dtype, spread, seed):
    rng = np.random.default_rng(seed)
    centres = rng.uniform(-spread, spread, size=(K, D))
    X = (centres[rng.integers(K, size=N)] + rng.normal(size=(N, D))).astype(dtype)
    C = X[rng.choice(N, K, replace=False)].copy()
    return X, C


@pytest.mark.gpu
@pytest.mark.parametrize("N,D,K,dtype,spread", SHAPES)
def test_naive_kernel_matches_oracle(N, D, K, dtype, spread):
    from tests.gpu_util import check_assign, to_dev
    X, C = _data(N, D, K, dtype, spread, 11)
    lab, md = ablation.naive_assign(to_dev(X), to_dev(C))
    check_assign(X, C, lab.cpu().numpy(), md.cpu().numpy())


def _check_expanded_form(X, C, lab, md):
    """The expanded form is decided in the working precision with no exact settlement, so a label
    may differ from the oracle's where the two distances are closer than that form's rounding
    error, which scales with the norms (not with the distance): |gap| <= 8 (D+4) u (|x|^2+|c|^2)."""
    from oracle import cpu as oracle
    from tests.gpu_util import exact_dist_to
    N, D = X.shape
    K = C.shape[0]
    dtype = X.dtype
    lab = lab.cpu().numpy()
    md = md.cpu().numpy().astype(np.float64)
    lab_o, d1, _ = oracle.assign(X, C)
    assert lab.min() >= 0 and lab.max() < K
    u = np.finfo(dtype).eps / 2
    xn = (X.astype(np.float64) ** 2).sum(1)
    cn = (C.astype(np.float64) ** 2).sum(1).max()
    bound = 8 * (D + 4) * u * (xn + cn)
    diff = np.flatnonzero(lab != lab_o)
    if diff.size:
        gap = exact_dist_to(X, C, diff, lab[diff]) - d1[diff]
        assert np.all(gap <= bound[diff]), "label differs beyond the rounding error of the expanded form"
    assert diff.size <= max(2, N // 100)
    assert np.all(md >= 0) and np.all(np.abs(md - d1) <= bound)


@pytest.mark.gpu
@pytest.mark.parametrize("N,D,K,dtype,spread", SHAPES)
def test_unfused_gemm_variant_matches_oracle_up_to_the_rounding_of_the_expanded_form(N, D, K, dtype, spread):
    from tests.gpu_util import to_dev
    X, C = _data(N, D, K, dtype, spread, 12)
    lab, md = ablation.gemm_assign(to_dev(X), to_dev(C))
    _check_expanded_form(X, C, lab, md)


FUSED_SHAPES = SHAPES + [  # several centroid blocks of 128 with a ragged last one, ragged point tile
    (5000, 8, 1000, np.float32, 10.0),
    (1025, 19, 300, np.float64, 4.0),
]


@pytest.mark.gpu
@pytest.mark.parametrize("variant", [2, 3])
@pytest.mark.parametrize("N,D,K,dtype,spread", FUSED_SHAPES)
def test_plain_alu_fused_variants_match_oracle_up_to_the_rounding_of_the_expanded_form(N, D, K, dtype, spread,
                                                                                     variant):
    from tests.gpu_util import to_dev
    if variant == 3 and dtype == np.float64:
        pytest.skip("the atomic key of variant 3 packs an fp32 distance")
    X, C = _data(N, D, K, dtype, spread, 13)
    lab, md = ablation.fused_alu_assign(to_dev(X), to_dev(C), variant)
    _check_expanded_form(X, C, lab, md)


@pytest.mark.gpu
def test_plain_alu_fused_variants_agree_with_each_other_bit_for_bit():
    """Both take the same products in the same order and break ties to the lowest index, so the
    block-wise reduction and the atomic merge must give identical labels and distances."""
    import torch
    from tests.gpu_util import to_dev
    X, C = _data(6000, 24, 700, np.float32, 6.0, 14)
    Xd, Cd = to_dev(X), to_dev(C)
    l2, m2 = ablation.fused_alu_assign(Xd, Cd, 2)
    l3, m3 = ablation.fused_alu_assign(Xd, Cd, 3)
    assert torch.equal(l2, l3) and torch.equal(m2, m3)


@pytest.mark.gpu
def test_ablation_library_rejects_bad_arguments():
    import torch
    lib = ablation.load()
    assert lib.ftk_abl_naive_assign(0, None, None, 10, 4, 2, None, None, None) == 1
    assert b"invalid" in lib.ftk_abl_last_error()
    X = torch.zeros(16, 4, device="cuda:0")
    C = torch.zeros(2, 4, device="cuda:0")
    lab = torch.zeros(16, dtype=torch.int32, device="cuda:0")
    ws = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    rc = lib.ftk_abl_gemm_assign(0, X.data_ptr(), C.data_ptr(), 16, 4, 2, lab.data_ptr(), None, ws.data_ptr(), 64, None)
    assert rc == 3
    rc = lib.ftk_abl_fused_alu_assign(0, X.data_ptr(), C.data_ptr(), 16, 4, 2, lab.data_ptr(), None, 2, ws.data_ptr(),
                                      64, None)
    assert rc == 3
    big = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    Xd, Cd = X.double(), C.double()
    rc = lib.ftk_abl_fused_alu_assign(1, Xd.data_ptr(), Cd.data_ptr(), 16, 4, 2, lab.data_ptr(), None, 3,
                                      big.data_ptr(), 4096, None)
    assert rc == 1


def test_ablation_library_exports_every_declared_symbol():
    if not ablation._LIB_PATH.exists():
        pytest.skip("libftk_ablation.so not built (run python __graft_entry__.py)")
    try:
        lib = ctypes.CDLL(str(ablation._LIB_PATH))
    except OSError as e:  # the vendor GEMM library it links may be absent on a CPU-only host
        pytest.skip("cannot load: %s" % e)
    for name in _declared():
        assert hasattr(lib, name), name

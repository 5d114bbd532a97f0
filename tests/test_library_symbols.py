"""The C-ABI library loads and exports every symbol include/ftkmeans.h declares (no GPU needed)."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_2408_01391_amd import binding

ROOT = Path(__file__).resolve().parent.parent


def _declared():
    text = (ROOT / "include" / "ftkmeans.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ftk_[a-z_0-9]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared() == sorted(binding.EXPORTS)


def test_library_exports_every_declared_symbol():
    if not binding._LIB_PATH.exists():
        pytest.skip("libftkmeans.so not built (run python __graft_entry__.py)")
    lib = ctypes.CDLL(str(binding._LIB_PATH))
    for name in _declared():
        assert hasattr(lib, name), name
    lib.ftk_version.restype = ctypes.c_char_p
    assert b"gfx950" in lib.ftk_version()


def test_host_only_entry_points_work_without_a_gpu():
    if not binding._LIB_PATH.exists():
        pytest.skip("libftkmeans.so not built")
    from oracle import cpu as oracle
    import numpy as np
    assert np.array_equal(binding.seeded_indices(5, 1000, 50), oracle.seeded_indices(5, 1000, 50))
    assert binding.workspace_bytes(binding.F32, 1 << 20, 8, 1024) > (1 << 20) * 8
    g = binding.assign_geometry(binding.F64, 1000, 512, 64)
    assert g.lanes == 64 and g.bits == 64 and g.workgroups >= 1
    with pytest.raises(binding.FtkError):
        binding.workspace_bytes(binding.F32, 0, 8, 4)


def test_workspace_reserves_every_padded_centroid_row():
    """The prologue writes one half-norm per padded centroid row of the chosen kernel variant; the
    reservation must cover the widest padding for every K, D, dtype and fault-tolerance mode."""
    if not binding._LIB_PATH.exists():
        pytest.skip("libftkmeans.so not built")
    ks = sorted(set(list(range(1, 200, 7)) + [2 ** e + d for e in range(5, 18) for d in (-1, 0, 1, 29)]
                    + [6090, 6091, 7560, 7561, 25536, 25537, 100000, 1000003]))
    for dtype in (binding.F32, binding.F64):
        for D in (4, 8, 12, 16, 24, 32, 33, 128, 512):
            for K in ks:
                planned, reserved = binding.plan_padded_rows(dtype, max(K, 1 << 20), D, K)
                assert K <= planned <= reserved, (dtype, D, K, planned, reserved)

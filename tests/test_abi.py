"""CPU-only checks of the C-ABI library: it loads and exports every symbol the header declares, and the
pure host functions behave (no GPU compute is called)."""
import os
import re

import pytest

from paper_2007_00784_amd import kfac as K

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "kfac.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(kfac_[a-z_]+)\s*\(", src)))


def test_header_symbols_all_exported():
    if not os.path.exists(K.LIB_PATH):
        from paper_2007_00784_amd import build
        build.build()
    L = K.lib()
    syms = declared_symbols()
    assert set(syms) == set(K.EXPORTS)
    for s in syms:
        assert hasattr(L, s), s


def test_host_functions():
    assert K.kfac_strerror(0) == "success"
    assert "workspace" in K.kfac_strerror(K.KFAC_EWORKSPACE)
    assert K.kfac_schedule_due(0, 10, 100) == (True, True)
    assert K.kfac_schedule_due(10, 10, 100) == (True, False)
    assert K.kfac_schedule_due(11, 10, 100) == (False, False)
    nf = ne = 0
    for k in range(200):
        f, e = K.kfac_schedule_due(k, 10, 100)
        nf += f
        ne += e
    assert (nf, ne) == (20, 2)
    with pytest.raises(K.KfacError):
        K.kfac_schedule_due(-1, 10, 100)
    # workspace queries are monotone and cover the exact eig requirement
    a = K.kfac_workspace_bytes(577, 4, 131072)
    b = K.kfac_workspace_bytes(4609, 4, 131072)
    assert 0 < a < b
    assert K.kfac_eig_workspace_bytes([577, 64, 577, 16]) <= a
    assert K.kfac_eig_workspace_bytes([0]) == 0
    assert K.kfac_workspace_bytes(100000, 1, 1) == 0


def test_workspace_query_covers_every_operand_form():
    """kfac_workspace_bytes(max_d, 1, max_R) suffices for one factor update of that size whatever the layout and
    element type of its samples (the split plans differ between the operand forms)."""
    for d in (64, 257, 1153, 4609):
        for R in (1568, 25088, 401408):
            cap = K.kfac_workspace_bytes(d, 1, R)
            assert cap > 0
            for dtype in (K.KFAC_F32, K.KFAC_BF16):
                for T in (1, 4, 5, 8, 9, 49, 196, R):
                    N = max(1, R // T)
                    for layout in (K.KFAC_LAYOUT_RD, K.KFAC_LAYOUT_NDT):
                        it = dict(X=None, dtype=dtype, layout=layout, N=N, d=d - 1, T=T, append_ones=1, scale=1.0, decay=0.0, F=None)
                        need = K.kfac_update_factors_workspace_bytes([it])
                        assert 0 < need <= cap, (d, R, dtype, T, layout, need, cap)

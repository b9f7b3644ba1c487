"""The C-ABI library loads without a GPU and exports every function include/augur.h declares;
argument checks that need no device return the documented error codes."""
import ctypes as C
import os
import re

from paper_1312_3613_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "augur.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(augur_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert len(names) >= 30
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert b"gfx950" in L.augur_version()


def test_argument_errors_without_device():
    L = B.lib()
    h = C.c_void_p()
    assert L.augur_lda_create(None, None, None, C.byref(h)) == B.ERR_INVALID_ARG
    assert "NULL" in B.last_error()
    cfg = B.LdaConfig(0, 5, 3, 0.1, 0.1, 1, 0, None, 0)
    assert L.augur_lda_create(C.byref(cfg), None, None, C.byref(h)) == B.ERR_INVALID_ARG
    cfg = B.LdaConfig(2, 5, 3, -0.1, 0.1, 1, 0, None, 0)
    assert L.augur_lda_create(C.byref(cfg), None, None, C.byref(h)) == B.ERR_INVALID_ARG
    assert "alpha" in B.last_error()
    cfg = B.LdaConfig(2, 5, 3, 0.1, float("nan"), 1, 0, None, 0)
    assert L.augur_lda_create(C.byref(cfg), None, None, C.byref(h)) == B.ERR_INVALID_ARG
    cfg = B.LdaConfig(2, 5, 3, 0.1, 0.1, 1, 0, None, 0x80)
    assert L.augur_lda_create(C.byref(cfg), None, None, C.byref(h)) == B.ERR_INVALID_ARG
    assert L.augur_lda_create(C.byref(cfg), None, None, None) == B.ERR_INVALID_ARG
    assert h.value is None
    g = B.GmmConfig(0, 8, 16, 1.0, 10.0, 1.0, 0.0, 0.0, 1, 0, None, 0)
    assert L.augur_gmm_create(C.byref(g), None, C.byref(h)) == B.ERR_INVALID_ARG
    for fn in (L.augur_lda_sync, L.augur_gmm_sync, L.augur_lda_step_finish, L.augur_gmm_step_finish):
        assert fn(None) == B.ERR_INVALID_ARG
    assert L.augur_lda_sweep(None, 1) == B.ERR_INVALID_ARG
    L.augur_lda_destroy(None)
    L.augur_gmm_destroy(None)

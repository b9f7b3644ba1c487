"""The C-ABI library loads without a GPU and exports every function include/augur.h declares;
argument checks that need no device return the documented error codes."""
import ctypes as C
import os
import re

from paper_1312_3613_amd import binding as B
from tests import parity as P

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
    # dim 1, K = 4096 passes K * dim <= 4096 but its z kernel would need 96 KiB of LDS
    dummy = (C.c_float * 4)()
    g = B.GmmConfig(100, 1, 4096, 1.0, 10.0, 1.0, 0.0, 0.0, 1, 0, None, 0)
    assert L.augur_gmm_create(C.byref(g), dummy, C.byref(h)) == B.ERR_INVALID_ARG
    assert "K * (dim + 2)" in B.last_error()
    for fn in (L.augur_lda_sync, L.augur_gmm_sync, L.augur_lda_step_finish, L.augur_gmm_step_finish):
        assert fn(None) == B.ERR_INVALID_ARG
    assert L.augur_lda_sweep(None, 1) == B.ERR_INVALID_ARG
    L.augur_lda_destroy(None)
    L.augur_gmm_destroy(None)


def test_parity_topic_counts_reach_every_sampler_instance():
    assert {P.quad_stripes(K) for K in P.QUAD_TOPIC_COUNTS} == set(range(1, 17))
    assert max(P.QUAD_TOPIC_COUNTS) == 256 < min(P.ROW_TOPIC_COUNTS)
    assert {P.row_stripes(K) for K in P.ROW_TOPIC_COUNTS} == set(range(5, 17))

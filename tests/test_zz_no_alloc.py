"""The entry point that allocates nothing (augur_lda_loglik_static) against the handle-based
augur_lda_loglik, through the C ABI, on two calls in a row, the second with a smaller input."""
import ctypes as C

import numpy as np
import pytest

from paper_1312_3613_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


def _handle_and_arrays(B, torch, D, V, K, mean_len, seed, sweeps):
    cfg = dict(synth.LDA_CONFIGS["tiny"], D=D, V=V, K=K, mean_len=mean_len)
    c = synth.lda_corpus(**cfg)
    lens = c["doc_len"].copy()
    g = B.LDA(D, V, K, 0.1, 0.01, seed, lens, c["w"])
    g.sweep(sweeps)
    z, th, ph, _ = g.get_state()
    want = g.loglik()
    g.close()
    ld = (K + 3) // 4 * 4 + 4           # a stride wider than the handle's own, padding poisoned
    dev = torch.device("cuda", 0)
    th_d = torch.full((D, ld), float("nan"), dtype=torch.float32, device=dev)
    ph_d = torch.full((V, ld), float("nan"), dtype=torch.float32, device=dev)
    th_d[:, :K] = torch.as_tensor(th)
    ph_d[:, :K] = torch.as_tensor(ph)
    arrays = dict(doc_len=torch.as_tensor(lens).to(dev), w=torch.as_tensor(c["w"]).to(dev),
                  z=torch.as_tensor(z).to(dev), theta=th_d, phi=ph_d)
    return arrays, ld, want


def test_static_loglik_matches_the_handle_call_twice_in_a_row():
    import torch
    from paper_1312_3613_amd import binding as B
    B.lib()
    dev = torch.device("cuda", 0)
    out = torch.zeros(2, dtype=torch.float64, device=dev)
    stream = torch.cuda.Stream()
    cases = [(700, 900, 50, 80, 5, 2), (90, 120, 7, 30, 6, 1)]     # the second is smaller
    prepared = [_handle_and_arrays(B, torch, *c) for c in cases]
    torch.cuda.synchronize()
    for (D, V, K, _, _, _), (a, ld, want) in zip(cases, prepared):
        out.fill_(-1.0)
        torch.cuda.synchronize()
        B.lda_loglik_static(D, V, K, ld, 0.1, 0.01, a["doc_len"], a["w"], a["z"], a["theta"], a["phi"],
                            out, stream=stream)
        stream.synchronize()
        got = out.cpu().numpy()
        assert np.isfinite(got).all()
        for g, w_ in zip(got, want):
            assert abs(g - w_) <= P.REAL_RTOL * abs(w_), (got, want)
            assert abs(g - w_) <= 1e-9 * abs(w_), (got, want)   # same kernels, same order: far closer


def test_static_loglik_rejects_sizes_beyond_its_scratch():
    import torch
    from paper_1312_3613_amd import binding as B
    L = B.lib()
    dev = torch.device("cuda", 0)
    t = torch.zeros(64, dtype=torch.float32, device=dev)
    i = torch.zeros(64, dtype=torch.int32, device=dev)
    out = torch.zeros(2, dtype=torch.float64, device=dev)

    def call(D, V, K, ld):
        a = B.LdaStaticArgs(D, V, K, ld, 0.1, 0.1, i.data_ptr(), i.data_ptr(), i.data_ptr(),
                            t.data_ptr(), t.data_ptr(), 0, None)
        return L.augur_lda_loglik_static(C.byref(a), out.data_ptr())

    assert call((1 << 20) + 1, 4, 4, 4) == B.ERR_INVALID_ARG and "1048576" in B.last_error()
    assert call(4, 4, 2000, 2000) == B.ERR_INVALID_ARG
    assert call(4, 4, 5, 6) == B.ERR_INVALID_ARG          # stride not a multiple of 4
    assert call(4, 4, 5, 4) == B.ERR_INVALID_ARG          # stride below K
    assert call(2, 4, 4, 4) == B.OK                       # and a valid call still works afterwards
    torch.cuda.synchronize()

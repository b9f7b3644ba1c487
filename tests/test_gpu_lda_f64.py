"""GPU parity of the LDA sweep with theta and phi held in fp64 (the precision of the paper's own
experiments, Sect. 5): the HIP path (through the C ABI) against the oracle's fp64 state mode,
element by element, from the same state and the same random streams.  z must agree except where
the threshold lies within 1e-12 relative of a boundary of the running sums (the two sides add
the same fp64 products in different orders); theta, phi and the log densities within 1e-10
relative (their exp and log routines differ in the last bits)."""
import ctypes as C

import numpy as np
import pytest

from oracle import oracle as O
from paper_1312_3613_amd import synth
from tests import parity as P
from tests.test_gpu_lda import ragged_corpus, np_, _oracle_z_on_ranges

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1312_3613_amd import binding
    binding.lib()
    return binding


def make_pair(B, D, V, K, alpha, beta, seed, lens, w, **kw):
    g = B.LDA(D, V, K, alpha, beta, seed, lens, w, state_f64=True, **kw)
    o = O.OracleLDA(D, V, K, alpha, beta, seed, lens, w, f64=True)
    return g, o


def close64(got, want, what):
    got = np_(got)
    assert got.dtype == np.float64
    P.assert_real_close(got, want, what, rtol=P.REAL_RTOL_F64, floor=P.DBL_MIN)


def lockstep_sweep(g, o, check_loglik=False):
    """One sweep, both sides restarted from the oracle's state before every step."""
    t = o.sweep_index + 1
    theta0, phi0 = o.theta.copy(), o.phi.copy()
    g.set_state(z=o.z, theta=o.theta, phi=o.phi, sweep=o.sweep_index)
    g.step_sample_z(); o.step_sample_z()
    zg = np_(g.get_state(theta=False, phi=False)[0])
    nm = P.assert_z_lda(zg, o.z, o.doc_off, o.w, theta0, phi0, o.seed, t, f64=True,
                        boundary_rtol=P.Z_BOUNDARY_RTOL_F64)
    g.set_state(z=o.z)
    g.step_count(); o.step_count()
    n_dk, n_wk = (np_(a) for a in g.get_counts())
    assert np.array_equal(n_dk, o.n_dk) and np.array_equal(n_wk, o.n_wk)
    g.step_resample_theta(); o.step_resample_theta()
    g.step_resample_phi(); o.step_resample_phi()
    _, th, ph, _ = g.get_state(z=False)
    close64(th, o.theta, "theta")
    close64(ph, o.phi, "phi")
    g.step_finish(); o.step_finish()
    if check_loglik:
        g.set_state(theta=o.theta, phi=o.phi)
        lj, lm = g.loglik()
        olj, olm = o.loglik()
        assert abs(lj - olj) <= P.REAL_RTOL_F64 * abs(olj) and abs(lm - olm) <= P.REAL_RTOL_F64 * abs(olm)
    return nm


def test_initial_state_and_twenty_lockstep_sweeps(B):
    cfg = synth.LDA_CONFIGS["tiny"]
    c = synth.lda_corpus(**cfg)
    g, o = make_pair(B, cfg["D"], cfg["V"], cfg["K"], cfg["alpha"], cfg["beta"], cfg["seed"],
                     c["doc_len"], c["w"])
    z, th, ph, sw = g.get_state()
    assert sw == 0 and np.array_equal(z, o.z)
    close64(th, o.theta, "theta0")
    close64(ph, o.phi, "phi0")
    # stored values are doubles that no float holds: the state really is fp64
    assert (np_(th) != np_(th).astype(np.float32)).mean() > 0.9
    total = 0
    for s in range(cfg["sweeps"]):
        total += lockstep_sweep(g, o, check_loglik=(s % 5 == 4))
    assert total == 0, "fp64 running sums should not meet a boundary on so few tokens"
    assert g.get_degenerate() == 0 and o.degenerate == 0
    g.close()


def test_free_running_chain_stays_on_the_oracles(B):
    # with fp64 products a boundary decision is so rare that the two chains stay together for many
    # sweeps on a small corpus; theta and phi then agree to rounding after every sweep
    cfg = synth.LDA_CONFIGS["tiny"]
    c = synth.lda_corpus(**cfg)
    g, o = make_pair(B, cfg["D"], cfg["V"], cfg["K"], cfg["alpha"], cfg["beta"], cfg["seed"],
                     c["doc_len"], c["w"])
    g.sweep(10); o.sweep(10)
    z, th, ph, sw = g.get_state()
    assert sw == 10
    agree = (np_(z) == o.z).mean()
    print("fp64 free-running agreement after 10 sweeps", agree)
    assert agree > 0.9
    if agree == 1.0:
        # theta and phi of sweep t feed sweep t + 1's z only through comparisons, so that equal z
        # means the parameters are still one rounding apart, not ten
        close64(th, o.theta, "theta after 10 sweeps")
        close64(ph, o.phi, "phi after 10 sweeps")
    lj, lm = g.loglik()
    olj, olm = o.loglik()
    assert abs(lm - olm) < 0.02 * abs(olm)
    g.close()


@pytest.mark.parametrize("K", [1, 2, 7, 16, 20, 48, 65, 100, 200, 256, 257, 300, 500, 700, 1000, 1024])
def test_topic_counts_span_stripes_and_tails(B, K):
    D, V = 120, 300
    lens, w = ragged_corpus(D, V, K, seed=K, mean_len=100)
    assert w.size >= 10_000
    g, o = make_pair(B, D, V, K, 0.1, 0.01, 1000 + K, lens, w)
    assert np.array_equal(np_(g.get_state(theta=False, phi=False)[0]), o.z)
    for _ in range(2):
        lockstep_sweep(g, o, check_loglik=True)
    # the sweep entry point (document counts inside the z kernel, second stream) against the steps
    results = []
    g.set_state(z=o.z, theta=o.theta, phi=o.phi, sweep=o.sweep_index)
    g.sweep(1)
    results.append([np_(a).copy() for a in g.get_state()[:3] + g.get_counts()])
    g.set_state(z=o.z, theta=o.theta, phi=o.phi, sweep=o.sweep_index)
    g.step_sample_z(); g.step_count(); g.step_resample_theta(); g.step_resample_phi(); g.step_finish()
    results.append([np_(a).copy() for a in g.get_state()[:3] + g.get_counts()])
    for x, y in zip(*results):
        assert np.array_equal(x, y)
    g.close()


@pytest.mark.parametrize("K", [200, 700])
def test_dense_parameters_many_live_topics(B, K):
    D, V = 64, 500
    lens, w = ragged_corpus(D, V, K, seed=5, mean_len=300)
    g, o = make_pair(B, D, V, K, 1.0, 1.0, 77, lens, w)
    for _ in range(3):
        lockstep_sweep(g, o)
    g.close()


def test_edge_corpora(B):
    for lens, w, V, K in [([1], [2], 5, 3), ([0, 0, 0], [], 4, 3), ([3, 0, 2], [0, 0, 0, 0, 0], 1, 4)]:
        lens, w = np.array(lens, dtype=np.int32), np.array(w, dtype=np.int32)
        g, o = make_pair(B, len(lens), V, K, 0.5, 0.5, 3, lens, w)
        lockstep_sweep(g, o, check_loglik=w.size > 0)
        g.sweep(2); o.sweep(2)
        assert np.array_equal(np_(g.get_state(theta=False, phi=False)[0]), o.z)
        g.close()


def test_zero_mass_topics_and_degenerate_rows(B):
    D, V, K = 6, 50, 12
    lens, w = ragged_corpus(D, V, K, seed=9, lens=[40, 40, 40, 40, 40, 40])
    g, o = make_pair(B, D, V, K, 0.1, 0.1, 5, lens, w)
    theta = o.theta.copy()
    theta[:, 3] = 0.0
    theta[1, :] = 0.0
    theta[2, :] = np.nan
    o.set_state(theta=theta)
    g.set_state(z=o.z, theta=theta, phi=o.phi, sweep=o.sweep_index)
    g.step_sample_z(); o.step_sample_z()
    zg = np_(g.get_state(theta=False, phi=False)[0])
    assert np.array_equal(zg, o.z)
    live = np.r_[0:40, 120:240]
    assert (zg[live] != 3).all()
    assert g.get_degenerate() == 80 == o.degenerate
    g.close()


def test_values_below_the_fp32_range_keep_their_mass(B):
    # a document whose theta lies far below FLT_MIN everywhere: an fp32 state would have floored
    # or flushed it; in fp64 the conditional is the same as for theta scaled back up
    D, V, K = 4, 60, 24
    lens, w = ragged_corpus(D, V, K, seed=3, lens=[200, 200, 200, 200])
    g, o = make_pair(B, D, V, K, 0.1, 0.1, 8, lens, w)
    theta = o.theta.copy()
    theta[1] *= 1e-200
    o.set_state(theta=theta)
    g.set_state(z=o.z, theta=theta, phi=o.phi, sweep=o.sweep_index)
    g.step_sample_z(); o.step_sample_z()
    zg = np_(g.get_state(theta=False, phi=False)[0])
    assert np.array_equal(zg, o.z)
    assert g.get_degenerate() == 0 == o.degenerate
    # and scaling a document's theta does not change its draws (up to boundary cases)
    o2 = O.OracleLDA(D, V, K, 0.1, 0.1, 8, lens, w, f64=True)
    o2.step_sample_z()
    assert (o2.z[200:400] == o.z[200:400]).mean() > 0.99
    g.close()


@pytest.mark.parametrize("K", [20, 300])
def test_long_documents_are_cut_into_segments(B, K):
    lens = [5000, 3, 1025, 1021, 0, 2500, 1024, 1020, 7]
    D, V = len(lens), 400
    lens, w = ragged_corpus(D, V, K, seed=K + 1, lens=lens)
    g, o = make_pair(B, D, V, K, 0.1, 0.01, 500 + K, lens, w)
    for _ in range(2):
        lockstep_sweep(g, o, check_loglik=True)
    g2 = B.LDA(D, V, K, 0.1, 0.01, 500 + K, lens, w, state_f64=True)
    g2.sweep(3)
    g3 = B.LDA(D, V, K, 0.1, 0.01, 500 + K, lens, w, state_f64=True)
    for _ in range(3):
        g3.step_sample_z(); g3.step_count(); g3.step_resample_theta(); g3.step_resample_phi(); g3.step_finish()
    for x, y in zip(g2.get_state() + g2.get_counts(), g3.get_state() + g3.get_counts()):
        assert np.array_equal(np_(x), np_(y))
    for h in (g, g2, g3):
        h.close()


def test_resume_graph_replay_and_device_pointers(B):
    import torch
    cfg = dict(synth.LDA_CONFIGS["tiny"], D=60, V=200, K=20)
    c = synth.lda_corpus(**cfg)
    args = (cfg["D"], cfg["V"], cfg["K"], cfg["alpha"], cfg["beta"], 4242, c["doc_len"], c["w"])
    a, b = B.LDA(*args, state_f64=True), B.LDA(*args, state_f64=True)
    a.sweep(10)
    b.sweep(5)
    z, th, ph, sw = b.get_state()
    r = B.LDA(*args, state_f64=True)
    r.set_state(z, th, ph, sw)
    r.sweep(5)
    for x, y in zip(a.get_state(), r.get_state()):
        assert np.array_equal(x, y)
    assert a.loglik() == r.loglik()
    # on a stream of the caller's (sweeps replayed from a recorded graph) with device pointers
    stream = torch.cuda.Stream()
    dl = torch.from_numpy(c["doc_len"]).cuda()
    wd = torch.from_numpy(c["w"]).cuda()
    torch.cuda.synchronize()
    s = B.LDA(*args[:6], dl, wd, stream=stream, device_ptrs=True, state_f64=True)
    for _ in range(5):
        s.sweep(2)
    zs, ths, phs, sws = s.get_state()
    assert sws == 10 and ths.dtype == torch.float64
    for x, y in zip(a.get_state()[:3], (zs, ths, phs)):
        assert np.array_equal(x, np_(y))
    for h in (a, b, r, s):
        h.close()


def test_each_state_type_has_its_own_accessors(B):
    cfg = synth.LDA_CONFIGS["tiny"]
    c = synth.lda_corpus(**cfg)
    args = (cfg["D"], cfg["V"], cfg["K"], cfg["alpha"], cfg["beta"], 1, c["doc_len"], c["w"])
    g64, g32 = B.LDA(*args, state_f64=True), B.LDA(*args)
    L = B.lib()
    th32 = np.zeros((cfg["D"], cfg["K"]), dtype=np.float32)
    th64 = np.zeros((cfg["D"], cfg["K"]), dtype=np.float64)
    sw = C.c_int64()
    assert L.augur_lda_get_state(g64._h, None, th32.ctypes.data, None, C.byref(sw)) == B.ERR_INVALID_ARG
    assert "fp64" in B.last_error()
    assert L.augur_lda_get_state_f64(g32._h, None, th64.ctypes.data, None, C.byref(sw)) == B.ERR_INVALID_ARG
    assert L.augur_lda_set_state(g64._h, None, th32.ctypes.data, None, -1) == B.ERR_INVALID_ARG
    assert L.augur_lda_set_state_f64(g32._h, None, th64.ctypes.data, None, -1) == B.ERR_INVALID_ARG
    # z and the sweep index alone are served by either
    assert L.augur_lda_get_state(g64._h, None, None, None, C.byref(sw)) == B.OK and sw.value == 0
    with pytest.raises(B.AugurError):
        g64.probe_gather(1)
    # the two states hold the same draws, rounded to their own type
    t64, t32 = g64.get_state()[1], g32.get_state()[1]
    big = t64 > 1e-30
    assert np.allclose(t64[big], t32[big].astype(np.float64), rtol=1e-6)
    g64.close(); g32.close()


def test_medium_config_sample_z_and_counts(B):
    # the medium benchmark configuration (3M tokens, K = 100): one z step from the oracle's state
    cfg = synth.LDA_CONFIGS["medium"]
    c = synth.lda_corpus(**cfg)
    g, o = make_pair(B, cfg["D"], cfg["V"], cfg["K"], cfg["alpha"], cfg["beta"], cfg["seed"],
                     c["doc_len"], c["w"])
    nm = lockstep_sweep(g, o, check_loglik=True)
    print("medium fp64: z mismatches", nm)
    g.close()


def test_full_size_config_sampled_parity(B):
    """BASELINE's K=200 configuration (about 75M tokens) with the fp64 state, through sweep(): z of
    the sweep on ranges of documents the oracle redoes one by one, both count tables in full,
    theta on sampled ranges, phi in full."""
    from scipy import special
    cfg = synth.LDA_CONFIGS["large"]
    c = synth.lda_corpus(**cfg)
    D, V, K, N = cfg["D"], cfg["V"], cfg["K"], c["N"]
    alpha, beta, seed = float(np.float32(cfg["alpha"])), float(np.float32(cfg["beta"])), cfg["seed"]
    g = B.LDA(D, V, K, cfg["alpha"], cfg["beta"], seed, c["doc_len"], c["w"], state_f64=True)
    off = O.doc_offsets(c["doc_len"])
    g.sweep(1)
    _, theta, phi, sw = g.get_state(z=False)
    assert sw == 1 and theta.dtype == np.float64
    g.sweep(1)                                   # the sweep under test: index 2
    z1, th1, ph1, sw = g.get_state()
    assert sw == 2 and z1.min() >= 0 and z1.max() < K
    ranges = [(d0, d0 + 1000) for d0 in (0, D // 2 + 777, D - 1000)]
    checked = _oracle_z_on_ranges(c, off, theta, phi, seed, 2, z1, D, K, ranges, f64=True)
    print("fp64 large: z checked on", checked, "tokens")
    n_dk, n_wk = g.get_counts()
    o_dk, o_wk = O.lda_count(off, c["w"], z1, D, V, K)
    assert np.array_equal(n_dk, o_dk) and np.array_equal(n_wk, o_wk)
    del o_dk, o_wk
    for d0 in (0, 2 * D // 3, D - 2000):
        nd = np.ascontiguousarray(n_dk[d0:d0 + 2000])
        lg = O.gamma_log_draws((alpha + nd).ravel(), seed, first=d0 * K, sweep=2, stream=O.STREAM_THETA).reshape(2000, K)
        want = np.maximum(np.exp(lg - special.logsumexp(lg, axis=1, keepdims=True)), P.DBL_MIN)
        P.assert_real_close(th1[d0:d0 + 2000], want, "theta rows", rtol=P.REAL_RTOL_F64, floor=P.DBL_MIN)
    close64(ph1, O.lda_resample_phi(n_wk, beta, seed, 2, f64=True), "phi")
    g.close()

"""Pins of the oracle's fp64 state mode (theta and phi stored as doubles; the precision the
paper's experiments ran in, Sect. 5).  The fp32-state functions are pinned in test_oracle_lda.py;
here the fp64 ones are tied to them where the two must agree exactly, and to enumeration, library
densities and invariants where doubles that no float represents come in."""
import itertools

import numpy as np
import pytest
from scipy import special, stats

from oracle import oracle as O
from paper_1312_3613_amd import synth

DBL_MIN = float(np.finfo(np.float64).tiny)
FLT_MIN = float(np.finfo(np.float32).tiny)


def _small_model_f64(seed=0, D=2, V=3, K=3, lens=(3, 2)):
    rng = np.random.default_rng(seed)
    theta = rng.dirichlet(np.ones(K), size=D)                 # doubles that no float represents
    phi = rng.dirichlet(np.ones(V), size=K).T.copy()          # [V][K]
    w = rng.integers(0, V, size=sum(lens)).astype(np.int32)
    return theta, phi, w, np.array(lens, dtype=np.int32)


def test_f64_conditional_equals_bruteforce_enumeration():
    theta, phi, w, lens = _small_model_f64()
    assert not np.array_equal(theta, theta.astype(np.float32))          # really fp64 inputs
    K, N = theta.shape[1], w.size
    doc = np.repeat(np.arange(len(lens)), lens)
    joint = {}
    for zz in itertools.product(range(K), repeat=N):
        joint[zz] = np.prod([theta[doc[i], zz[i]] * phi[w[i], zz[i]] for i in range(N)])
    for i in range(N):
        cdf, _ = O.lda_token_cdf(theta[doc[i]], phi[w[i]], seed=1, token=i, sweep=1, f64=True)
        p = np.diff(np.concatenate([[0.0], cdf])) / cdf[-1]
        for rest in itertools.product(range(K), repeat=N - 1):
            ws = np.array([joint[rest[:i] + (k,) + rest[i:]] for k in range(K)])
            assert np.allclose(ws / ws.sum(), p, rtol=1e-12, atol=0)
    # the fp32 functions see other numbers: rounding the state to float moves the conditional
    cdf32, _ = O.lda_token_cdf(theta[0], phi[w[0]], seed=1, token=0, sweep=1)
    cdf64, _ = O.lda_token_cdf(theta[0], phi[w[0]], seed=1, token=0, sweep=1, f64=True)
    assert not np.array_equal(cdf32, cdf64) and np.allclose(cdf32, cdf64, rtol=1e-6)


def test_f64_draws_follow_the_conditional():
    theta, phi, w, lens = _small_model_f64(seed=1)
    K = theta.shape[1]
    off = O.doc_offsets(lens)
    doc = np.repeat(np.arange(len(lens)), lens)
    T = 30_000
    zs = np.stack([O.lda_sample_z(off, w, theta, phi, seed=77, sweep=s, f64=True)[0] for s in range(1, T + 1)])
    for i in range(w.size):
        p = theta[doc[i]] * phi[w[i]]
        p /= p.sum()
        assert stats.chisquare(np.bincount(zs[:, i], minlength=K), p * T).pvalue > 1e-4


def test_f64_functions_equal_the_f32_ones_on_float_states():
    """A state whose doubles are floats: both modes form the same products and sums in fp64, so z,
    the running sums and the log densities must agree to the last bit."""
    cfg = dict(synth.LDA_CONFIGS["tiny"], D=30, V=80, K=7, mean_len=40)
    c = synth.lda_corpus(**cfg)
    a = O.OracleLDA(cfg["D"], cfg["V"], cfg["K"], 0.1, 0.01, 9, c["doc_len"], c["w"])
    a.sweep(2)
    th64, ph64 = a.theta.astype(np.float64), a.phi.astype(np.float64)
    for sweep in (3, 4):
        z32, d32 = O.lda_sample_z(a.doc_off, a.w, a.theta, a.phi, a.seed, sweep)
        z64, d64 = O.lda_sample_z(a.doc_off, a.w, th64, ph64, a.seed, sweep, f64=True)
        assert np.array_equal(z32, z64) and d32 == d64 == 0
    assert O.lda_loglik(a.doc_off, a.w, a.z, a.theta, a.phi, a.alpha, a.beta) == \
        O.lda_loglik(a.doc_off, a.w, a.z, th64, ph64, a.alpha, a.beta, f64=True)
    c32, t32 = O.lda_token_cdf(a.theta[3], a.phi[5], a.seed, 11, 2)
    c64, t64 = O.lda_token_cdf(th64[3], ph64[5], a.seed, 11, 2, f64=True)
    assert np.array_equal(c32, c64) and t32 == t64


def test_f64_dirichlet_draws_round_to_the_f32_ones_and_keep_what_f32_floors():
    rng = np.random.default_rng(3)
    n_dk = rng.integers(0, 30, size=(200, 12)).astype(np.int32)
    n_dk[rng.random(n_dk.shape) < 0.6] = 0
    for alpha in (0.05, 0.5, 3.0):
        t32 = O.lda_resample_theta(n_dk, alpha, seed=5, sweep=2)
        t64 = O.lda_resample_theta(n_dk, alpha, seed=5, sweep=2, f64=True)
        assert t64.dtype == np.float64 and t64.min() >= DBL_MIN
        above = t64 >= FLT_MIN
        assert np.array_equal(t64[above].astype(np.float32), t32[above])        # the same Gamma draws
        assert (t32[~above] == np.float32(FLT_MIN)).all()                       # what fp32 floors, fp64 keeps
        assert np.abs(t64.sum(axis=1) - 1.0).max() < 1e-12
    assert (~(O.lda_resample_theta(n_dk, 0.05, seed=5, sweep=2, f64=True) >= FLT_MIN)).any()
    n_wk = rng.integers(0, 5, size=(300, 6)).astype(np.int32)
    p32 = O.lda_resample_phi(n_wk, 0.01, seed=5, sweep=2)
    p64 = O.lda_resample_phi(n_wk, 0.01, seed=5, sweep=2, f64=True)
    above = p64 >= FLT_MIN
    assert np.array_equal(p64[above].astype(np.float32), p32[above])
    assert np.abs(p64.sum(axis=0) - 1.0).max() < 1e-12                          # normalised over words


def test_f64_floor_is_the_smallest_normal_double():
    # shapes so small that a draw underflows a double: Gamma(1e-4) has P(g < 1e-320) = 1e-320^1e-4 = 0.93
    n = np.zeros((50, 8), dtype=np.int32)
    n[:, 0] = 1000
    t64 = O.lda_resample_theta(n, 1e-4, seed=8, sweep=1, f64=True)
    assert t64.min() == DBL_MIN and np.isfinite(np.log(t64)).all()


def test_f64_log_joint_against_term_by_term_evaluation():
    cfg = dict(synth.LDA_CONFIGS["tiny"], D=12, V=30, K=4, mean_len=9)
    c = synth.lda_corpus(**cfg)
    D, V, K = cfg["D"], cfg["V"], cfg["K"]
    m = O.OracleLDA(D, V, K, cfg["alpha"], cfg["beta"], seed=4, doc_len=c["doc_len"], w=c["w"], f64=True)
    m.sweep(3)
    assert m.theta.dtype == np.float64 and not np.array_equal(m.theta, m.theta.astype(np.float32))
    lj, lm = m.loglik()
    a, b = m.alpha, m.beta
    th, ph = m.theta, m.phi
    want = 0.0
    for k in range(K):
        want += special.gammaln(V * b) - V * special.gammaln(b) + ((b - 1) * np.log(ph[:, k])).sum()
    for d in range(D):
        want += special.gammaln(K * a) - K * special.gammaln(a) + ((a - 1) * np.log(th[d])).sum()
    i, marg = 0, 0.0
    for d in range(D):
        for _ in range(c["doc_len"][d]):
            want += np.log(th[d, m.z[i]]) + np.log(ph[m.w[i], m.z[i]])
            marg += np.log(th[d] @ ph[m.w[i]])
            i += 1
    assert abs(lj - want) < 1e-9 * abs(want) and abs(lm - marg) < 1e-9 * abs(marg)


def test_f64_sweep_is_the_steps_in_order_and_resumes():
    cfg = dict(synth.LDA_CONFIGS["tiny"], D=20, V=60, K=6, mean_len=25)
    c = synth.lda_corpus(**cfg)
    args = (cfg["D"], cfg["V"], cfg["K"], 0.1, 0.01, 21, c["doc_len"], c["w"])
    a, b = O.OracleLDA(*args, f64=True), O.OracleLDA(*args, f64=True)
    # initial state: the f32 mode's z and counts; theta, phi the same draws unrounded
    f = O.OracleLDA(*args)
    assert np.array_equal(a.z, f.z) and np.array_equal(a.n_wk, f.n_wk)
    big = a.theta >= FLT_MIN
    assert np.array_equal(a.theta[big].astype(np.float32), f.theta[big])
    a.sweep(3)
    for _ in range(3):
        b.step_sample_z(); b.step_count(); b.step_resample_theta(); b.step_resample_phi(); b.step_finish()
    for x, y in zip(a.get_state()[:3] + a.get_counts(), b.get_state()[:3] + b.get_counts()):
        assert np.array_equal(x, y)
    r = O.OracleLDA(*args, f64=True)
    r.set_state(*a.get_state())
    r.sweep(2); a.sweep(2)
    assert np.array_equal(r.z, a.z) and np.array_equal(r.phi, a.phi)
    # phi observed: phi and the word table stay
    phi0 = a.phi.copy()
    a.set_observed(phi=True)
    a.sweep(2)
    assert np.array_equal(a.phi, phi0) and (a.n_dk.sum(1) == c["doc_len"]).all()

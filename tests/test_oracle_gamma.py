"""Pins for the oracle's Gamma and Dirichlet draws: library CDFs (scipy), closed-form
moments, and the special cases of the Dirichlet-from-Gammas construction
(Sect. 4.3, Alg. 1; App. B, Alg. 2)."""
import numpy as np
import pytest
from scipy import special, stats

from oracle import oracle as O

FLT_MIN = float(np.finfo(np.float32).tiny)
SHAPES = [0.01, 0.05, 0.1, 0.5, 1.0, 2.5, 50.0, 5000.0]


@pytest.mark.parametrize("a", SHAPES)
def test_gamma_log_draws_match_gamma_cdf(a):
    n = 200_000
    lg, att, capped = O.gamma_log_draws(np.full(n, a), seed=5, first=1000, sweep=2,
                                        stream=O.STREAM_THETA, return_attempts=True)
    assert capped == 0 and np.isfinite(lg).all()
    # ln g has CDF P(a, e^y) (regularised lower incomplete gamma)
    ks = stats.kstest(lg, lambda y: special.gammainc(a, np.exp(y)))
    assert ks.pvalue > 1e-4, ks
    # E[ln g] = psi(a), Var[ln g] = psi'(a)
    se = np.sqrt(special.polygamma(1, a) / n)
    assert abs(lg.mean() - special.digamma(a)) < 5 * se
    if a >= 0.5:
        g = np.exp(lg)
        assert abs(g.mean() - a) < 5 * np.sqrt(a / n)
        # Var[g] = a; the variance of the sample variance uses the 4th central moment 3a^2+6a
        assert abs(g.var() - a) < 5 * np.sqrt((3 * a * a + 6 * a - a * a) / n)
    # acceptance: Marsaglia & Tsang report > 95 % for every shape
    assert att.min() >= 1 and att.mean() < 1.06


def test_gamma_streams_independent():
    n = 100_000
    a = np.full(n, 0.7)
    x = O.gamma_log_draws(a, seed=1, first=0, sweep=1, stream=O.STREAM_THETA)
    for kw in [dict(seed=2, first=0, sweep=1, stream=O.STREAM_THETA),
               dict(seed=1, first=n, sweep=1, stream=O.STREAM_THETA),
               dict(seed=1, first=0, sweep=2, stream=O.STREAM_THETA),
               dict(seed=1, first=0, sweep=1, stream=O.STREAM_PHI)]:
        y = O.gamma_log_draws(a, **kw)
        assert abs(np.corrcoef(x, y)[0, 1]) < 5 / np.sqrt(n)
    assert (O.gamma_log_draws(a, seed=1, first=0, sweep=1, stream=O.STREAM_THETA) == x).all()


def test_gamma_boost_uses_shape_plus_one():
    # a < 1: ln g = ln Gamma(a+1)-draw + ln(U')/a with U' from word 3 of the accepted block
    a, seed, idx, sweep = 0.3, 9, 77, 4
    lg, att, _ = O.gamma_log_draws([a], seed, idx, sweep, O.STREAM_PHI, return_attempts=True)
    blk = O.random_block(seed, idx, sweep, O.STREAM_PHI, int(att[0]) - 1)
    lg1 = O.gamma_log_draws([a + 1.0], seed, idx, sweep, O.STREAM_PHI)
    assert abs(lg[0] - (lg1[0] + np.log(O.uniform32(blk[3])) / a)) < 1e-12


def test_squeeze_never_changes_a_draw():
    # The squeeze U < 1 - 0.0331 x^4 is only a shortcut: it lies inside the region of the exact
    # test (Marsaglia & Tsang 2000, Sect. 4), so a sampler that applies the exact test alone to
    # the same random blocks must accept at the same attempt and return the same value.
    n, seed, sweep = 4000, 21, 3
    for a in (0.02, 0.6, 1.0, 7.5, 300.0):
        lg, att, capped = O.gamma_log_draws(np.full(n, a), seed, 0, sweep, O.STREAM_THETA,
                                            return_attempts=True)
        assert capped == 0
        a1 = a + 1.0 if a < 1.0 else a
        d = a1 - 1.0 / 3.0
        c = 1.0 / np.sqrt(9.0 * d)
        squeeze_hits = 0
        for i in range(n):
            for j in range(64):
                r = O.random_block(seed, i, sweep, O.STREAM_THETA, j)
                x = np.sqrt(-2.0 * np.log(O.uniform32(r[0]))) * np.cos(2.0 * np.pi * O.uniform32(r[1]))
                t = 1.0 + c * x
                if t <= 0.0:
                    continue
                v, U = t ** 3, O.uniform32(r[2])
                squeeze_hits += U < 1.0 - 0.0331 * x ** 4
                if np.log(U) < 0.5 * x * x + d * (1.0 - v + np.log(v)):
                    break
            want = np.log(d) + np.log(v) + (np.log(O.uniform32(r[3])) / a if a < 1.0 else 0.0)
            assert att[i] == j + 1, (a, i)
            assert abs(lg[i] - want) <= 1e-12 * max(1.0, abs(want)), (a, i)
        assert squeeze_hits > 0.9 * n          # the shortcut is the common path


def test_dirichlet_rows_moments_and_simplex():
    D, K, alpha = 60_000, 4, 0.1
    c = np.array([0, 3, 1, 10], dtype=np.int32)
    theta = O.lda_resample_theta(np.tile(c, (D, 1)), alpha, seed=3, sweep=6).astype(np.float64)
    assert np.abs(theta.sum(axis=1) - 1).max() < 1e-6
    assert theta.min() >= FLT_MIN
    a = alpha + c
    a0 = a.sum()
    mean, var = a / a0, a * (a0 - a) / (a0 * a0 * (a0 + 1))
    assert (np.abs(theta.mean(axis=0) - mean) < 5 * np.sqrt(var / D)).all()
    assert (np.abs(theta.var(axis=0) - var) < 0.05 * var + 1e-6).all()
    # marginal of one coordinate is Beta(a_k, a0 - a_k)
    for k in (1, 3):
        assert stats.kstest(theta[:, k], "beta", args=(a[k], a0 - a[k])).pvalue > 1e-4
    # covariance of two coordinates: -a_i a_j / (a0^2 (a0+1))
    cov = np.cov(theta[:, 1], theta[:, 3])[0, 1]
    want = -a[1] * a[3] / (a0 * a0 * (a0 + 1))
    assert abs(cov - want) < 0.1 * abs(want)


def test_dirichlet_special_cases():
    # K = 1: theta is identically 1
    th = O.lda_resample_theta(np.array([[5], [0]], dtype=np.int32), 0.01, seed=1, sweep=1)
    assert (th == 1.0).all()
    # all counts zero (an empty document): a draw from the prior; K = 2 -> Beta(alpha, alpha)
    D, alpha = 50_000, 0.5
    th = O.lda_resample_theta(np.zeros((D, 2), dtype=np.int32), alpha, seed=2, sweep=1)
    assert stats.kstest(th[:, 0].astype(np.float64), "beta", args=(alpha, alpha)).pvalue > 1e-4
    # tiny concentration: entries underflow fp32 but are floored at FLT_MIN, rows still sum to 1
    th = O.lda_resample_theta(np.zeros((2000, 8), dtype=np.int32), 0.001, seed=3, sweep=1)
    assert th.min() == np.float32(FLT_MIN)
    assert np.abs(th.astype(np.float64).sum(axis=1) - 1).max() < 1e-6
    assert np.isfinite(np.log(th.astype(np.float64))).all()


def test_phi_columns_are_dirichlet_over_words():
    # phi is [V][K]; topic k's distribution is column k, Dirichlet(beta + n_wk[:, k])
    V, K, beta = 5, 3, 0.2
    n_wk = np.array([[4, 0, 1], [0, 0, 2], [1, 7, 0], [0, 0, 0], [2, 1, 1]], dtype=np.int32)
    T = 20_000
    draws = np.stack([O.lda_resample_phi(n_wk, beta, seed=8, sweep=s) for s in range(T)]).astype(np.float64)
    assert np.abs(draws.sum(axis=1) - 1).max() < 1e-6          # each column sums to 1 over words
    a = beta + n_wk
    a0 = a.sum(axis=0, keepdims=True)
    mean, var = a / a0, a * (a0 - a) / (a0 * a0 * (a0 + 1))
    assert (np.abs(draws.mean(axis=0) - mean) < 5 * np.sqrt(var / T)).all()
    assert stats.kstest(draws[:, 2, 1], "beta", args=(a[2, 1], a0[0, 1] - a[2, 1])).pvalue > 1e-4
    # variable index of entry (v,k) is v*K+k on the phi stream
    lg = O.gamma_log_draws(a.ravel(), seed=8, first=0, sweep=5, stream=O.STREAM_PHI).reshape(V, K)
    want = np.exp(lg - special.logsumexp(lg, axis=0, keepdims=True))
    got = O.lda_resample_phi(n_wk, beta, seed=8, sweep=5)
    assert np.allclose(got, want, rtol=1e-6, atol=0)

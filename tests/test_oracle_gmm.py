"""Pins for the oracle's Gaussian-mixture sweep (supplementary Gaussian mixture model, in the
known-covariance variant): library densities for the z conditional, library sums for the
statistics, the textbook Normal-Normal posterior, Dirichlet moments, an independent log joint,
recovery of the generating means, determinism."""
import numpy as np
from scipy import special, stats

from oracle import oracle as O
from paper_1312_3613_amd import synth


def _toy(seed=0, N=6, dim=3, K=4):
    rng = np.random.default_rng(seed)
    mu = rng.normal(0, 2, size=(K, dim)).astype(np.float32)
    pi = rng.dirichlet(np.ones(K)).astype(np.float32)
    x = rng.normal(0, 2, size=(N, dim)).astype(np.float32)
    return x, pi, mu


def test_z_conditional_matches_library_densities():
    x, pi, mu = _toy()
    sigma = 1.5
    for i in range(x.shape[0]):
        cdf, t = O.gmm_point_cdf(x[i], pi, mu, sigma, seed=3, point=i, sweep=2)
        p = np.diff(np.concatenate([[0.0], cdf])) / cdf[-1]
        logw = np.log(pi.astype(np.float64)) + np.array(
            [stats.multivariate_normal.logpdf(x[i].astype(np.float64), mu[k].astype(np.float64),
                                              sigma ** 2 * np.eye(x.shape[1])) for k in range(pi.size)])
        want = np.exp(logw - special.logsumexp(logw))
        assert np.allclose(p, want, rtol=1e-10, atol=1e-300)
        assert t == O.datum_uniforms(3, i, 1, 2, O.STREAM_Z)[0] * cdf[-1]


def test_z_draws_follow_conditional():
    x, pi, mu = _toy(seed=1, N=3)
    sigma, T, K = 2.0, 30_000, pi.size
    zs = np.stack([O.gmm_sample_z(x, pi, mu, sigma, seed=10, sweep=s)[0] for s in range(1, T + 1)])
    for i in range(x.shape[0]):
        cdf, _ = O.gmm_point_cdf(x[i], pi, mu, sigma, seed=10, point=i, sweep=1)
        p = np.diff(np.concatenate([[0.0], cdf])) / cdf[-1]
        keep = p * T > 5
        obs = np.bincount(zs[:, i], minlength=K)
        assert obs[~keep].sum() <= 30
        assert stats.chisquare(obs[keep], p[keep] / p[keep].sum() * obs[keep].sum()).pvalue > 1e-4
    z, _ = O.gmm_sample_z(x, pi, mu, sigma, seed=10, sweep=7)
    for i in range(x.shape[0]):
        cdf, t = O.gmm_point_cdf(x[i], pi, mu, sigma, seed=10, point=i, sweep=7)
        assert z[i] == int((cdf <= t).sum())


def test_stats_match_library_sums():
    d = synth.gmm_points(N=5000, dim=8, K=16, seed=1)
    z = O.lda_init_z(5000, 16, seed=4)
    n_k, s_k = O.gmm_stats(d["x"], z, 16)
    assert (n_k == np.bincount(z, minlength=16)).all()
    want = np.zeros((16, 8))
    np.add.at(want, z, d["x"].astype(np.float64))
    assert np.allclose(s_k, want, rtol=1e-12, atol=1e-9)


def test_single_component_is_textbook_normal_posterior():
    # K = 1: mu | x ~ N( sum(x)/sigma^2 / lambda, 1/lambda ), lambda = 1/prior_sd^2 + N/sigma^2
    rng = np.random.default_rng(2)
    N, dim, sigma, prior_sd = 50, 2, 2.0, 3.0
    x = rng.normal(1.0, sigma, size=(N, dim)).astype(np.float32)
    n_k = np.array([N], dtype=np.int32)
    s_k = x.astype(np.float64).sum(axis=0, keepdims=True)
    T = 20_000
    mus = np.stack([O.gmm_resample(n_k, s_k, 1.0, prior_sd, sigma, seed=6, sweep=s)[1][0] for s in range(T)])
    lam = 1 / prior_sd ** 2 + N / sigma ** 2
    mean = (s_k[0] / sigma ** 2) / lam
    # equivalent textbook form: N xbar / (N + sigma^2 / prior_sd^2)
    assert np.allclose(mean, N * x.astype(np.float64).mean(axis=0) / (N + sigma ** 2 / prior_sd ** 2))
    for j in range(dim):
        assert stats.kstest(mus[:, j], "norm", args=(mean[j], lam ** -0.5)).pvalue > 1e-4
    assert abs(np.corrcoef(mus[:, 0], mus[:, 1])[0, 1]) < 5 / np.sqrt(T)
    pi = O.gmm_resample(n_k, s_k, 1.0, prior_sd, sigma, seed=6, sweep=1)[0]
    assert pi[0] == 1.0
    # empty component: a draw from the prior
    mus0 = np.stack([O.gmm_resample(np.array([0], dtype=np.int32), np.zeros((1, 1)), 1.0, prior_sd, sigma,
                                    seed=7, sweep=s)[1][0, 0] for s in range(T)])
    assert stats.kstest(mus0, "norm", args=(0.0, prior_sd)).pvalue > 1e-4


def test_weights_are_dirichlet_posterior():
    n_k = np.array([5, 0, 12], dtype=np.int32)
    s_k = np.zeros((3, 1))
    alpha, T = 0.5, 20_000
    pis = np.stack([O.gmm_resample(n_k, s_k, alpha, 10.0, 1.0, seed=3, sweep=s)[0] for s in range(T)]).astype(np.float64)
    a = alpha + n_k
    a0 = a.sum()
    assert np.abs(pis.sum(axis=1) - 1).max() < 1e-6
    assert (np.abs(pis.mean(axis=0) - a / a0) < 5 * np.sqrt(a * (a0 - a) / (a0 ** 2 * (a0 + 1)) / T)).all()
    assert stats.kstest(pis[:, 1], "beta", args=(a[1], a0 - a[1])).pvalue > 1e-4


def test_log_joint_against_library_densities():
    d = synth.gmm_points(N=300, dim=4, K=3, seed=5)
    m = O.OracleGMM(3, 1.0, 10.0, 1.0, seed=1, x=d["x"])
    m.sweep(4)
    pi, mu, x = m.pi.astype(np.float64), m.mu.astype(np.float64), m.x.astype(np.float64)
    want = stats.dirichlet.logpdf(pi / pi.sum(), np.full(3, 1.0))
    want += stats.norm.logpdf(mu, 0.0, 10.0).sum()
    want += np.log(pi[m.z]).sum() + stats.norm.logpdf(x, mu[m.z], 1.0).sum()
    assert abs(m.loglik() - want) < 1e-9 * abs(want)
    # a non-trivial Dirichlet parameter exercises the (alpha-1) sum ln pi term
    lj = O.gmm_loglik(m.x, m.z, m.pi, m.mu, 2.5, 10.0, 1.0)
    want2 = want - stats.dirichlet.logpdf(pi / pi.sum(), np.full(3, 1.0)) + stats.dirichlet.logpdf(pi / pi.sum(), np.full(3, 2.5))
    assert abs(lj - want2) < 1e-6 * abs(want2)


def test_recovers_means_from_scrambled_truth():
    cfg = dict(synth.GMM_CONFIG, N=20_000)
    d = synth.gmm_points(return_truth=True, **cfg)
    K = cfg["K"]
    rng = np.random.default_rng(0)
    z0 = d["z"].copy()
    flip = rng.random(z0.size) < 0.2
    z0[flip] = rng.integers(0, K, size=int(flip.sum()))
    m = O.OracleGMM(K, cfg["alpha"], cfg["prior_sd"], cfg["sigma"], seed=11, x=d["x"])
    m.set_state(z=z0)
    m.step_resample(); m.step_finish()
    m.sweep(20)
    n_true = np.bincount(d["z"], minlength=K)
    big = n_true > 50
    err = np.abs(m.mu.astype(np.float64) - d["mu"])[big]
    assert (err < 4.0 / np.sqrt(n_true[big])[:, None] + 1e-3).all(), err.max()
    assert (np.abs(m.pi - d["pi"]) < 4 * np.sqrt(d["pi"] * (1 - d["pi"]) / z0.size) + 2e-3).all()
    assert (m.z == d["z"]).mean() > 0.97
    assert m.degenerate == 0


def test_gmm_determinism_and_steps():
    d = synth.gmm_points(N=2000, dim=8, K=16, seed=3)
    a = O.OracleGMM(16, 1.0, 10.0, 1.0, seed=5, x=d["x"])
    b = O.OracleGMM(16, 1.0, 10.0, 1.0, seed=5, x=d["x"])
    a.sweep(5)
    for _ in range(2):
        b.step_sample_z(); b.step_stats(); b.step_resample(); b.step_finish()
    z, pi, mu, t = b.get_state()
    r = O.OracleGMM(16, 1.0, 10.0, 1.0, seed=5, x=d["x"])
    r.set_state(z, pi, mu, t)
    r.sweep(3)
    for x, y in zip(a.get_state(), r.get_state()):
        assert np.array_equal(x, y)

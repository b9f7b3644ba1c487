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


# ---------------------------------------------- unknown component variances (the listing's model)
def test_uv_conditional_matches_library_densities():
    x, pi, mu = _toy(seed=3)
    var = np.array([0.5, 2.0, 1.0, 4.0], dtype=np.float32)
    for i in range(x.shape[0]):
        cdf, t = O.gmmuv_point_cdf(x[i], pi, mu, var, seed=3, point=i, sweep=2)
        p = np.diff(np.concatenate([[0.0], cdf])) / cdf[-1]
        logw = np.log(pi.astype(np.float64)) + np.array(
            [stats.multivariate_normal.logpdf(x[i].astype(np.float64), mu[k].astype(np.float64),
                                              float(var[k]) * np.eye(x.shape[1])) for k in range(pi.size)])
        # p comes from differences of a running sum of magnitude 1: absolute rounding of 1e-16
        assert np.allclose(p, np.exp(logw - special.logsumexp(logw)), rtol=1e-10, atol=1e-14)
    z, _ = O.gmmuv_sample_z(x, pi, mu, var, seed=3, sweep=2)
    for i in range(x.shape[0]):
        cdf, t = O.gmmuv_point_cdf(x[i], pi, mu, var, seed=3, point=i, sweep=2)
        assert z[i] == int((cdf <= t).sum())


def test_uv_variance_is_inverse_gamma_posterior_and_mean_uses_variance():
    rng = np.random.default_rng(4)
    N, dim, a0, b0, prior_sd = 40, 2, 1.0, 1.0, 3.0
    x = rng.normal(2.0, 1.5, size=(N, dim)).astype(np.float32)
    z = np.zeros(N, dtype=np.int32)
    n_k, s_k = O.gmm_stats(x, z, 1)
    var0 = np.array([2.5], dtype=np.float32)
    T = 20_000
    mus, vars_ = np.empty((T, dim)), np.empty(T)
    for s in range(T):
        _, mu, var = O.gmmuv_resample(x, z, n_k, s_k, var0, 1.0, prior_sd, a0, b0, seed=8, sweep=s)
        mus[s], vars_[s] = mu[0], var[0]
    lam = 1 / prior_sd ** 2 + N / 2.5
    mean = (s_k[0] / 2.5) / lam
    for j in range(dim):
        assert stats.kstest(mus[:, j], "norm", args=(mean[j], lam ** -0.5)).pvalue > 1e-4
    # var | mu ~ InvGamma(a0 + N dim / 2, b0 + SS(mu)/2): check through the pivot
    # (b0 + SS/2) / var ~ Gamma(shape), whatever mu was drawn
    ss = ((x.astype(np.float64)[None, :, :] - mus[:, None, :].astype(np.float32).astype(np.float64)) ** 2).sum(axis=(1, 2))
    pivot = (b0 + 0.5 * ss) / vars_
    assert stats.kstest(pivot, "gamma", args=(a0 + 0.5 * N * dim,)).pvalue > 1e-4
    # an empty component draws its variance from the prior InvGamma(a0, b0)
    e_n, e_s = np.array([0], dtype=np.int32), np.zeros((1, dim))
    v0 = np.array([O.gmmuv_resample(x[:0].reshape(0, dim), z[:0], e_n, e_s, var0, 1.0, prior_sd, 3.0, 2.0,
                                    seed=9, sweep=s)[2][0] for s in range(T)], dtype=np.float64)
    assert stats.kstest(v0, "invgamma", args=(3.0, 0, 2.0)).pvalue > 1e-4


def test_uv_log_joint_against_library_densities():
    d = synth.gmm_points(N=200, dim=3, K=3, seed=6)
    m = O.OracleGMMUV(3, 1.5, 10.0, 2.0, 3.0, seed=2, x=d["x"])
    m.sweep(3)
    pi, mu, var, x = (m.pi.astype(np.float64), m.mu.astype(np.float64), m.var.astype(np.float64),
                      m.x.astype(np.float64))
    want = stats.dirichlet.logpdf(pi / pi.sum(), np.full(3, 1.5))
    want += stats.norm.logpdf(mu, 0.0, 10.0).sum()
    want += stats.invgamma.logpdf(var, 2.0, scale=3.0).sum()
    want += np.log(pi[m.z]).sum() + stats.norm.logpdf(x, mu[m.z], np.sqrt(var[m.z])[:, None]).sum()
    assert abs(m.loglik() - want) < 1e-9 * abs(want)


def test_uv_recovers_means_and_variances():
    rng = np.random.default_rng(1)
    K, dim, N = 3, 2, 12_000
    mu_t = np.array([[-6.0, 0.0], [0.0, 5.0], [7.0, -3.0]])
    var_t = np.array([0.5, 2.0, 4.0])
    z_t = rng.integers(0, K, size=N)
    x = (mu_t[z_t] + np.sqrt(var_t[z_t])[:, None] * rng.standard_normal((N, dim))).astype(np.float32)
    m = O.OracleGMMUV(K, 1.0, 10.0, 1.0, 1.0, seed=5, x=x)
    z0 = z_t.copy().astype(np.int32)
    flip = rng.random(N) < 0.2
    z0[flip] = rng.integers(0, K, size=int(flip.sum()))
    m.set_state(z=z0)
    m.step_resample(); m.step_finish()
    m.sweep(30)
    assert np.abs(m.mu - mu_t).max() < 0.1
    assert np.abs(m.var / var_t - 1).max() < 0.1
    assert (m.z == z_t).mean() > 0.97 and m.degenerate == 0
    # determinism and the step-wise calls
    a = O.OracleGMMUV(K, 1.0, 10.0, 1.0, 1.0, seed=5, x=x)
    b = O.OracleGMMUV(K, 1.0, 10.0, 1.0, 1.0, seed=5, x=x)
    a.sweep(3)
    for _ in range(3):
        b.step_sample_z(); b.step_stats(); b.step_resample(); b.step_finish()
    assert np.array_equal(a.z, b.z) and np.array_equal(a.mu, b.mu) and np.array_equal(a.var, b.var)


def test_uv_initial_state_starts_from_the_prior_mean_variance():
    # var^0 = b0 / a0 for every component, then pi, mu and var from their conditionals with
    # sweep index 0 (the first sweep, index 1, draws from fresh random blocks)
    rng = np.random.default_rng(4)
    N, dim, K, a0, b0 = 600, 2, 3, 2.0, 3.0
    x = rng.normal(0.0, 4.0, size=(N, dim)).astype(np.float32)
    o = O.OracleGMMUV(K, 1.0, 10.0, a0, b0, 23, x)
    z0 = O.lda_init_z(N, K, seed=23)      # the mixture shares the init stream of z
    assert o.sweep_index == 0 and np.array_equal(o.z, z0)
    n_k, s_k = O.gmm_stats(x, z0, K)
    pi, mu, var = O.gmmuv_resample(x, z0, n_k, s_k, np.full(K, b0 / a0), 1.0, 10.0, a0, b0,
                                   seed=23, sweep=0)
    assert np.array_equal(o.pi, pi) and np.array_equal(o.mu, mu) and np.array_equal(o.var, var)
    # the starting variance matters: another one moves the means' conditional
    _, mu_other, _ = O.gmmuv_resample(x, z0, n_k, s_k, np.full(K, a0 / b0), 1.0, 10.0, a0, b0,
                                      seed=23, sweep=0)
    assert not np.array_equal(mu, mu_other)

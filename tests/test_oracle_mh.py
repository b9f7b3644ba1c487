"""Pins of the oracle's Metropolis-Hastings sampler on the multivariate regression model
(Sect. 4.1; Fig. "regression"; supplement, "Multivariate Regression")."""
import numpy as np
from scipy import stats

from oracle import oracle as O
from paper_1312_3613_amd import synth


def test_log_f_is_the_sum_of_the_programs_log_densities():
    d = synth.regression_data(N=57, K=3, seed=1, l=-2.0, u=3.0)
    theta = np.array([0.3, -1.2, 0.8, 0.5, 0.7])
    x, y = d["x"].astype(np.float64), d["y"].astype(np.float64)
    want = stats.norm.logpdf(theta[:4], 0.0, 10.0).sum()                # w and b
    want += stats.invgamma.logpdf(theta[4], 3.0, scale=1.0)             # tau
    want += stats.uniform.logpdf(x, -2.0, 5.0).sum()                    # x_n
    want += stats.norm.logpdf(y, x @ theta[:3] + theta[3], np.sqrt(theta[4])).sum()
    got = O.mhreg_logf(d["x"], d["y"], theta, 10.0, 3.0, 1.0, -2.0, 3.0)
    assert abs(got - want) < 1e-11 * abs(want)
    theta[4] = 0.0
    assert O.mhreg_logf(d["x"], d["y"], theta, 10.0, 3.0, 1.0, -2.0, 3.0) == -np.inf
    theta[4] = -1.0
    assert O.mhreg_logf(d["x"], d["y"], theta, 10.0, 3.0, 1.0, -2.0, 3.0) == -np.inf


def test_proposal_and_acceptance_use_their_own_streams():
    theta = np.array([1.0, 2.0, 3.0, 4.0])
    for t in (1, 2, 77):
        n = np.array([O.normals(11, e, 1, t, O.STREAM_MH_PROPOSAL)[0] for e in range(4)])
        assert np.array_equal(O.mhreg_propose(theta, 0.25, 11, t), theta + 0.25 * n)
        assert O.mhreg_accept_uniform(11, t) == O.uniform32(O.random_block(11, 0, t, O.STREAM_MH_ACCEPT)[0])
    # the steps of a chain are distinct draws, standard normal over steps
    z = np.array([(O.mhreg_propose(np.zeros(3), 1.0, 5, t)) for t in range(1, 4001)])
    for e in range(3):
        assert stats.kstest(z[:, e], "norm").pvalue > 1e-3
    assert abs(np.corrcoef(z[:, 0], z[:, 1])[0, 1]) < 0.06


def test_chain_follows_the_accept_rule_and_never_leaves_the_support():
    d = synth.regression_data(N=40, K=2, seed=3)
    m = O.OracleMHRegression(d["x"], d["y"], 10.0, 3.0, 1.0, -1.0, 1.0, step=0.4, seed=8,
                             theta0=[0.0, 0.0, 0.0, 0.2])
    prev, prev_lf = m.theta.copy(), m.logf
    tr = m.run(3000, trace=True)
    acc = 0
    for s, row in enumerate(tr):
        t = s + 1
        prop = O.mhreg_propose(prev, m.step, 8, t)
        lp = m.evaluate(prop)
        take = np.log(O.mhreg_accept_uniform(8, t)) < lp - prev_lf
        if take:
            prev, prev_lf = prop, lp
            acc += 1
        assert np.array_equal(row[:-1], prev) and row[-1] == prev_lf
    assert acc == m.accepted and 0 < acc < 3000
    assert (tr[:, 3] > 0).all()                 # tau
    # with step 0.4 around tau = 0.2 many proposals have tau <= 0: all refused
    assert acc < 2500


def test_chain_targets_the_posterior_computed_by_quadrature():
    # one predictor: the posterior of (w, b, tau) on a grid.  Given tau the posterior of (w, b) is
    # Gaussian, so only tau needs a grid: E[.] = sum over tau of p(tau | data) E[. | tau].
    d = synth.regression_data(N=12, K=1, seed=4, noise_var=0.5)
    x, y = d["x"].astype(np.float64), d["y"].astype(np.float64)
    X = np.column_stack([x[:, 0], np.ones(12)])
    prior_sd, a0, b0 = 3.0, 3.0, 1.0
    taus = np.exp(np.linspace(np.log(0.02), np.log(40.0), 4000))
    logp, means = np.zeros(taus.size), np.zeros((taus.size, 2))
    for i, tau in enumerate(taus):
        P = X.T @ X / tau + np.eye(2) / prior_sd ** 2            # posterior precision of (w, b)
        mu = np.linalg.solve(P, X.T @ y / tau)
        # marginal likelihood of y given tau (Gaussian integral), times the prior of tau
        S = tau * np.eye(12) + prior_sd ** 2 * X @ X.T
        logp[i] = stats.multivariate_normal.logpdf(y, np.zeros(12), S) + stats.invgamma.logpdf(tau, a0, scale=b0)
        means[i] = mu
    wt = np.exp(logp - logp.max()) * taus                          # d tau = tau d ln tau
    wt /= wt.sum()
    want = np.array([wt @ means[:, 0], wt @ means[:, 1], wt @ taus])
    m = O.OracleMHRegression(d["x"], d["y"], prior_sd, a0, b0, -1.0, 1.0, step=0.35, seed=21)
    m.run(5_000)
    tr = m.run(400_000, trace=True)[:, :3]
    got = tr.mean(axis=0)
    bm = tr.reshape(100, 4000, 3).mean(axis=1)                     # batch means
    se = bm.std(axis=0, ddof=1) / np.sqrt(100)
    assert (np.abs(got - want) < 4.5 * se).all(), (got, want, se)
    assert (se < 0.05 * np.maximum(np.abs(want), 0.2)).all()       # the test has resolving power


def test_recovers_generating_parameters_and_is_deterministic():
    d = synth.regression_data(N=3000, K=4, seed=6, return_truth=True)
    a = O.OracleMHRegression(d["x"], d["y"], 10.0, 3.0, 1.0, -1.0, 1.0, step=0.01, seed=2)
    a.run(30_000)
    tr = a.run(20_000, trace=True)
    est = tr[:, :6].mean(axis=0)
    assert np.abs(est[:4] - d["w"]).max() < 0.08 and abs(est[4] - d["b"]) < 0.05
    assert abs(est[5] / d["tau"] - 1) < 0.15
    b = O.OracleMHRegression(d["x"], d["y"], 10.0, 3.0, 1.0, -1.0, 1.0, step=0.01, seed=2)
    b.run(25_000); b.run(25_000)
    assert np.array_equal(a.theta, b.theta) and a.logf == b.logf and a.accepted == b.accepted

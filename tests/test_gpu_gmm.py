"""GPU parity of the Gaussian-mixture sweep against the oracle, step by step from a shared state."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_1312_3613_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1312_3613_amd import binding
    binding.lib()
    return binding


def lockstep(g, o, check_loglik=True):
    t = o.sweep_index + 1
    pi0, mu0 = o.pi.copy(), o.mu.copy()
    g.set_state(z=o.z, pi=o.pi, mu=o.mu, sweep=o.sweep_index)
    g.step_sample_z(); o.step_sample_z()
    zg = g.get_state()[0]
    nm = P.assert_z_gmm(zg, o.z, o.x, pi0, mu0, o.sigma, o.seed, t)
    g.set_state(z=o.z)
    g.step_stats(); o.step_stats()
    n_k, s_k = g.get_stats()
    assert np.array_equal(n_k, o.n_k)
    assert np.allclose(s_k, o.s_k, rtol=1e-12, atol=1e-9)
    g.step_resample(); o.step_resample()
    _, pi, mu, _ = g.get_state()
    P.assert_real_close(pi, o.pi, "pi")
    lam = 1.0 / o.prior_sd ** 2 + o.n_k / o.sigma ** 2
    err = np.abs(mu.astype(np.float64) - o.mu)
    assert (err <= P.REAL_RTOL * np.maximum(np.abs(o.mu), (lam ** -0.5)[:, None])).all()
    g.step_finish(); o.step_finish()
    if check_loglik:
        g.set_state(pi=o.pi, mu=o.mu)
        lj, olj = g.loglik(), o.loglik()
        assert abs(lj - olj) <= P.REAL_RTOL * abs(olj)
    return nm


def test_gmm_initial_state_and_lockstep(B):
    cfg = dict(synth.GMM_CONFIG, N=50_001)
    d = synth.gmm_points(**cfg)
    g = B.GMM(cfg["K"], cfg["alpha"], cfg["prior_sd"], cfg["sigma"], 21, d["x"])
    o = O.OracleGMM(cfg["K"], cfg["alpha"], cfg["prior_sd"], cfg["sigma"], 21, d["x"])
    z, pi, mu, sw = g.get_state()
    assert sw == 0 and np.array_equal(z, o.z)
    P.assert_real_close(pi, o.pi, "pi0")
    n_k, s_k = g.get_stats()
    assert np.array_equal(n_k, o.n_k) and np.allclose(s_k, o.s_k, rtol=1e-12, atol=1e-9)
    total = sum(lockstep(g, o) for _ in range(10))
    print("gmm: z mismatches over 10 sweeps", total)
    assert g.get_degenerate() == 0
    g.close()


@pytest.mark.parametrize("N,dim,K", [(1, 1, 1), (5, 3, 2), (1023, 8, 16), (1025, 2, 5), (4099, 14, 33)])
def test_gmm_shapes(B, N, dim, K):
    d = synth.gmm_points(N=N, dim=dim, K=K, seed=N + K)
    g = B.GMM(K, 1.0, 10.0, 1.0, 5, d["x"])
    o = O.OracleGMM(K, 1.0, 10.0, 1.0, 5, d["x"])
    for _ in range(3):
        lockstep(g, o)
    g.close()


def test_gmm_full_config_free_running_and_resume(B):
    cfg = synth.GMM_CONFIG
    d = synth.gmm_points(return_truth=True, **cfg)
    args = (cfg["K"], cfg["alpha"], cfg["prior_sd"], cfg["sigma"], cfg["seed"], d["x"])
    g, o = B.GMM(*args), O.OracleGMM(*args)
    lockstep(g, o)
    lockstep(g, o)
    a, b = B.GMM(*args), B.GMM(*args)
    a.sweep(6)
    b.sweep(3)
    st = b.get_state()
    r = B.GMM(*args)
    r.set_state(*st)
    r.sweep(3)
    for x, y in zip(a.get_state(), r.get_state()):
        assert np.array_equal(x, y)
    # statistics invariants at full size
    n_k, s_k = a.get_stats()
    assert n_k.sum() == cfg["N"]
    assert np.allclose(s_k.sum(0), d["x"].astype(np.float64).sum(0), rtol=1e-10)
    for h in (g, a, b, r):
        h.close()


def test_gmm_degenerate_and_errors(B):
    d = synth.gmm_points(N=100, dim=2, K=3, seed=1)
    g = B.GMM(3, 1.0, 10.0, 1.0, 5, d["x"])
    o = O.OracleGMM(3, 1.0, 10.0, 1.0, 5, d["x"])
    pi = np.array([np.nan, 0.5, 0.5], dtype=np.float32)
    o.set_state(pi=pi)
    g.set_state(z=o.z, pi=pi, mu=o.mu)
    g.step_sample_z(); o.step_sample_z()
    assert np.array_equal(g.get_state()[0], o.z)
    assert g.get_degenerate() == 100 == o.degenerate
    with pytest.raises(B.AugurError):
        g.set_state(z=np.full(100, 3, dtype=np.int32))
    with pytest.raises(B.AugurError):
        B.GMM(3, -1.0, 10.0, 1.0, 5, d["x"])
    g.close()


# ------------------------------------------------------- unknown component variances
def uv_points(N, dim, K, seed):
    """Points from components of different spreads (variance 0.25 .. 4)."""
    rng = np.random.default_rng(seed)
    mu = rng.normal(0.0, 10.0, size=(K, dim))
    var = 0.25 * 16.0 ** rng.random(K)
    z = rng.integers(0, K, size=N)
    return (mu[z] + np.sqrt(var[z])[:, None] * rng.standard_normal((N, dim))).astype(np.float32)


def lockstep_uv(g, o):
    t = o.sweep_index + 1
    pi0, mu0, var0 = o.pi.copy(), o.mu.copy(), o.var.copy()
    g.set_state(z=o.z, pi=o.pi, mu=o.mu, sweep=o.sweep_index)
    g.set_var(o.var)
    g.step_sample_z(); o.step_sample_z()
    zg = g.get_state()[0]
    nm = P.assert_z_gmmuv(zg, o.z, o.x, pi0, mu0, var0, o.seed, t)
    g.set_state(z=o.z)
    g.step_stats(); o.step_stats()
    n_k, s_k = g.get_stats()
    assert np.array_equal(n_k, o.n_k)
    assert np.allclose(s_k, o.s_k, rtol=1e-12, atol=1e-9)
    g.step_resample(); o.step_resample()
    _, pi, mu, _ = g.get_state()
    var = g.get_var()
    P.assert_real_close(pi, o.pi, "pi")
    lam = 1.0 / o.prior_sd ** 2 + o.n_k / var0.astype(np.float64)
    err = np.abs(mu.astype(np.float64) - o.mu)
    assert (err <= P.REAL_RTOL * np.maximum(np.abs(o.mu), (lam ** -0.5)[:, None])).all()
    # The variance draw depends on the fp32 mean just drawn; a mean that differs from the
    # oracle's in its last bit moves the sum of squares by far less than the tolerance (the
    # sum is stationary at the component's average, which the mean is close to).
    assert np.allclose(var, o.var, rtol=P.REAL_RTOL, atol=0)
    g.step_finish(); o.step_finish()
    g.set_state(pi=o.pi, mu=o.mu)
    g.set_var(o.var)
    lj, olj = g.loglik(), o.loglik()
    assert abs(lj - olj) <= P.REAL_RTOL * abs(olj)
    return nm


def test_gmm_unknown_variances_initial_state_and_lockstep(B):
    N, dim, K = 50_001, 8, 16
    x = uv_points(N, dim, K, seed=77)
    g = B.GMM(K, 1.0, 10.0, 1.0, 31, x, var_shape=2.0, var_scale=3.0)
    o = O.OracleGMMUV(K, 1.0, 10.0, 2.0, 3.0, 31, x)
    z, pi, mu, sw = g.get_state()
    assert sw == 0 and np.array_equal(z, o.z)
    P.assert_real_close(pi, o.pi, "pi0")
    assert np.allclose(g.get_var(), o.var, rtol=P.REAL_RTOL, atol=0)
    total = sum(lockstep_uv(g, o) for _ in range(10))
    print("gmm, unknown variances: z mismatches over 10 sweeps", total)
    assert g.get_degenerate() == 0
    g.close()


@pytest.mark.parametrize("N,dim,K", [(1, 1, 1), (5, 3, 2), (511, 8, 16), (513, 2, 5), (4099, 14, 33)])
def test_gmm_unknown_variances_shapes(B, N, dim, K):
    x = uv_points(N, dim, K, seed=N + K)
    g = B.GMM(K, 1.0, 10.0, 1.0, 5, x, var_shape=1.0, var_scale=1.0)
    o = O.OracleGMMUV(K, 1.0, 10.0, 1.0, 1.0, 5, x)
    for _ in range(3):
        lockstep_uv(g, o)
    g.close()


def test_gmm_unknown_variances_full_size_recovers_and_resumes(B):
    cfg = synth.GMM_CONFIG
    N, dim, K = cfg["N"], cfg["dim"], cfg["K"]
    x = uv_points(N, dim, K, seed=78)
    kw = dict(var_shape=1.0, var_scale=1.0)
    args = (K, 1.0, 10.0, 1.0, cfg["seed"], x)
    g, o = B.GMM(*args, **kw), O.OracleGMMUV(K, 1.0, 10.0, 1.0, 1.0, cfg["seed"], x)
    lockstep_uv(g, o)
    a, b = B.GMM(*args, **kw), B.GMM(*args, **kw)
    a.sweep(6)
    b.sweep(3)
    r = B.GMM(*args, **kw)
    r.set_state(*b.get_state())
    r.set_var(b.get_var())
    r.sweep(3)
    for u, v in zip(a.get_state() + (a.get_var(),), r.get_state() + (r.get_var(),)):
        assert np.array_equal(u, v)
    # the variance conditional, re-derived at full size from the data in fp64
    z, _, mu, _ = a.get_state()
    ss = np.zeros(K)
    np.add.at(ss, z, ((x.astype(np.float64) - mu.astype(np.float64)[z]) ** 2).sum(axis=1))
    n_k = np.bincount(z, minlength=K)
    post_mean = (1.0 + 0.5 * ss) / (1.0 + 0.5 * n_k * dim - 1.0)
    assert np.abs(a.get_var() / post_mean - 1.0).max() < 0.05   # shape ~ 250000: sd 0.2 %
    for h in (g, a, b, r):
        h.close()


def test_gmm_unknown_variances_errors(B):
    x = uv_points(100, 2, 3, seed=1)
    g = B.GMM(3, 1.0, 10.0, 1.0, 5, x, var_shape=1.0, var_scale=1.0)
    with pytest.raises(B.AugurError):
        g.set_var(np.array([1.0, 0.0, 1.0], dtype=np.float32))
    with pytest.raises(B.AugurError):
        g.set_var(np.array([1.0, np.nan, 1.0], dtype=np.float32))
    g.close()
    with pytest.raises(B.AugurError):
        B.GMM(3, 1.0, 10.0, 1.0, 5, x, var_shape=1.0, var_scale=0.0)
    with pytest.raises(B.AugurError):
        B.GMM(3, 1.0, 10.0, 1.0, 5, x, var_shape=-1.0, var_scale=1.0)
    k = B.GMM(3, 1.0, 10.0, 1.0, 5, x)
    with pytest.raises(B.AugurError):
        k.get_var()
    k.close()


@pytest.mark.parametrize("unknown_var", [False, True])
def test_gmm_sweeps_replayed_from_a_graph_match_direct_launches(B, unknown_var):
    import torch
    d = synth.gmm_points(N=20011, dim=8, K=16, seed=4)
    kw = dict(var_shape=1.0, var_scale=1.0) if unknown_var else {}
    stream = torch.cuda.Stream()
    a = B.GMM(16, 1.0, 10.0, 1.0, 5, d["x"], stream=stream, **kw)     # records
    b = B.GMM(16, 1.0, 10.0, 1.0, 5, d["x"], **kw)                    # default stream: direct launches

    def same():
        for x, y in zip(a.get_state() + a.get_stats(), b.get_state() + b.get_stats()):
            assert np.array_equal(x, y)
        assert a.loglik() == b.loglik()

    a.sweep(3); b.sweep(3); same()
    a.sweep(1); b.sweep(1); same()
    for h in (a, b):
        h.step_sample_z(); h.step_stats(); h.step_resample(); h.step_finish()
    same()
    a.sweep(2); b.sweep(2); same()
    a.sweep_profile(2); b.sweep_profile(2); same()
    z, pi, mu, sw = b.get_state()
    for h in (a, b):
        h.set_state(z=z, pi=pi, mu=mu, sweep=2)
    a.sweep(3); b.sweep(3); same()
    a.set_graph(False)
    a.sweep(2); b.sweep(2); same()
    with pytest.raises(B.AugurError):
        b.set_graph(True)
    a.close(); b.close()

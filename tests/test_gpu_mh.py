"""GPU parity of the Metropolis-Hastings sampler on the regression model against the oracle."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_1312_3613_amd import synth

pytestmark = pytest.mark.gpu

LOGF_RTOL = 1e-11      # fp64 sums in a different order: N * 2^-53 at worst, far below this
THETA_RTOL = 1e-12     # the proposal adds step * normal; the normal's last bits may differ
HYPER = dict(prior_sd=10.0, a0=3.0, b0=1.0, l=-1.0, u=1.0)


@pytest.fixture(scope="module")
def B():
    from paper_1312_3613_amd import binding
    binding.lib()
    return binding


def make_pair(B, d, step, seed, theta0=None, schedule=0):
    g = B.MHRegression(d["x"], d["y"], HYPER["prior_sd"], HYPER["a0"], HYPER["b0"], HYPER["l"],
                       HYPER["u"], step, seed, theta0=theta0)
    g.set_schedule(schedule)
    o = O.OracleMHRegression(d["x"], d["y"], HYPER["prior_sd"], HYPER["a0"], HYPER["b0"], HYPER["l"],
                             HYPER["u"], step, seed, theta0=theta0)
    return g, o


def close(a, b, rtol, floor):
    """|a - b| <= rtol * max(|b|, floor): a parameter that walks through zero keeps the absolute
    rounding error of the steps that brought it there."""
    return np.all(np.abs(np.asarray(a) - np.asarray(b)) <= rtol * np.maximum(np.abs(b), floor))


def compare_traces(tg, o, before, to, first_step):
    """Rows agree to rounding.  A decision may differ only where ln u lies within rounding of the
    log ratio; the chains then part for good and the comparison stops there.  Returns the number
    of rows compared."""
    prev, prev_lf = before
    for s in range(len(to)):
        if not close(tg[s, :-1], to[s, :-1], THETA_RTOL, o.step):
            t = first_step + s
            lp = o.evaluate(O.mhreg_propose(prev, o.step, o.seed, t))
            lu = np.log(O.mhreg_accept_uniform(o.seed, t))
            assert abs(lu - (lp - prev_lf)) <= 1e-9 * max(1.0, abs(lp)), \
                (f"step {t}: decisions differ", tg[s], to[s], lu, lp - prev_lf)
            return s
        assert abs(tg[s, -1] - to[s, -1]) <= LOGF_RTOL * abs(to[s, -1]), (s, tg[s, -1], to[s, -1])
        prev, prev_lf = to[s, :-1], to[s, -1]
    return len(to)


@pytest.mark.parametrize("schedule", [1, 2])
@pytest.mark.parametrize("N,K", [(1, 1), (7, 3), (1000, 8), (1025, 11), (4898, 11), (20_000, 5)])
def test_chain_matches_oracle_step_by_step(B, N, K, schedule):
    d = synth.regression_data(N=N, K=K, seed=N + K)
    step = 0.3 / np.sqrt(N)
    g, o = make_pair(B, d, step, seed=13, schedule=schedule)
    th, lf, si, acc = g.get_state()
    assert si == 0 and acc == 0 and np.array_equal(th, o.theta)
    assert abs(lf - o.logf) <= LOGF_RTOL * abs(o.logf)
    before = (o.theta.copy(), o.logf)
    n = 400
    tg, to = g.run(n, trace=True), o.run(n, trace=True)
    assert compare_traces(tg, o, before, to, 1) == n
    th, lf, si, acc = g.get_state()
    assert si == n and acc == o.accepted and 0 < acc < n
    assert close(th, o.theta, THETA_RTOL, o.step) and np.array_equal(th, tg[-1, :-1]) and lf == tg[-1, -1]
    g.close()


def test_schedules_agree_bit_for_bit_and_runs_compose(B):
    d = synth.regression_data(N=9000, K=8, seed=5)
    kw = dict(step=0.004, seed=3)
    a, _ = make_pair(B, d, schedule=1, **kw)
    b, _ = make_pair(B, d, schedule=2, **kw)
    c, _ = make_pair(B, d, schedule=0, **kw)
    ta, tb = a.run(300, trace=True), b.run(300, trace=True)
    assert np.array_equal(ta, tb)
    c.run(100); c.run(0); c.run(200)                      # no trace, split run
    assert np.array_equal(c.get_state()[0], a.get_state()[0]) and c.get_state()[1:] == a.get_state()[1:]
    # resume from a saved state on a fresh handle
    th, lf, si, acc = a.get_state()
    r, _ = make_pair(B, d, schedule=2, **kw)
    r.set_state(theta=th, step_index=si)
    assert r.get_state()[1] == lf
    a.run(50); r.run(50)
    assert np.array_equal(a.get_state()[0], r.get_state()[0])
    for h in (a, b, c, r):
        h.close()


def test_proposals_outside_the_support_are_refused(B):
    d = synth.regression_data(N=300, K=2, seed=9)
    theta0 = np.array([0.0, 0.0, 0.0, 0.05])
    for schedule in (1, 2):
        g, o = make_pair(B, d, step=0.2, seed=4, theta0=theta0, schedule=schedule)
        before = (o.theta.copy(), o.logf)
        tg, to = g.run(500, trace=True), o.run(500, trace=True)
        assert compare_traces(tg, o, before, to, 1) == 500
        assert (tg[:, 3] > 0).all() and g.get_state()[3] == o.accepted
        g.close()


def test_large_data_set_and_device_pointers(B):
    import torch
    N, K = 1_000_000, 8
    d = synth.regression_data(N=N, K=K, seed=2)
    x, y = torch.as_tensor(d["x"]).cuda(), torch.as_tensor(d["y"]).cuda()
    stream = torch.cuda.Stream()
    step = 0.3 / np.sqrt(N)
    g = B.MHRegression(x, y, 10.0, 3.0, 1.0, -1.0, 1.0, step, 17, device_ptrs=True, stream=stream)
    o = O.OracleMHRegression(d["x"], d["y"], 10.0, 3.0, 1.0, -1.0, 1.0, step, 17)
    before = (o.theta.copy(), o.logf)
    tg = g.run(60, trace=True)
    g.sync()
    to = o.run(60, trace=True)
    assert compare_traces(tg.cpu().numpy(), o, before, to, 1) == 60
    assert g.get_state()[3] == o.accepted
    g.close()


def test_invalid_inputs_are_rejected(B):
    d = synth.regression_data(N=50, K=2, seed=1)
    ok = dict(prior_sd=10.0, tau_shape=3.0, tau_scale=1.0, x_lo=-1.0, x_hi=1.0, step=0.1, seed=1)
    for bad in (dict(step=0.0), dict(prior_sd=-1.0), dict(x_lo=1.0, x_hi=1.0), dict(tau_shape=np.nan),
                dict(x_hi=0.5)):                                     # x beyond x_hi
        with pytest.raises(B.AugurError):
            B.MHRegression(d["x"], d["y"], **dict(ok, **bad))
    y = d["y"].copy(); y[3] = np.inf
    with pytest.raises(B.AugurError):
        B.MHRegression(d["x"], y, **ok)
    with pytest.raises(B.AugurError):
        B.MHRegression(d["x"], d["y"], theta0=np.array([0.0, 0.0, 0.0, -1.0]), **ok)
    g = B.MHRegression(d["x"], d["y"], **ok)
    with pytest.raises(B.AugurError):
        g.set_state(theta=np.array([0.0, np.nan, 0.0, 1.0]))
    with pytest.raises(B.AugurError):
        g.run(-1)
    g.close()

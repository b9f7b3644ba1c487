"""ctypes access to the oracle (oracle/augur_oracle.cpp).  TEST INFRASTRUCTURE.

Argument marshalling only: every number is computed by the C++ file.  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import this.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None

(STREAM_INIT_Z, STREAM_Z, STREAM_THETA, STREAM_PHI, STREAM_GMM_PI, STREAM_GMM_MU,
 STREAM_GMM_VAR, STREAM_MH_PROPOSAL, STREAM_MH_ACCEPT) = range(9)


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def lib():
    global _LIB
    if _LIB is None:
        path = os.environ.get("AUGUR_ORACLE_LIB")   # e.g. the sanitizer build, made by its test
        if not path:
            path = _build.LIB
            if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
                _build.build()
        L = C.CDLL(path)
        L.orc_uniform24.restype = C.c_double
        L.orc_uniform24.argtypes = [C.c_uint32]
        L.orc_uniform32.restype = C.c_double
        L.orc_uniform32.argtypes = [C.c_uint32]
        L.orc_gamma_log_draws.restype = C.c_int
        L.orc_lda_sample_z.restype = C.c_int64
        L.orc_lda_sweep.restype = C.c_int64
        L.orc_lda_sweep_phi_observed.restype = C.c_int64
        L.orc_lda_sample_z_f64.restype = C.c_int64
        L.orc_lda_sweep_f64.restype = C.c_int64
        L.orc_lda_sweep_phi_observed_f64.restype = C.c_int64
        L.orc_lda_resample_theta_f64.restype = C.c_int
        L.orc_lda_resample_phi_f64.restype = C.c_int
        L.orc_gmm_sample_z.restype = C.c_int64
        L.orc_gmm_sweep.restype = C.c_int64
        L.orc_gmm_loglik.restype = C.c_double
        L.orc_lda_resample_theta.restype = C.c_int
        L.orc_lda_resample_phi.restype = C.c_int
        L.orc_gmm_resample.restype = C.c_int
        L.orc_gmmuv_sample_z.restype = C.c_int64
        L.orc_gmmuv_sweep.restype = C.c_int64
        L.orc_gmmuv_resample.restype = C.c_int
        L.orc_gmmuv_loglik.restype = C.c_double
        L.orc_mhreg_logf.restype = C.c_double
        L.orc_mhreg_accept_uniform.restype = C.c_double
        L.orc_mhreg_run.restype = C.c_int64
        _LIB = L
    return _LIB


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# ----------------------------------------------------------------- primitives
def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(ctr, C.c_uint32), _p(key, C.c_uint32), _p(out, C.c_uint32))
    return out


def random_block(seed, index, sweep, stream, attempt=0):
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_random_block(C.c_uint64(seed), C.c_uint64(index), C.c_uint32(sweep),
                           C.c_uint32(stream), C.c_uint32(attempt), _p(out, C.c_uint32))
    return out


def uniform24(r):
    return lib().orc_uniform24(int(r))


def uniform32(r):
    return lib().orc_uniform32(int(r))


def datum_uniforms(seed, first, n, sweep, stream):
    u = np.zeros(n, dtype=np.float64)
    lib().orc_datum_uniforms(C.c_uint64(seed), C.c_uint64(first), C.c_int64(n), C.c_uint32(sweep),
                             C.c_uint32(stream), _p(u, C.c_double))
    return u


def normals(seed, first, n, sweep, stream):
    out = np.zeros(n, dtype=np.float64)
    lib().orc_normals(C.c_uint64(seed), C.c_uint64(first), C.c_int64(n), C.c_uint32(sweep),
                      C.c_uint32(stream), _p(out, C.c_double))
    return out


def gamma_log_draws(a, seed, first=0, sweep=0, stream=STREAM_THETA, return_attempts=False):
    a = _f64(a).ravel()
    lg = np.zeros(a.size, dtype=np.float64)
    att = np.zeros(a.size, dtype=np.int32)
    capped = lib().orc_gamma_log_draws(_p(a, C.c_double), C.c_int64(a.size), C.c_uint64(seed),
                                       C.c_uint64(first), C.c_uint32(sweep), C.c_uint32(stream),
                                       _p(lg, C.c_double), _p(att, C.c_int32))
    if return_attempts:
        return lg, att, capped
    return lg


# ------------------------------------------------------------------------ LDA
# f64=True selects the oracle's fp64 state mode (theta and phi stored as doubles): the exported
# functions ending in _f64.
def _state(f64):
    """(array converter, ctypes element type, numpy dtype, function-name suffix) of a state mode."""
    return (_f64, C.c_double, np.float64, "_f64") if f64 else (_f32, C.c_float, np.float32, "")


def doc_offsets(doc_len):
    off = np.zeros(len(doc_len) + 1, dtype=np.int64)
    np.cumsum(np.asarray(doc_len, dtype=np.int64), out=off[1:])
    return off


def lda_init_z(N, K, seed):
    z = np.zeros(N, dtype=np.int32)
    lib().orc_lda_init_z(C.c_int64(N), C.c_int32(K), C.c_uint64(seed), _p(z, C.c_int32))
    return z


def lda_sample_z(doc_off, w, theta, phi, seed, sweep, f64=False):
    conv, ct, _, sfx = _state(f64)
    doc_off, w, theta, phi = _i64(doc_off), _i32(w), conv(theta), conv(phi)
    D, K = theta.shape
    z = np.zeros(w.size, dtype=np.int32)
    deg = getattr(lib(), "orc_lda_sample_z" + sfx)(
        C.c_int32(D), C.c_int32(K), _p(doc_off, C.c_int64), _p(w, C.c_int32), _p(theta, ct),
        _p(phi, ct), C.c_uint64(seed), C.c_uint32(sweep), _p(z, C.c_int32))
    return z, deg


def lda_token_cdf(theta_d, phi_v, seed, token, sweep, f64=False):
    conv, ct, _, sfx = _state(f64)
    theta_d, phi_v = conv(theta_d), conv(phi_v)
    K = theta_d.size
    cdf = np.zeros(K, dtype=np.float64)
    t = C.c_double(0.0)
    getattr(lib(), "orc_lda_token_cdf" + sfx)(
        C.c_int32(K), _p(theta_d, ct), _p(phi_v, ct), C.c_uint64(seed), C.c_uint64(token),
        C.c_uint32(sweep), _p(cdf, C.c_double), C.byref(t))
    return cdf, t.value


def lda_count(doc_off, w, z, D, V, K):
    doc_off, w, z = _i64(doc_off), _i32(w), _i32(z)
    n_dk = np.zeros((D, K), dtype=np.int32)
    n_wk = np.zeros((V, K), dtype=np.int32)
    lib().orc_lda_count(C.c_int32(D), C.c_int32(V), C.c_int32(K), _p(doc_off, C.c_int64),
                        _p(w, C.c_int32), _p(z, C.c_int32), _p(n_dk, C.c_int32),
                        _p(n_wk, C.c_int32))
    return n_dk, n_wk


def lda_resample_theta(n_dk, alpha, seed, sweep, f64=False):
    _, ct, dt, sfx = _state(f64)
    n_dk = _i32(n_dk)
    D, K = n_dk.shape
    theta = np.zeros((D, K), dtype=dt)
    getattr(lib(), "orc_lda_resample_theta" + sfx)(
        C.c_int32(D), C.c_int32(K), C.c_double(alpha), _p(n_dk, C.c_int32), C.c_uint64(seed),
        C.c_uint32(sweep), _p(theta, ct))
    return theta


def lda_resample_phi(n_wk, beta, seed, sweep, f64=False):
    _, ct, dt, sfx = _state(f64)
    n_wk = _i32(n_wk)
    V, K = n_wk.shape
    phi = np.zeros((V, K), dtype=dt)
    getattr(lib(), "orc_lda_resample_phi" + sfx)(
        C.c_int32(V), C.c_int32(K), C.c_double(beta), _p(n_wk, C.c_int32), C.c_uint64(seed),
        C.c_uint32(sweep), _p(phi, ct))
    return phi


def lda_loglik(doc_off, w, z, theta, phi, alpha, beta, f64=False):
    conv, ct, _, sfx = _state(f64)
    doc_off, w, z, theta, phi = _i64(doc_off), _i32(w), _i32(z), conv(theta), conv(phi)
    D, K = theta.shape
    V = phi.shape[0]
    lj, lm = C.c_double(0.0), C.c_double(0.0)
    getattr(lib(), "orc_lda_loglik" + sfx)(
        C.c_int32(D), C.c_int32(V), C.c_int32(K), C.c_double(alpha), C.c_double(beta),
        _p(doc_off, C.c_int64), _p(w, C.c_int32), _p(z, C.c_int32), _p(theta, ct), _p(phi, ct),
        C.byref(lj), C.byref(lm))
    return lj.value, lm.value


class OracleLDA:
    """State holder around the oracle's LDA functions; same call names as the
    HIP binding so a test can drive both in lock-step."""

    def __init__(self, D, V, K, alpha, beta, seed, doc_len, w, f64=False):
        self.f64 = bool(f64)
        self._conv, self._ct, self._dt, self._sfx = _state(self.f64)
        self.D, self.V, self.K = int(D), int(V), int(K)
        self.alpha, self.beta, self.seed = float(np.float32(alpha)), float(np.float32(beta)), int(seed)
        self.doc_off = doc_offsets(doc_len)
        self.w = _i32(w).copy()
        self.N = int(self.doc_off[-1])
        assert self.w.size == self.N
        self.z = np.zeros(self.N, dtype=np.int32)
        self.theta = np.zeros((self.D, self.K), dtype=self._dt)
        self.phi = np.zeros((self.V, self.K), dtype=self._dt)
        self.n_dk = np.zeros((self.D, self.K), dtype=np.int32)
        self.n_wk = np.zeros((self.V, self.K), dtype=np.int32)
        self.sweep_index = 0
        self.degenerate = 0
        self.phi_observed = False
        getattr(lib(), "orc_lda_init" + self._sfx)(
            C.c_int32(self.D), C.c_int32(self.V), C.c_int32(self.K), C.c_double(self.alpha),
            C.c_double(self.beta), _p(self.doc_off, C.c_int64), _p(self.w, C.c_int32),
            C.c_uint64(self.seed), _p(self.z, C.c_int32), _p(self.theta, self._ct),
            _p(self.phi, self._ct), _p(self.n_dk, C.c_int32), _p(self.n_wk, C.c_int32))

    def set_observed(self, phi=False):
        self.phi_observed = bool(phi)

    def sweep(self, n=1):
        for _ in range(n):
            t = self.sweep_index + 1
            if self.phi_observed:
                scratch = np.zeros_like(self.n_wk)
                self.degenerate += getattr(lib(), "orc_lda_sweep_phi_observed" + self._sfx)(
                    C.c_int32(self.D), C.c_int32(self.V), C.c_int32(self.K), C.c_double(self.alpha),
                    _p(self.doc_off, C.c_int64), _p(self.w, C.c_int32), C.c_uint64(self.seed),
                    C.c_uint32(t), _p(self.z, C.c_int32), _p(self.theta, self._ct),
                    _p(self.phi, self._ct), _p(self.n_dk, C.c_int32), _p(scratch, C.c_int32))
                self.sweep_index = t
                continue
            self.degenerate += getattr(lib(), "orc_lda_sweep" + self._sfx)(
                C.c_int32(self.D), C.c_int32(self.V), C.c_int32(self.K), C.c_double(self.alpha),
                C.c_double(self.beta), _p(self.doc_off, C.c_int64), _p(self.w, C.c_int32),
                C.c_uint64(self.seed), C.c_uint32(t), _p(self.z, C.c_int32),
                _p(self.theta, self._ct), _p(self.phi, self._ct), _p(self.n_dk, C.c_int32),
                _p(self.n_wk, C.c_int32))
            self.sweep_index = t

    # step-level calls: all use sweep index sweep_index + 1; step_finish advances it
    def step_sample_z(self):
        self.z, deg = lda_sample_z(self.doc_off, self.w, self.theta, self.phi, self.seed,
                                   self.sweep_index + 1, f64=self.f64)
        self.degenerate += deg

    def step_count(self):
        self.n_dk, self.n_wk = lda_count(self.doc_off, self.w, self.z, self.D, self.V, self.K)

    def step_resample_theta(self):
        self.theta = lda_resample_theta(self.n_dk, self.alpha, self.seed, self.sweep_index + 1, f64=self.f64)

    def step_resample_phi(self):
        self.phi = lda_resample_phi(self.n_wk, self.beta, self.seed, self.sweep_index + 1, f64=self.f64)

    def step_finish(self):
        self.sweep_index += 1

    def loglik(self):
        return lda_loglik(self.doc_off, self.w, self.z, self.theta, self.phi, self.alpha, self.beta,
                          f64=self.f64)

    def get_state(self):
        return self.z.copy(), self.theta.copy(), self.phi.copy(), self.sweep_index

    def set_state(self, z=None, theta=None, phi=None, sweep=None):
        if z is not None:
            self.z = _i32(z).copy()
            self.step_count()
        if theta is not None:
            self.theta = self._conv(theta).reshape(self.D, self.K).copy()
        if phi is not None:
            self.phi = self._conv(phi).reshape(self.V, self.K).copy()
        if sweep is not None:
            self.sweep_index = int(sweep)

    def get_counts(self):
        return self.n_dk.copy(), self.n_wk.copy()


# ------------------------------------------------------------------------ GMM
def gmm_sample_z(x, pi, mu, sigma, seed, sweep):
    x, pi, mu = _f32(x), _f32(pi), _f32(mu)
    N, dim = x.shape
    K = pi.size
    z = np.zeros(N, dtype=np.int32)
    deg = lib().orc_gmm_sample_z(C.c_int64(N), C.c_int32(dim), C.c_int32(K), C.c_double(sigma),
                                 _p(x, C.c_float), _p(pi, C.c_float), _p(mu, C.c_float),
                                 C.c_uint64(seed), C.c_uint32(sweep), _p(z, C.c_int32))
    return z, deg


def gmm_point_cdf(x_i, pi, mu, sigma, seed, point, sweep):
    x_i, pi, mu = _f32(x_i), _f32(pi), _f32(mu)
    K, dim = pi.size, x_i.size
    cdf = np.zeros(K, dtype=np.float64)
    t = C.c_double(0.0)
    lib().orc_gmm_point_cdf(C.c_int32(dim), C.c_int32(K), C.c_double(sigma), _p(x_i, C.c_float),
                            _p(pi, C.c_float), _p(mu, C.c_float), C.c_uint64(seed),
                            C.c_uint64(point), C.c_uint32(sweep), _p(cdf, C.c_double), C.byref(t))
    return cdf, t.value


def gmm_stats(x, z, K):
    x, z = _f32(x), _i32(z)
    N, dim = x.shape
    n_k = np.zeros(K, dtype=np.int32)
    s_k = np.zeros((K, dim), dtype=np.float64)
    lib().orc_gmm_stats(C.c_int64(N), C.c_int32(dim), C.c_int32(K), _p(x, C.c_float),
                        _p(z, C.c_int32), _p(n_k, C.c_int32), _p(s_k, C.c_double))
    return n_k, s_k


def gmm_resample(n_k, s_k, alpha, prior_sd, sigma, seed, sweep):
    n_k, s_k = _i32(n_k), _f64(s_k)
    K, dim = s_k.shape
    pi = np.zeros(K, dtype=np.float32)
    mu = np.zeros((K, dim), dtype=np.float32)
    lib().orc_gmm_resample(C.c_int32(dim), C.c_int32(K), C.c_double(alpha), C.c_double(prior_sd),
                           C.c_double(sigma), _p(n_k, C.c_int32), _p(s_k, C.c_double),
                           C.c_uint64(seed), C.c_uint32(sweep), _p(pi, C.c_float),
                           _p(mu, C.c_float))
    return pi, mu


def gmm_loglik(x, z, pi, mu, alpha, prior_sd, sigma):
    x, z, pi, mu = _f32(x), _i32(z), _f32(pi), _f32(mu)
    N, dim = x.shape
    return lib().orc_gmm_loglik(C.c_int64(N), C.c_int32(dim), C.c_int32(pi.size),
                                C.c_double(alpha), C.c_double(prior_sd), C.c_double(sigma),
                                _p(x, C.c_float), _p(z, C.c_int32), _p(pi, C.c_float),
                                _p(mu, C.c_float))


class OracleGMM:
    def __init__(self, K, alpha, prior_sd, sigma, seed, x):
        self.x = _f32(x).copy()
        self.N, self.dim = self.x.shape
        self.K = int(K)
        self.alpha = float(np.float32(alpha))
        self.prior_sd = float(np.float32(prior_sd))
        self.sigma = float(np.float32(sigma))
        self.seed = int(seed)
        self.z = np.zeros(self.N, dtype=np.int32)
        self.pi = np.zeros(self.K, dtype=np.float32)
        self.mu = np.zeros((self.K, self.dim), dtype=np.float32)
        self.n_k = np.zeros(self.K, dtype=np.int32)
        self.s_k = np.zeros((self.K, self.dim), dtype=np.float64)
        self.sweep_index = 0
        self.degenerate = 0
        lib().orc_gmm_init(C.c_int64(self.N), C.c_int32(self.dim), C.c_int32(self.K),
                           C.c_double(self.alpha), C.c_double(self.prior_sd),
                           C.c_double(self.sigma), _p(self.x, C.c_float), C.c_uint64(self.seed),
                           _p(self.z, C.c_int32), _p(self.pi, C.c_float), _p(self.mu, C.c_float),
                           _p(self.n_k, C.c_int32), _p(self.s_k, C.c_double))

    def sweep(self, n=1):
        for _ in range(n):
            t = self.sweep_index + 1
            self.degenerate += lib().orc_gmm_sweep(
                C.c_int64(self.N), C.c_int32(self.dim), C.c_int32(self.K), C.c_double(self.alpha),
                C.c_double(self.prior_sd), C.c_double(self.sigma), _p(self.x, C.c_float),
                C.c_uint64(self.seed), C.c_uint32(t), _p(self.z, C.c_int32),
                _p(self.pi, C.c_float), _p(self.mu, C.c_float), _p(self.n_k, C.c_int32),
                _p(self.s_k, C.c_double))
            self.sweep_index = t

    def step_sample_z(self):
        self.z, deg = gmm_sample_z(self.x, self.pi, self.mu, self.sigma, self.seed,
                                   self.sweep_index + 1)
        self.degenerate += deg

    def step_stats(self):
        self.n_k, self.s_k = gmm_stats(self.x, self.z, self.K)

    def step_resample(self):
        self.pi, self.mu = gmm_resample(self.n_k, self.s_k, self.alpha, self.prior_sd, self.sigma,
                                        self.seed, self.sweep_index + 1)

    def step_finish(self):
        self.sweep_index += 1

    def loglik(self):
        return gmm_loglik(self.x, self.z, self.pi, self.mu, self.alpha, self.prior_sd, self.sigma)

    def get_state(self):
        return self.z.copy(), self.pi.copy(), self.mu.copy(), self.sweep_index

    def set_state(self, z=None, pi=None, mu=None, sweep=None):
        if z is not None:
            self.z = _i32(z).copy()
            self.step_stats()
        if pi is not None:
            self.pi = _f32(pi).copy()
        if mu is not None:
            self.mu = _f32(mu).reshape(self.K, self.dim).copy()
        if sweep is not None:
            self.sweep_index = int(sweep)

    def get_stats(self):
        return self.n_k.copy(), self.s_k.copy()


# ------------------------------------------- GMM with unknown component variances
def gmmuv_sample_z(x, pi, mu, var, seed, sweep):
    x, pi, mu, var = _f32(x), _f32(pi), _f32(mu), _f32(var)
    N, dim = x.shape
    z = np.zeros(N, dtype=np.int32)
    deg = lib().orc_gmmuv_sample_z(C.c_int64(N), C.c_int32(dim), C.c_int32(pi.size), _p(x, C.c_float),
                                   _p(pi, C.c_float), _p(mu, C.c_float), _p(var, C.c_float),
                                   C.c_uint64(seed), C.c_uint32(sweep), _p(z, C.c_int32))
    return z, deg


def gmmuv_point_cdf(x_i, pi, mu, var, seed, point, sweep):
    x_i, pi, mu, var = _f32(x_i), _f32(pi), _f32(mu), _f32(var)
    cdf = np.zeros(pi.size, dtype=np.float64)
    t = C.c_double(0.0)
    lib().orc_gmmuv_point_cdf(C.c_int32(x_i.size), C.c_int32(pi.size), _p(x_i, C.c_float),
                              _p(pi, C.c_float), _p(mu, C.c_float), _p(var, C.c_float),
                              C.c_uint64(seed), C.c_uint64(point), C.c_uint32(sweep),
                              _p(cdf, C.c_double), C.byref(t))
    return cdf, t.value


def gmmuv_resample(x, z, n_k, s_k, var, alpha, prior_sd, a0, b0, seed, sweep):
    x, z, n_k, s_k = _f32(x), _i32(z), _i32(n_k), _f64(s_k)
    var = _f32(var).copy()
    N, dim = x.shape
    K = n_k.size
    pi = np.zeros(K, dtype=np.float32)
    mu = np.zeros((K, dim), dtype=np.float32)
    lib().orc_gmmuv_resample(C.c_int64(N), C.c_int32(dim), C.c_int32(K), C.c_double(alpha),
                             C.c_double(prior_sd), C.c_double(a0), C.c_double(b0), _p(x, C.c_float),
                             _p(z, C.c_int32), _p(n_k, C.c_int32), _p(s_k, C.c_double),
                             C.c_uint64(seed), C.c_uint32(sweep), _p(pi, C.c_float), _p(mu, C.c_float),
                             _p(var, C.c_float))
    return pi, mu, var


def gmmuv_loglik(x, z, pi, mu, var, alpha, prior_sd, a0, b0):
    x, z, pi, mu, var = _f32(x), _i32(z), _f32(pi), _f32(mu), _f32(var)
    N, dim = x.shape
    return lib().orc_gmmuv_loglik(C.c_int64(N), C.c_int32(dim), C.c_int32(pi.size), C.c_double(alpha),
                                  C.c_double(prior_sd), C.c_double(a0), C.c_double(b0),
                                  _p(x, C.c_float), _p(z, C.c_int32), _p(pi, C.c_float),
                                  _p(mu, C.c_float), _p(var, C.c_float))


class OracleGMMUV(OracleGMM):
    """Mixture with var_k ~ InverseGamma(a0, b0) per component."""

    def __init__(self, K, alpha, prior_sd, a0, b0, seed, x):
        self.x = _f32(x).copy()
        self.N, self.dim = self.x.shape
        self.K = int(K)
        self.alpha, self.prior_sd = float(np.float32(alpha)), float(np.float32(prior_sd))
        self.a0, self.b0 = float(np.float32(a0)), float(np.float32(b0))
        self.sigma = None
        self.seed = int(seed)
        self.z = np.zeros(self.N, dtype=np.int32)
        self.pi = np.zeros(self.K, dtype=np.float32)
        self.mu = np.zeros((self.K, self.dim), dtype=np.float32)
        self.var = np.zeros(self.K, dtype=np.float32)
        self.n_k = np.zeros(self.K, dtype=np.int32)
        self.s_k = np.zeros((self.K, self.dim), dtype=np.float64)
        self.sweep_index = 0
        self.degenerate = 0
        lib().orc_gmmuv_init(C.c_int64(self.N), C.c_int32(self.dim), C.c_int32(self.K),
                             C.c_double(self.alpha), C.c_double(self.prior_sd), C.c_double(self.a0),
                             C.c_double(self.b0), _p(self.x, C.c_float), C.c_uint64(self.seed),
                             _p(self.z, C.c_int32), _p(self.pi, C.c_float), _p(self.mu, C.c_float),
                             _p(self.var, C.c_float), _p(self.n_k, C.c_int32), _p(self.s_k, C.c_double))

    def sweep(self, n=1):
        for _ in range(n):
            t = self.sweep_index + 1
            self.degenerate += lib().orc_gmmuv_sweep(
                C.c_int64(self.N), C.c_int32(self.dim), C.c_int32(self.K), C.c_double(self.alpha),
                C.c_double(self.prior_sd), C.c_double(self.a0), C.c_double(self.b0),
                _p(self.x, C.c_float), C.c_uint64(self.seed), C.c_uint32(t), _p(self.z, C.c_int32),
                _p(self.pi, C.c_float), _p(self.mu, C.c_float), _p(self.var, C.c_float),
                _p(self.n_k, C.c_int32), _p(self.s_k, C.c_double))
            self.sweep_index = t

    def step_sample_z(self):
        self.z, deg = gmmuv_sample_z(self.x, self.pi, self.mu, self.var, self.seed, self.sweep_index + 1)
        self.degenerate += deg

    def step_resample(self):
        self.pi, self.mu, self.var = gmmuv_resample(self.x, self.z, self.n_k, self.s_k, self.var,
                                                    self.alpha, self.prior_sd, self.a0, self.b0,
                                                    self.seed, self.sweep_index + 1)

    def loglik(self):
        return gmmuv_loglik(self.x, self.z, self.pi, self.mu, self.var, self.alpha, self.prior_sd,
                            self.a0, self.b0)

    def get_state(self):
        return self.z.copy(), self.pi.copy(), self.mu.copy(), self.sweep_index

    def set_var(self, var):
        self.var = _f32(var).copy()


# ------------------------------- Metropolis-Hastings on the multivariate regression
def mhreg_logf(x, y, theta, prior_sd, a0, b0, l, u):
    x, y, theta = _f32(x), _f32(y), _f64(theta)
    N, K = x.shape
    return lib().orc_mhreg_logf(C.c_int64(N), C.c_int32(K), _p(x, C.c_float), _p(y, C.c_float),
                                _p(theta, C.c_double), C.c_double(prior_sd), C.c_double(a0),
                                C.c_double(b0), C.c_double(l), C.c_double(u))


def mhreg_propose(theta, step, seed, t):
    theta = _f64(theta)
    out = np.zeros_like(theta)
    lib().orc_mhreg_propose(C.c_int32(theta.size - 2), _p(theta, C.c_double), C.c_double(step),
                            C.c_uint64(seed), C.c_uint32(t), _p(out, C.c_double))
    return out


def mhreg_accept_uniform(seed, t):
    return lib().orc_mhreg_accept_uniform(C.c_uint64(seed), C.c_uint32(t))


class OracleMHRegression:
    """Random-walk Metropolis-Hastings chain over theta = (w_0..w_{K-1}, b, tau)."""

    def __init__(self, x, y, prior_sd, a0, b0, l, u, step, seed, theta0=None):
        self.x, self.y = _f32(x).copy(), _f32(y).copy()
        self.N, self.K = self.x.shape
        f = lambda v: float(np.float32(v))
        self.prior_sd, self.a0, self.b0, self.l, self.u = f(prior_sd), f(a0), f(b0), f(l), f(u)
        self.step = f(step)
        self.seed = int(seed)
        if theta0 is None:
            theta0 = np.concatenate([np.zeros(self.K + 1), [1.0]])
        self.theta = _f64(theta0).copy()
        self.logf = self.evaluate(self.theta)
        self.step_index = 0
        self.accepted = 0

    def evaluate(self, theta):
        return mhreg_logf(self.x, self.y, theta, self.prior_sd, self.a0, self.b0, self.l, self.u)

    def run(self, n, trace=False):
        tr = np.zeros((n, self.K + 3), dtype=np.float64) if trace else None
        lf = C.c_double(self.logf)
        self.accepted += lib().orc_mhreg_run(
            C.c_int64(self.N), C.c_int32(self.K), _p(self.x, C.c_float), _p(self.y, C.c_float),
            C.c_double(self.prior_sd), C.c_double(self.a0), C.c_double(self.b0), C.c_double(self.l),
            C.c_double(self.u), C.c_double(self.step), C.c_uint64(self.seed),
            C.c_uint32(self.step_index + 1), C.c_int64(n), _p(self.theta, C.c_double), C.byref(lf),
            _p(tr, C.c_double) if trace else None)
        self.logf = lf.value
        self.step_index += n
        return tr

    def set_state(self, theta, step_index=None):
        self.theta = _f64(theta).copy()
        self.logf = self.evaluate(self.theta)
        if step_index is not None:
            self.step_index = int(step_index)

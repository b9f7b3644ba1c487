"""Python face of the C ABI in include/augur.h: argument marshalling only.

Every computation happens in the HIP library (libaugur_hip.so).  Arrays cross the boundary
either as numpy arrays (host pointers) or, for handles created with device_ptrs=True, as torch
CUDA tensors (device pointers); torch is used for nothing but device memory and streams.
There is no fallback: if the library is absent and cannot be built, loading raises.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

OK, ERR_INVALID_ARG, ERR_HIP, ERR_DEGENERATE, ERR_UNIMPLEMENTED = 0, -1, -2, -3, -4
PTRS_DEVICE = 1
STATE_F64 = 2
LDA_NSTEPS = 5

_LIB = None


class AugurError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"augur error {code}: {message}")
        self.code = code


class LdaConfig(C.Structure):
    _fields_ = [("D", C.c_int32), ("V", C.c_int32), ("K", C.c_int32), ("alpha", C.c_float),
                ("beta", C.c_float), ("seed", C.c_uint64), ("device", C.c_int32),
                ("stream", C.c_void_p), ("flags", C.c_uint32)]


class GmmConfig(C.Structure):
    _fields_ = [("N", C.c_int64), ("dim", C.c_int32), ("K", C.c_int32), ("alpha", C.c_float),
                ("prior_sd", C.c_float), ("sigma", C.c_float), ("var_shape", C.c_float),
                ("var_scale", C.c_float), ("seed", C.c_uint64),
                ("device", C.c_int32), ("stream", C.c_void_p), ("flags", C.c_uint32)]


class LdaStaticArgs(C.Structure):
    _fields_ = [("D", C.c_int32), ("V", C.c_int32), ("K", C.c_int32), ("ld", C.c_int32),
                ("alpha", C.c_float), ("beta", C.c_float), ("doc_len", C.c_void_p),
                ("w", C.c_void_p), ("z", C.c_void_p), ("theta", C.c_void_p), ("phi", C.c_void_p),
                ("device", C.c_int32), ("stream", C.c_void_p)]


class MhRegConfig(C.Structure):
    _fields_ = [("N", C.c_int64), ("K", C.c_int32), ("prior_sd", C.c_float),
                ("tau_shape", C.c_float), ("tau_scale", C.c_float), ("x_lo", C.c_float),
                ("x_hi", C.c_float), ("step", C.c_float), ("seed", C.c_uint64),
                ("device", C.c_int32), ("stream", C.c_void_p), ("flags", C.c_uint32)]


def lib():
    """Load libaugur_hip.so, building it first if it is absent or was built from other sources
    than the ones present (a digest of the sources is kept beside the library).  A failed build
    raises: a library older than its sources is never loaded."""
    global _LIB
    if _LIB is None:
        if _build.stale():
            _build.build(force=True)
        if not os.path.exists(_build.LIB):
            raise RuntimeError("HIP library libaugur_hip.so is missing and could not be built")
        # One HIP runtime per process: torch ships its own libamdhip64 (same soname as the
        # system one).  Loading torch first makes the dynamic linker bind this library to the
        # runtime torch uses, so device pointers and streams are shared; two runtimes in one
        # process do not see each other's devices.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(_build.LIB)
        L.augur_last_error.restype = C.c_char_p
        L.augur_version.restype = C.c_char_p
        vp = C.c_void_p
        L.augur_lda_create.argtypes = [C.POINTER(LdaConfig), vp, vp, C.POINTER(vp)]
        L.augur_lda_destroy.argtypes = [vp]
        L.augur_lda_destroy.restype = None
        L.augur_lda_sweep.argtypes = [vp, C.c_int32]
        L.augur_lda_sweep_profile.argtypes = [vp, C.c_int32, C.POINTER(C.c_double)]
        L.augur_lda_set_overlap.argtypes = [vp, C.c_int32]
        L.augur_lda_set_z_cache.argtypes = [vp, C.c_int32]
        L.augur_lda_set_graph.argtypes = [vp, C.c_int32]
        L.augur_lda_set_observed.argtypes = [vp, C.c_uint32]
        for name in ("step_sample_z", "step_count", "step_resample_theta", "step_resample_phi",
                     "step_finish", "sync"):
            getattr(L, "augur_lda_" + name).argtypes = [vp]
        L.augur_lda_loglik.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.augur_lda_get_state.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_int64)]
        L.augur_lda_set_state.argtypes = [vp, vp, vp, vp, C.c_int64]
        L.augur_lda_get_state_f64.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_int64)]
        L.augur_lda_set_state_f64.argtypes = [vp, vp, vp, vp, C.c_int64]
        L.augur_lda_get_counts.argtypes = [vp, vp, vp]
        L.augur_lda_get_degenerate.argtypes = [vp, C.POINTER(C.c_int64)]
        L.augur_lda_probe_gather.argtypes = [vp, C.c_int32, C.POINTER(C.c_double)]
        L.augur_probe_stream_copy.argtypes = [vp, vp, C.c_int64, C.c_int32, vp, C.POINTER(C.c_double)]
        L.augur_lda_loglik_static.argtypes = [C.POINTER(LdaStaticArgs), vp]
        L.augur_gmm_create.argtypes = [C.POINTER(GmmConfig), vp, C.POINTER(vp)]
        L.augur_gmm_destroy.argtypes = [vp]
        L.augur_gmm_destroy.restype = None
        L.augur_gmm_sweep.argtypes = [vp, C.c_int32]
        L.augur_gmm_set_graph.argtypes = [vp, C.c_int32]
        L.augur_gmm_sweep_profile.argtypes = [vp, C.c_int32, C.POINTER(C.c_double)]
        for name in ("step_sample_z", "step_stats", "step_resample", "step_finish", "sync"):
            getattr(L, "augur_gmm_" + name).argtypes = [vp]
        L.augur_gmm_loglik.argtypes = [vp, C.POINTER(C.c_double)]
        L.augur_gmm_get_state.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_int64)]
        L.augur_gmm_set_state.argtypes = [vp, vp, vp, vp, C.c_int64]
        L.augur_gmm_get_stats.argtypes = [vp, vp, vp]
        L.augur_gmm_get_var.argtypes = [vp, vp]
        L.augur_gmm_set_var.argtypes = [vp, vp]
        L.augur_gmm_get_degenerate.argtypes = [vp, C.POINTER(C.c_int64)]
        L.augur_mhreg_create.argtypes = [C.POINTER(MhRegConfig), vp, vp, vp, C.POINTER(vp)]
        L.augur_mhreg_destroy.argtypes = [vp]
        L.augur_mhreg_destroy.restype = None
        L.augur_mhreg_run.argtypes = [vp, C.c_int64, vp]
        L.augur_mhreg_get_state.argtypes = [vp, vp, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                            C.POINTER(C.c_int64)]
        L.augur_mhreg_set_state.argtypes = [vp, vp, C.c_int64]
        L.augur_mhreg_set_schedule.argtypes = [vp, C.c_int32]
        L.augur_mhreg_sync.argtypes = [vp]
        _LIB = L
    return _LIB


def last_error():
    return lib().augur_last_error().decode()


def _check(rc, allow=()):
    if rc != OK and rc not in allow:
        raise AugurError(rc, last_error())
    return rc


def _ptr(a):
    """Raw address of a numpy array or torch tensor (None -> NULL)."""
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        return a.ctypes.data
    return a.data_ptr()


def _stream_handle(stream):
    if stream is None:
        return None
    return getattr(stream, "cuda_stream", stream)


class _Arrays:
    """Allocates output buffers and normalises inputs on the side of the boundary the handle
    was created for: numpy (host) or torch CUDA tensors (device)."""

    def __init__(self, device_ptrs, device):
        self.device_ptrs = device_ptrs
        self.device = device
        if device_ptrs:
            import torch
            self.torch = torch
            self.tdev = torch.device("cuda", device)

    _np = {"i32": np.int32, "f32": np.float32, "f64": np.float64}

    def empty(self, shape, kind):
        if self.device_ptrs:
            dt = {"i32": self.torch.int32, "f32": self.torch.float32, "f64": self.torch.float64}[kind]
            return self.torch.empty(shape, dtype=dt, device=self.tdev)
        return np.empty(shape, dtype=self._np[kind])

    def input(self, a, kind, size=None):
        if a is None:
            return None
        if self.device_ptrs:
            dt = {"i32": self.torch.int32, "f32": self.torch.float32, "f64": self.torch.float64}[kind]
            t = a if self.torch.is_tensor(a) else self.torch.as_tensor(np.asarray(a))
            t = t.to(device=self.tdev, dtype=dt).contiguous()
        else:
            t = np.ascontiguousarray(a, dtype=self._np[kind])
        n = t.numel() if self.device_ptrs else t.size
        if size is not None and n != size:
            raise ValueError(f"array has {n} elements, expected {size}")
        return t


def lda_loglik_static(D, V, K, ld, alpha, beta, doc_len, w, z, theta, phi, out, device=0,
                      stream=None):
    """augur_lda_loglik_static: every array is a torch CUDA tensor the caller owns (out: two
    float64); nothing is allocated, copied or waited for here."""
    a = LdaStaticArgs(int(D), int(V), int(K), int(ld), float(alpha), float(beta), _ptr(doc_len),
                      _ptr(w), _ptr(z), _ptr(theta), _ptr(phi), int(device), _stream_handle(stream))
    _check(lib().augur_lda_loglik_static(C.byref(a), _ptr(out)))


def probe_stream_copy(src, dst, reps=10, stream=None):
    """augur_probe_stream_copy on two equally sized torch CUDA tensors: ms per copy."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst differ in size")
    ms = C.c_double()
    _check(lib().augur_probe_stream_copy(_ptr(src), _ptr(dst), nbytes, int(reps),
                                         _stream_handle(stream), C.byref(ms)))
    return ms.value


class LDA:
    """augur_lda_* handle.  Method names are the ABI's.  state_f64=True asks for the fp64 state
    (AUGUR_STATE_F64): get_state and set_state then carry theta and phi as float64 through the
    _f64 entry points."""

    def __init__(self, D, V, K, alpha, beta, seed, doc_len, w, device=0, stream=None,
                 device_ptrs=False, state_f64=False):
        self._h = None
        self.state_f64 = bool(state_f64)
        self.D, self.V, self.K = int(D), int(V), int(K)
        self._arr = _Arrays(device_ptrs, device)
        doc_len_a = self._arr.input(doc_len, "i32")
        w_a = self._arr.input(w, "i32")
        n_docs = doc_len_a.numel() if device_ptrs else doc_len_a.size
        if n_docs != self.D:
            raise ValueError(f"doc_len has {n_docs} entries, expected D = {self.D}")
        n_tok = w_a.numel() if device_ptrs else w_a.size
        self.N = int(doc_len_a.sum())
        if n_tok != self.N:
            raise ValueError(f"w has {n_tok} entries, sum(doc_len) = {self.N}")
        cfg = LdaConfig(self.D, self.V, self.K, float(alpha), float(beta), int(seed), int(device),
                        _stream_handle(stream),
                        (PTRS_DEVICE if device_ptrs else 0) | (STATE_F64 if state_f64 else 0))
        h = C.c_void_p()
        _check(lib().augur_lda_create(C.byref(cfg), _ptr(doc_len_a), _ptr(w_a), C.byref(h)))
        self._h = h

    def close(self):
        if self._h is not None:
            lib().augur_lda_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:  # interpreter shutdown: the module globals may be gone
            pass

    def sweep(self, n=1):
        _check(lib().augur_lda_sweep(self._h, int(n)))

    def set_observed(self, phi=False):
        _check(lib().augur_lda_set_observed(self._h, 1 if phi else 0))

    def set_overlap(self, on):
        _check(lib().augur_lda_set_overlap(self._h, 1 if on else 0))

    def set_z_cache(self, mode):
        _check(lib().augur_lda_set_z_cache(self._h, int(mode)))

    def set_word_table(self, mode):
        _check(lib().augur_lda_set_word_table(self._h, int(mode)))

    def set_graph(self, on):
        _check(lib().augur_lda_set_graph(self._h, 1 if on else 0))

    def sweep_profile(self, n=1):
        ms = (C.c_double * LDA_NSTEPS)()
        _check(lib().augur_lda_sweep_profile(self._h, int(n), ms))
        return dict(zip(("sample_z", "count_accumulate", "resample_theta", "resample_phi", "sweep"),
                        list(ms)))

    def probe_gather(self, reps=5):
        ms = C.c_double()
        _check(lib().augur_lda_probe_gather(self._h, int(reps), C.byref(ms)))
        return ms.value

    def step_sample_z(self):
        _check(lib().augur_lda_step_sample_z(self._h))

    def step_count(self):
        _check(lib().augur_lda_step_count(self._h))

    def step_resample_theta(self):
        _check(lib().augur_lda_step_resample_theta(self._h))

    def step_resample_phi(self):
        _check(lib().augur_lda_step_resample_phi(self._h))

    def step_finish(self):
        _check(lib().augur_lda_step_finish(self._h))

    def sync(self):
        _check(lib().augur_lda_sync(self._h))

    def loglik(self, raise_on_degenerate=False):
        lj, lm = C.c_double(), C.c_double()
        _check(lib().augur_lda_loglik(self._h, C.byref(lj), C.byref(lm)),
               allow=() if raise_on_degenerate else (ERR_DEGENERATE,))
        return lj.value, lm.value

    def get_state(self, z=True, theta=True, phi=True):
        za = self._arr.empty((self.N,), "i32") if z else None
        kind = "f64" if self.state_f64 else "f32"
        ta = self._arr.empty((self.D, self.K), kind) if theta else None
        pa = self._arr.empty((self.V, self.K), kind) if phi else None
        sw = C.c_int64()
        get = lib().augur_lda_get_state_f64 if self.state_f64 else lib().augur_lda_get_state
        _check(get(self._h, _ptr(za), _ptr(ta), _ptr(pa), C.byref(sw)))
        return za, ta, pa, sw.value

    def set_state(self, z=None, theta=None, phi=None, sweep=None):
        za = self._arr.input(z, "i32", self.N)
        kind = "f64" if self.state_f64 else "f32"
        ta = self._arr.input(theta, kind, self.D * self.K)
        pa = self._arr.input(phi, kind, self.V * self.K)
        put = lib().augur_lda_set_state_f64 if self.state_f64 else lib().augur_lda_set_state
        _check(put(self._h, _ptr(za), _ptr(ta), _ptr(pa), -1 if sweep is None else int(sweep)))

    def get_counts(self):
        n_dk = self._arr.empty((self.D, self.K), "i32")
        n_wk = self._arr.empty((self.V, self.K), "i32")
        _check(lib().augur_lda_get_counts(self._h, _ptr(n_dk), _ptr(n_wk)))
        return n_dk, n_wk

    def get_degenerate(self):
        c = C.c_int64()
        _check(lib().augur_lda_get_degenerate(self._h, C.byref(c)))
        return c.value


class GMM:
    """augur_gmm_* handle."""

    def __init__(self, K, alpha, prior_sd, sigma, seed, x, device=0, stream=None,
                 device_ptrs=False, var_shape=0.0, var_scale=0.0):
        self._h = None
        self._arr = _Arrays(device_ptrs, device)
        xa = self._arr.input(x, "f32")
        if xa.ndim != 2:
            raise ValueError("x must be [N][dim]")
        self.N, self.dim, self.K = int(xa.shape[0]), int(xa.shape[1]), int(K)
        cfg = GmmConfig(self.N, self.dim, self.K, float(alpha), float(prior_sd), float(sigma),
                        float(var_shape), float(var_scale), int(seed), int(device),
                        _stream_handle(stream),
                        PTRS_DEVICE if device_ptrs else 0)
        h = C.c_void_p()
        _check(lib().augur_gmm_create(C.byref(cfg), _ptr(xa), C.byref(h)))
        self._h = h

    def close(self):
        if self._h is not None:
            lib().augur_gmm_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:  # interpreter shutdown: the module globals may be gone
            pass

    def sweep(self, n=1):
        _check(lib().augur_gmm_sweep(self._h, int(n)))

    def set_graph(self, on):
        _check(lib().augur_gmm_set_graph(self._h, 1 if on else 0))

    def step_sample_z(self):
        _check(lib().augur_gmm_step_sample_z(self._h))

    def sweep_profile(self, n=1):
        ms = (C.c_double * 4)()
        _check(lib().augur_gmm_sweep_profile(self._h, int(n), ms))
        return dict(zip(("sample_z", "stats", "resample", "sweep"), list(ms)))

    def step_stats(self):
        _check(lib().augur_gmm_step_stats(self._h))

    def step_resample(self):
        _check(lib().augur_gmm_step_resample(self._h))

    def step_finish(self):
        _check(lib().augur_gmm_step_finish(self._h))

    def sync(self):
        _check(lib().augur_gmm_sync(self._h))

    def loglik(self, raise_on_degenerate=False):
        lj = C.c_double()
        _check(lib().augur_gmm_loglik(self._h, C.byref(lj)),
               allow=() if raise_on_degenerate else (ERR_DEGENERATE,))
        return lj.value

    def get_state(self):
        z = self._arr.empty((self.N,), "i32")
        pi = self._arr.empty((self.K,), "f32")
        mu = self._arr.empty((self.K, self.dim), "f32")
        sw = C.c_int64()
        _check(lib().augur_gmm_get_state(self._h, _ptr(z), _ptr(pi), _ptr(mu), C.byref(sw)))
        return z, pi, mu, sw.value

    def set_state(self, z=None, pi=None, mu=None, sweep=None):
        za = self._arr.input(z, "i32", self.N)
        pa = self._arr.input(pi, "f32", self.K)
        ma = self._arr.input(mu, "f32", self.K * self.dim)
        _check(lib().augur_gmm_set_state(self._h, _ptr(za), _ptr(pa), _ptr(ma),
                                         -1 if sweep is None else int(sweep)))

    def get_var(self):
        var = self._arr.empty((self.K,), "f32")
        _check(lib().augur_gmm_get_var(self._h, _ptr(var)))
        return var

    def set_var(self, var):
        _check(lib().augur_gmm_set_var(self._h, _ptr(self._arr.input(var, "f32", self.K))))

    def get_stats(self):
        n_k = self._arr.empty((self.K,), "i32")
        s_k = self._arr.empty((self.K, self.dim), "f64")
        _check(lib().augur_gmm_get_stats(self._h, _ptr(n_k), _ptr(s_k)))
        return n_k, s_k

    def get_degenerate(self):
        c = C.c_int64()
        _check(lib().augur_gmm_get_degenerate(self._h, C.byref(c)))
        return c.value


class MHRegression:
    """augur_mhreg_* handle: random-walk Metropolis-Hastings over theta = (w, b, tau)."""

    def __init__(self, x, y, prior_sd, tau_shape, tau_scale, x_lo, x_hi, step, seed, theta0=None,
                 device=0, stream=None, device_ptrs=False):
        self._h = None
        self._arr = _Arrays(device_ptrs, device)
        xa = self._arr.input(x, "f32")
        if xa.ndim != 2:
            raise ValueError("x must be [N][K]")
        self.N, self.K = int(xa.shape[0]), int(xa.shape[1])
        ya = self._arr.input(y, "f32", self.N)
        ta = self._arr.input(theta0, "f64", self.K + 2)
        cfg = MhRegConfig(self.N, self.K, float(prior_sd), float(tau_shape), float(tau_scale),
                          float(x_lo), float(x_hi), float(step), int(seed), int(device),
                          _stream_handle(stream), PTRS_DEVICE if device_ptrs else 0)
        h = C.c_void_p()
        _check(lib().augur_mhreg_create(C.byref(cfg), _ptr(xa), _ptr(ya), _ptr(ta), C.byref(h)))
        self._h = h

    def close(self):
        if self._h is not None:
            lib().augur_mhreg_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:  # interpreter shutdown: the module globals may be gone
            pass

    def run(self, n, trace=False):
        tr = self._arr.empty((int(n), self.K + 3), "f64") if trace else None
        _check(lib().augur_mhreg_run(self._h, int(n), _ptr(tr)))
        return tr

    def get_state(self):
        theta = self._arr.empty((self.K + 2,), "f64")
        lf, si, acc = C.c_double(), C.c_int64(), C.c_int64()
        _check(lib().augur_mhreg_get_state(self._h, _ptr(theta), C.byref(lf), C.byref(si),
                                           C.byref(acc)))
        return theta, lf.value, si.value, acc.value

    def set_state(self, theta=None, step_index=None):
        ta = self._arr.input(theta, "f64", self.K + 2)
        _check(lib().augur_mhreg_set_state(self._h, _ptr(ta), -1 if step_index is None else int(step_index)))

    def set_schedule(self, schedule):
        _check(lib().augur_mhreg_set_schedule(self._h, int(schedule)))

    def sync(self):
        _check(lib().augur_mhreg_sync(self._h))

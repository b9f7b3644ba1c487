"""Seeded synthetic inputs: LDA corpora and Gaussian-mixture point clouds.

This module only draws inputs (with numpy's own generator); it contains none of
the sampler's arithmetic and is the one module that both the HIP path's callers
and the oracle's tests use.  The corpora stand in for the paper's Simple English
Wikipedia corpus (Sect. "Experimental study": 48,556 documents, 37,276 words,
about 3.3M tokens), which is not available; they are drawn from the LDA
generative program of Fig. 1 at the sizes of the benchmark configurations.
"""
import numpy as np

LDA_CONFIGS = {
    # name: D docs, V words, K topics, Poisson mean length, alpha, beta, Zipf exponent, sweeps
    "tiny": dict(D=100, V=500, K=10, mean_len=50, alpha=0.1, beta=0.01, zipf=None, sweeps=20,
                 seed=20131212),
    "medium": dict(D=20_000, V=50_000, K=100, mean_len=150, alpha=0.1, beta=0.01, zipf=1.1,
                   sweeps=50, seed=20131214),
    "large": dict(D=300_000, V=100_000, K=200, mean_len=250, alpha=0.05, beta=0.01, zipf=1.1,
                  sweeps=20, seed=20131215),
    "widek": dict(D=50_000, V=100_000, K=1000, mean_len=200, alpha=0.01, beta=0.01, zipf=1.1,
                  sweeps=10, seed=20131216),
    # the shape of the paper's own corpus (Sect. "Experimental study": 47,556 training documents,
    # 37,276 words, about 3.2M tokens), generated with 100 topics; used for the run over the
    # number of topics (the paper's figure of run time against K)
    "paper_shape": dict(D=47_556, V=37_276, K=100, mean_len=68, alpha=0.1, beta=0.01, zipf=1.1,
                        sweeps=50, seed=20131217),
}

GMM_CONFIG = dict(N=1_000_000, dim=8, K=16, alpha=1.0, prior_sd=10.0, sigma=1.0, sweeps=50,
                  seed=20131213)


def _bits(n):
    return max(1, int(np.ceil(np.log2(max(2, n)))))


def lda_corpus(D, V, K, mean_len, alpha, beta, seed, zipf=None, return_truth=False, **_unused):
    """Draw a corpus from the LDA generative process.

    theta*_d ~ Dirichlet(alpha 1_K); phi*_k ~ Dirichlet(b) with b = beta 1_V, or, with a Zipf
    exponent s, b_v = beta V q(rank(v)), q(r) proportional to r^-s and rank a seeded random
    permutation of the vocabulary (mean concentration beta, Zipf-shaped word marginals, word id
    uncorrelated with frequency).  Document lengths are Poisson(mean_len), zeros redrawn.
    Tokens of a document are in random order.  Returns doc_len int32[D], w int32[N] (doc-major)
    and, if asked, the generating z, theta, phi ([V][K]).
    """
    rng = np.random.default_rng(seed)
    doc_len = rng.poisson(mean_len, size=D).astype(np.int64)
    while True:
        zero = doc_len == 0
        if not zero.any():
            break
        doc_len[zero] = rng.poisson(mean_len, size=int(zero.sum()))
    N = int(doc_len.sum())

    # topic counts per document, in chunks of documents to bound memory
    counts = np.zeros((D, K), dtype=np.int32)
    theta_true = np.zeros((D, K), dtype=np.float32) if return_truth else None
    step = 50_000
    for lo in range(0, D, step):
        hi = min(D, lo + step)
        g = rng.standard_gamma(alpha, size=(hi - lo, K))
        s = g.sum(axis=1, keepdims=True)
        bad = s[:, 0] <= 0
        if bad.any():
            g[bad] = 1.0
            s = g.sum(axis=1, keepdims=True)
        th = g / s
        # guard the multinomial against rounding: renormalise so each row sums to <= 1
        th /= th.sum(axis=1, keepdims=True) * (1.0 + 1e-12)
        counts[lo:hi] = rng.multinomial(doc_len[lo:hi], th)
        if return_truth:
            theta_true[lo:hi] = th
    n_k = counts.sum(axis=0, dtype=np.int64)

    if zipf is None:
        b = np.full(V, beta, dtype=np.float64)
    else:
        rank = rng.permutation(V)
        q = (rank + 1.0) ** (-float(zipf))
        q /= q.sum()
        b = beta * V * q

    bd, bw, bz = _bits(D), _bits(V), _bits(K)
    pack_z = return_truth and (bd + bw + bz <= 56)
    br = 64 - bd - bw - (bz if pack_z else 0)
    keys = np.empty(N, dtype=np.uint64)
    phi_true = np.zeros((V, K), dtype=np.float32) if return_truth else None
    docs = np.arange(D, dtype=np.uint64)
    pos = 0
    for k in range(K):
        g = rng.standard_gamma(b)
        s = g.sum()
        if s <= 0:
            g = b.copy()
            s = g.sum()
        cdf = np.cumsum(g)
        if return_truth:
            phi_true[:, k] = g / s
        n = int(n_k[k])
        if n == 0:
            continue
        words = np.searchsorted(cdf, rng.random(n) * cdf[-1], side="right").astype(np.uint64)
        np.minimum(words, np.uint64(V - 1), out=words)
        d_of = np.repeat(docs, counts[:, k])
        r = rng.integers(0, 1 << min(br, 32), size=n, dtype=np.uint64)
        key = (d_of << np.uint64(64 - bd)) | (r << np.uint64(64 - bd - min(br, 32)))
        if pack_z:
            key |= np.uint64(k) << np.uint64(bw)
        key |= words
        keys[pos:pos + n] = key
        pos += n
    assert pos == N
    keys.sort()
    w = (keys & np.uint64((1 << bw) - 1)).astype(np.int32)
    out = dict(doc_len=doc_len.astype(np.int32), w=w, N=N)
    if return_truth:
        out["theta"] = theta_true
        out["phi"] = phi_true
        if pack_z:
            out["z"] = ((keys >> np.uint64(bw)) & np.uint64((1 << bz) - 1)).astype(np.int32)
    return out


def categorical_mixture(N, K, V, seed, alpha=0.5, beta=0.5, return_truth=False):
    """N draws from the categorical mixture of the paper's supplement: weights ~ Dirichlet(beta 1_K),
    K component distributions over V values ~ Dirichlet(alpha 1_V), z_i ~ Categorical(weights),
    x_i ~ Categorical(component z_i).  In LDA terms: one document of N tokens."""
    rng = np.random.default_rng(seed)
    weights = rng.dirichlet(np.full(K, beta))
    comp = rng.dirichlet(np.full(V, alpha), size=K)
    z = rng.choice(K, size=N, p=weights).astype(np.int32)
    x = np.empty(N, dtype=np.int32)
    for k in range(K):
        mine = np.nonzero(z == k)[0]
        cdf = np.cumsum(comp[k])
        x[mine] = np.minimum(np.searchsorted(cdf, rng.random(mine.size) * cdf[-1], side="right"), V - 1)
    out = dict(x=x)
    if return_truth:
        out.update(z=z, weights=weights.astype(np.float32), comp=comp.astype(np.float32))
    return out


def gmm_points(N, dim, K, seed, mean_sd=10.0, sigma=1.0, return_truth=False, **_unused):
    """N points in R^dim from K unit-covariance components: means ~ N(0, mean_sd^2 I),
    weights ~ Dirichlet(1), x = mu_z + sigma * N(0, I).  fp32."""
    rng = np.random.default_rng(seed)
    mu = rng.normal(0.0, mean_sd, size=(K, dim))
    pi = rng.dirichlet(np.ones(K))
    z = rng.choice(K, size=N, p=pi).astype(np.int32)
    x = (mu[z] + sigma * rng.standard_normal((N, dim))).astype(np.float32)
    out = dict(x=x)
    if return_truth:
        out.update(z=z, mu=mu.astype(np.float32), pi=pi.astype(np.float32))
    return out


def regression_data(N, K, seed, l=-1.0, u=1.0, noise_var=0.25, return_truth=False):
    """(x, y) from the multivariate regression program: x_nk ~ Uniform(l, u), weights and bias
    ~ N(0, 1) (tighter than the model's prior so that y stays O(1)), y_n ~ N(x_n . w + b,
    noise_var).  fp32.  Stands in for the UCI regression tables of the paper's supplement
    (roughly 300 to 5000 rows, 6 to 11 predictors), which are not available here."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(K)
    b = rng.standard_normal()
    x = rng.uniform(l, u, size=(N, K)).astype(np.float32)
    y = (x.astype(np.float64) @ w + b + np.sqrt(noise_var) * rng.standard_normal(N)).astype(np.float32)
    out = dict(x=x, y=y)
    if return_truth:
        out.update(w=w, b=b, tau=noise_var)
    return out

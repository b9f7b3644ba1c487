// Oracle for the uncollapsed Gibbs sweep of Augur (arXiv 1312.3613) on LDA and
// on a Gaussian mixture (known covariance, or unknown per-component variances),
// and for its data-parallel random-walk Metropolis-Hastings sampler on the
// multivariate regression model.
//
// THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded CPU
// program written from the paper's statement of the method so that a reader can
// check it against the paper by eye.  It shares no code with the HIP library and
// must never be called from the product path: only tests, the smoke check and
// the benchmark's cpu_baseline leg load it.
//
// What it follows, passage by passage:
//   * LDA model (Fig. 1): phi_k ~ Dirichlet(beta), theta_m ~ Dirichlet(alpha),
//     z_mj ~ Categorical(theta_m), w_mj ~ Categorical(phi_{z_mj}).
//   * Sect. 4.2 (Gibbs): theta_m | z ~ Dirichlet(alpha + c_m), c_m[k] = number of
//     z in document m equal to k; phi_k | z, w ~ Dirichlet(beta + c_k), c_k[v] =
//     number of tokens of word v assigned to topic k; each z_mj is discrete, so
//     its univariate conditional, proportional to theta_m[k] * phi_k[w_mj], is
//     computed exactly and sampled from; all z are conditionally independent.
//     A sweep draws z, then theta, then phi (the order of the conditioning
//     superscripts tau+1 in Sect. 4.2).
//   * Sect. 4.3, Alg. 1 and App. B, Alg. 2: a Dirichlet draw is a vector of
//     Gamma draws divided by its sum (the sum of the draws, not of the
//     parameters, which is how Alg. 2 prints it).
//   * Sect. 4.1: densities are evaluated in log space, the per-datum terms
//     summed.
//   * Supplementary Gaussian mixture (Fig. "GMM"), in the variant with known
//     covariance sigma^2 I, prior N(0, prior_sd^2 I) on the means and a
//     symmetric Dirichlet(alpha) on the weights; and as printed, with an
//     inverse-Gamma prior on each component's variance.
//   * Sect. 4.1 and Fig. "regression": the function f proportional to the
//     posterior of the regression model is the product of the priors of b, tau
//     and w_k and of the per-datum terms p(x_n) p(y_n | x_n . w + b, tau),
//     evaluated in log space; a library random-walk Metropolis-Hastings
//     sampler (no tuning; supplement, "Multivariate Regression") drives it.
//
// Readings where the paper is silent (all listed in the design notes):
//   * phi is stored [V][K] (row = word), theta [D][K].
//   * Gamma(a,1) draws use Marsaglia & Tsang (2000), in fp64, returned as ln g.
//   * Random numbers: Philox4x32-10 (Salmon et al., SC'11), key = 64-bit seed,
//     counter = (index lo, index hi, sweep, stream<<24 | attempt).
//   * Inverse-CDF rule: z = smallest k with C_k > u*S (strict), C_k the running
//     sum of the K products in index order, accumulated in fp64.
//   * Stored theta/phi/pi are fp32, clamped below at FLT_MIN.  LDA also has an fp64
//     state mode (the exported functions ending in _f64): theta and phi are stored
//     as doubles, clamped below at DBL_MIN; everything else is the same code.  The
//     paper's experiments ran in double precision (Sect. 5, experimental setup).
//
// parity pins: every exported function is pinned by tests/test_oracle_*.py
// (brute-force enumeration, closed-form posteriors, library CDFs, invariants).

#include <cfloat>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

namespace {

// ---------------------------------------------------------------- Philox4x32-10
// One round: two 32x32->64 products; ten rounds; the key is bumped by the
// Weyl constants between rounds (Salmon, Moraes, Dror, Shaw, SC'11).
void philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
  uint32_t k0 = key_in[0], k1 = key_in[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += W0; k1 += W1; }
    const uint64_t p0 = M0 * (uint64_t)c0;
    const uint64_t p1 = M1 * (uint64_t)c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    const uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

enum Stream : uint32_t {
  STREAM_INIT_Z = 0, STREAM_Z = 1, STREAM_THETA = 2, STREAM_PHI = 3,
  STREAM_GMM_PI = 4, STREAM_GMM_MU = 5, STREAM_GMM_VAR = 6, STREAM_MH_PROPOSAL = 7,
  STREAM_MH_ACCEPT = 8
};

// The block of four 32-bit words belonging to (seed, variable index, sweep,
// stream, attempt).
void random_block(uint64_t seed, uint64_t index, uint32_t sweep, uint32_t stream,
                  uint32_t attempt, uint32_t out[4]) {
  const uint32_t ctr[4] = {(uint32_t)index, (uint32_t)(index >> 32), sweep,
                           (stream << 24) | (attempt & 0xFFFFFFu)};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  philox4x32_10(ctr, key, out);
}

// Uniform on (0,1) with 23 random bits, an odd multiple of 2^-24: exact in fp32.
double uniform24(uint32_t r) { return (double)(2u * (r >> 9) + 1u) * (1.0 / 16777216.0); }
// Uniform on (0,1) with 32 random bits, (r + 1/2) 2^-32: exact in fp64.
double uniform32(uint32_t r) { return ((double)r + 0.5) * (1.0 / 4294967296.0); }

// The uniform that decides variable i of a per-datum categorical draw: four
// consecutive variables share one Philox block.
double datum_uniform(uint64_t seed, uint64_t i, uint32_t sweep, uint32_t stream) {
  uint32_t r[4];
  random_block(seed, i >> 2, sweep, stream, 0, r);
  return uniform24(r[i & 3]);
}
uint32_t datum_word(uint64_t seed, uint64_t i, uint32_t sweep, uint32_t stream) {
  uint32_t r[4];
  random_block(seed, i >> 2, sweep, stream, 0, r);
  return r[i & 3];
}

const double TWO_PI = 6.283185307179586476925286766559;

// Standard normal by Box-Muller (cosine branch) from words 0 and 1 of a block.
double normal_from(const uint32_t r[4]) {
  return std::sqrt(-2.0 * std::log(uniform32(r[0]))) * std::cos(TWO_PI * uniform32(r[1]));
}

const int GAMMA_ATTEMPT_CAP = 64;

// ln of a Gamma(a,1) draw, a > 0, by Marsaglia & Tsang's method: with
// d = a - 1/3, c = 1/sqrt(9d), propose v = (1 + c x)^3 for x ~ N(0,1), accept
// with the squeeze U < 1 - 0.0331 x^4 or the exact test
// ln U < x^2/2 + d (1 - v + ln v); the draw is d v.  For a < 1 the draw for
// a + 1 is multiplied by U'^(1/a).  Attempt j uses Philox block j of the
// variable: word 0,1 -> x, word 2 -> U, word 3 -> U'.
double gamma_log_draw(double a, uint64_t seed, uint64_t index, uint32_t sweep,
                      uint32_t stream, int* attempts, int* capped) {
  const double a1 = (a < 1.0) ? a + 1.0 : a;
  const double d = a1 - 1.0 / 3.0;
  const double c = 1.0 / std::sqrt(9.0 * d);
  for (int j = 0; j < GAMMA_ATTEMPT_CAP; ++j) {
    uint32_t r[4];
    random_block(seed, index, sweep, stream, (uint32_t)j, r);
    const double x = normal_from(r);
    const double t = 1.0 + c * x;
    if (t <= 0.0) continue;
    const double v = t * t * t;
    const double U = uniform32(r[2]);
    const double x2 = x * x;
    bool accept = U < 1.0 - 0.0331 * x2 * x2;
    if (!accept) accept = std::log(U) < 0.5 * x2 + d * (1.0 - v + std::log(v));
    if (accept) {
      double lg = std::log(d) + std::log(v);
      if (a < 1.0) lg += std::log(uniform32(r[3])) / a;
      if (attempts) *attempts = j + 1;
      return lg;
    }
  }
  if (attempts) *attempts = GAMMA_ATTEMPT_CAP;
  if (capped) *capped += 1;
  return std::log(d);
}

// Normalise K log-Gamma draws into a Dirichlet draw stored as T (fp32 or fp64) with
// the floor at T's smallest positive normal number (FLT_MIN or DBL_MIN).  lg has
// stride `stride`; out has the same stride.
template <typename T>
void normalise_log_draws(const double* lg, int64_t n, int64_t stride, T* out) {
  double m = lg[0];
  for (int64_t j = 1; j < n; ++j) if (lg[j * stride] > m) m = lg[j * stride];
  double s = 0.0;
  for (int64_t j = 0; j < n; ++j) s += std::exp(lg[j * stride] - m);
  const double L = m + std::log(s);
  const double floor_t = (double)std::numeric_limits<T>::min();
  for (int64_t j = 0; j < n; ++j) {
    double p = std::exp(lg[j * stride] - L);
    if (p < floor_t) p = floor_t;
    out[j * stride] = (T)p;
  }
}

// Smallest k with cdf[k] > t; if rounding leaves none, the largest k whose
// increment is positive.
int inverse_cdf(const double* cdf, int K, double t) {
  for (int k = 0; k < K; ++k) if (cdf[k] > t) return k;
  for (int k = K - 1; k > 0; --k) if (cdf[k] > cdf[k - 1]) return k;
  return 0;
}

// Running sums C_k of theta_d[k] * phi[v][k], products and sums in fp64.
template <typename T>
void lda_token_cdf(const T* theta_d, const T* phi_v, int K, double* cdf) {
  double C = 0.0;
  for (int k = 0; k < K; ++k) {
    C += (double)theta_d[k] * (double)phi_v[k];
    cdf[k] = C;
  }
}

// ln Dirichlet(x; a 1_n) density, x given as fp32 or fp64 with stride.
template <typename T>
double log_dirichlet_sym(const T* x, int64_t n, int64_t stride, double a) {
  double s = 0.0;
  for (int64_t j = 0; j < n; ++j) s += std::log((double)x[j * stride]);
  return std::lgamma((double)n * a) - (double)n * std::lgamma(a) + (a - 1.0) * s;
}

// Unnormalised log weights of the mixture conditional of point x:
// ln pi_k - |x - mu_k|^2 / (2 sigma^2), then exponentiated relative to the
// maximum and accumulated into a running sum.
void gmm_point_cdf(const float* x, const float* pi, const float* mu, int K, int dim,
                   double sigma, double* cdf) {
  std::vector<double> l(K);
  double m = -INFINITY;
  for (int k = 0; k < K; ++k) {
    double q = 0.0;
    for (int j = 0; j < dim; ++j) {
      const double df = (double)x[j] - (double)mu[(int64_t)k * dim + j];
      q += df * df;
    }
    l[k] = std::log((double)pi[k]) - q / (2.0 * sigma * sigma);
    if (l[k] > m) m = l[k];
  }
  double C = 0.0;
  for (int k = 0; k < K; ++k) {
    C += std::exp(l[k] - m);
    cdf[k] = C;
  }
}

// Mixture conditional with a variance per component:
// ln pi_k - (dim/2) ln var_k - |x - mu_k|^2 / (2 var_k).
void gmmuv_point_cdf(const float* x, const float* pi, const float* mu, const float* var, int K,
                     int dim, double* cdf) {
  std::vector<double> l(K);
  double m = -INFINITY;
  for (int k = 0; k < K; ++k) {
    double q = 0.0;
    for (int j = 0; j < dim; ++j) {
      const double df = (double)x[j] - (double)mu[(int64_t)k * dim + j];
      q += df * df;
    }
    const double v = (double)var[k];
    l[k] = std::log((double)pi[k]) - 0.5 * (double)dim * std::log(v) - q / (2.0 * v);
    if (l[k] > m) m = l[k];
  }
  double C = 0.0;
  for (int k = 0; k < K; ++k) {
    C += std::exp(l[k] - m);
    cdf[k] = C;
  }
}

}  // namespace

extern "C" {

// ------------------------------------------------------------ random primitives
void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}
void orc_random_block(uint64_t seed, uint64_t index, uint32_t sweep, uint32_t stream,
                      uint32_t attempt, uint32_t* out) {
  random_block(seed, index, sweep, stream, attempt, out);
}
double orc_uniform24(uint32_t r) { return uniform24(r); }
double orc_uniform32(uint32_t r) { return uniform32(r); }
// u[i] for variables first..first+n-1 of a per-datum stream.
void orc_datum_uniforms(uint64_t seed, uint64_t first, int64_t n, uint32_t sweep,
                        uint32_t stream, double* u) {
  for (int64_t i = 0; i < n; ++i) u[i] = datum_uniform(seed, first + (uint64_t)i, sweep, stream);
}
// n independent N(0,1) draws: variable index first+i, attempt 0.
void orc_normals(uint64_t seed, uint64_t first, int64_t n, uint32_t sweep, uint32_t stream,
                 double* out) {
  for (int64_t i = 0; i < n; ++i) {
    uint32_t r[4];
    random_block(seed, first + (uint64_t)i, sweep, stream, 0, r);
    out[i] = normal_from(r);
  }
}
// ln Gamma(a[i]) draws for variable index first+i; attempts may be NULL.
// Returns the number of draws that hit the attempt cap.
int orc_gamma_log_draws(const double* a, int64_t n, uint64_t seed, uint64_t first,
                        uint32_t sweep, uint32_t stream, double* lg, int32_t* attempts) {
  int capped = 0;
  for (int64_t i = 0; i < n; ++i) {
    int att = 0;
    lg[i] = gamma_log_draw(a[i], seed, first + (uint64_t)i, sweep, stream, &att, &capped);
    if (attempts) attempts[i] = att;
  }
  return capped;
}

// -------------------------------------------------------------------------- LDA
// Default initial assignment: z_i = floor(K r / 2^32), r the token's word of the
// init stream (sweep index 0).
void orc_lda_init_z(int64_t N, int32_t K, uint64_t seed, int32_t* z) {
  for (int64_t i = 0; i < N; ++i) {
    const uint32_t r = datum_word(seed, (uint64_t)i, 0, STREAM_INIT_Z);
    z[i] = (int32_t)(((uint64_t)r * (uint64_t)K) >> 32);
  }
}

// Counting phase (Sect. 4.2): c_m and c_k as two tables, n_dk[D][K], n_wk[V][K].
void orc_lda_count(int32_t D, int32_t V, int32_t K, const int64_t* doc_off, const int32_t* w,
                   const int32_t* z, int32_t* n_dk, int32_t* n_wk) {
  std::memset(n_dk, 0, sizeof(int32_t) * (size_t)D * K);
  std::memset(n_wk, 0, sizeof(int32_t) * (size_t)V * K);
  for (int32_t d = 0; d < D; ++d)
    for (int64_t i = doc_off[d]; i < doc_off[d + 1]; ++i) {
      n_dk[(int64_t)d * K + z[i]] += 1;
      n_wk[(int64_t)w[i] * K + z[i]] += 1;
    }
}

}  // extern "C"

namespace {

// Gibbs step for every z (Sect. 4.2, last conditional): token i of document d
// with word v draws from p(k) proportional to theta[d][k] * phi[v][k].
// Returns the number of tokens whose conditional had zero or non-finite mass
// (those take z = floor(u K)).
template <typename T>
int64_t lda_sample_z_impl(int32_t D, int32_t K, const int64_t* doc_off, const int32_t* w,
                         const T* theta, const T* phi, uint64_t seed,
                         uint32_t sweep, int32_t* z) {
  std::vector<double> cdf(K);
  int64_t degenerate = 0;
  for (int32_t d = 0; d < D; ++d) {
    for (int64_t i = doc_off[d]; i < doc_off[d + 1]; ++i) {
      lda_token_cdf(theta + (int64_t)d * K, phi + (int64_t)w[i] * K, K, cdf.data());
      const double S = cdf[K - 1];
      const double u = datum_uniform(seed, (uint64_t)i, sweep, STREAM_Z);
      if (!(S > 0.0) || !std::isfinite(S)) {
        z[i] = (int32_t)(u * (double)K);
        ++degenerate;
      } else {
        z[i] = inverse_cdf(cdf.data(), K, u * S);
      }
    }
  }
  return degenerate;
}

// The running sums C_k and the threshold t = u S of one token, for judging a
// disagreement about its draw.
template <typename T>
void lda_token_cdf_impl(int32_t K, const T* theta_d, const T* phi_v, uint64_t seed,
                       uint64_t token, uint32_t sweep, double* cdf, double* t) {
  lda_token_cdf(theta_d, phi_v, K, cdf);
  *t = datum_uniform(seed, token, sweep, STREAM_Z) * cdf[K - 1];
}

// theta_d ~ Dirichlet(alpha + n_dk[d][.]) for every document (App. B, Alg. 2).
// Variable index of entry (d,k) is d*K + k.  Returns capped-draw count.
template <typename T>
int lda_resample_theta_impl(int32_t D, int32_t K, double alpha, const int32_t* n_dk,
                           uint64_t seed, uint32_t sweep, T* theta) {
  std::vector<double> lg(K);
  int capped = 0;
  for (int32_t d = 0; d < D; ++d) {
    for (int32_t k = 0; k < K; ++k) {
      const int64_t e = (int64_t)d * K + k;
      lg[k] = gamma_log_draw(alpha + (double)n_dk[e], seed, (uint64_t)e, sweep, STREAM_THETA,
                             nullptr, &capped);
    }
    normalise_log_draws(lg.data(), K, 1, theta + (int64_t)d * K);
  }
  return capped;
}

// phi_k ~ Dirichlet(beta + n_wk[.][k]) for every topic (Sect. 4.3, Alg. 1): a
// V x K matrix of Gamma draws, each topic's column normalised over the words.
// Variable index of entry (v,k) is v*K + k.
template <typename T>
int lda_resample_phi_impl(int32_t V, int32_t K, double beta, const int32_t* n_wk,
                         uint64_t seed, uint32_t sweep, T* phi) {
  std::vector<double> lg((size_t)V * K);
  int capped = 0;
  for (int32_t v = 0; v < V; ++v)
    for (int32_t k = 0; k < K; ++k) {
      const int64_t e = (int64_t)v * K + k;
      lg[e] = gamma_log_draw(beta + (double)n_wk[e], seed, (uint64_t)e, sweep, STREAM_PHI,
                             nullptr, &capped);
    }
  for (int32_t k = 0; k < K; ++k) normalise_log_draws(lg.data() + k, V, K, phi + k);
  return capped;
}

// One sweep tau -> tau+1 in the order z, counts, theta, phi, all with sweep
// index `sweep`.
template <typename T>
int64_t lda_sweep_impl(int32_t D, int32_t V, int32_t K, double alpha, double beta,
                      const int64_t* doc_off, const int32_t* w, uint64_t seed, uint32_t sweep,
                      int32_t* z, T* theta, T* phi, int32_t* n_dk, int32_t* n_wk) {
  const int64_t deg = lda_sample_z_impl<T>(D, K, doc_off, w, theta, phi, seed, sweep, z);
  orc_lda_count(D, V, K, doc_off, w, z, n_dk, n_wk);
  lda_resample_theta_impl<T>(D, K, alpha, n_dk, seed, sweep, theta);
  lda_resample_phi_impl<T>(V, K, beta, n_wk, seed, sweep, phi);
  return deg;
}

// The same sweep with phi observed (Fig. 3, second call: the variable set
// {"phi"} is added to the observed ones): only z and theta are inferred.
template <typename T>
int64_t lda_sweep_phi_observed_impl(int32_t D, int32_t V, int32_t K, double alpha,
                                   const int64_t* doc_off, const int32_t* w, uint64_t seed,
                                   uint32_t sweep, int32_t* z, T* theta, const T* phi,
                                   int32_t* n_dk, int32_t* n_wk_scratch) {
  const int64_t deg = lda_sample_z_impl<T>(D, K, doc_off, w, theta, phi, seed, sweep, z);
  orc_lda_count(D, V, K, doc_off, w, z, n_dk, n_wk_scratch);
  lda_resample_theta_impl<T>(D, K, alpha, n_dk, seed, sweep, theta);
  return deg;
}

// Default initial state: z from the init stream, counts, then theta and phi
// drawn from their conditionals with sweep index 0.
template <typename T>
void lda_init_impl(int32_t D, int32_t V, int32_t K, double alpha, double beta,
                  const int64_t* doc_off, const int32_t* w, uint64_t seed, int32_t* z,
                  T* theta, T* phi, int32_t* n_dk, int32_t* n_wk) {
  orc_lda_init_z(doc_off[D], K, seed, z);
  orc_lda_count(D, V, K, doc_off, w, z, n_dk, n_wk);
  lda_resample_theta_impl<T>(D, K, alpha, n_dk, seed, 0, theta);
  lda_resample_phi_impl<T>(V, K, beta, n_wk, seed, 0, phi);
}

// Log joint density ln p(phi, theta, z, w) of Fig. 1's program and the log
// likelihood of the words with z summed out, ln p(w | theta, phi).
template <typename T>
void lda_loglik_impl(int32_t D, int32_t V, int32_t K, double alpha, double beta,
                    const int64_t* doc_off, const int32_t* w, const int32_t* z,
                    const T* theta, const T* phi, double* log_joint,
                    double* log_marginal_w) {
  double prior = 0.0;
  for (int32_t d = 0; d < D; ++d) prior += log_dirichlet_sym(theta + (int64_t)d * K, K, 1, alpha);
  for (int32_t k = 0; k < K; ++k) prior += log_dirichlet_sym(phi + k, V, K, beta);
  double lik = 0.0, marg = 0.0;
  std::vector<double> cdf(K);
  for (int32_t d = 0; d < D; ++d)
    for (int64_t i = doc_off[d]; i < doc_off[d + 1]; ++i) {
      const T* th = theta + (int64_t)d * K;
      const T* ph = phi + (int64_t)w[i] * K;
      lik += std::log((double)th[z[i]]) + std::log((double)ph[z[i]]);
      lda_token_cdf(th, ph, K, cdf.data());
      marg += std::log(cdf[K - 1]);
    }
  if (log_joint) *log_joint = prior + lik;
  if (log_marginal_w) *log_marginal_w = marg;
}

}  // namespace

extern "C" {

// The exported LDA functions: fp32 state (the benchmark's) and fp64 state (_f64).
#define ORC_LDA_EXPORTS(SUFFIX, T)                                                                      \
  int64_t orc_lda_sample_z##SUFFIX(int32_t D, int32_t K, const int64_t* doc_off, const int32_t* w,      \
                                   const T* theta, const T* phi, uint64_t seed, uint32_t sweep,         \
                                   int32_t* z) {                                                        \
    return lda_sample_z_impl<T>(D, K, doc_off, w, theta, phi, seed, sweep, z);                          \
  }                                                                                                     \
  void orc_lda_token_cdf##SUFFIX(int32_t K, const T* theta_d, const T* phi_v, uint64_t seed,            \
                                 uint64_t token, uint32_t sweep, double* cdf, double* t) {              \
    lda_token_cdf_impl<T>(K, theta_d, phi_v, seed, token, sweep, cdf, t);                               \
  }                                                                                                     \
  int orc_lda_resample_theta##SUFFIX(int32_t D, int32_t K, double alpha, const int32_t* n_dk,           \
                                     uint64_t seed, uint32_t sweep, T* theta) {                         \
    return lda_resample_theta_impl<T>(D, K, alpha, n_dk, seed, sweep, theta);                           \
  }                                                                                                     \
  int orc_lda_resample_phi##SUFFIX(int32_t V, int32_t K, double beta, const int32_t* n_wk,              \
                                   uint64_t seed, uint32_t sweep, T* phi) {                             \
    return lda_resample_phi_impl<T>(V, K, beta, n_wk, seed, sweep, phi);                                \
  }                                                                                                     \
  int64_t orc_lda_sweep##SUFFIX(int32_t D, int32_t V, int32_t K, double alpha, double beta,             \
                                const int64_t* doc_off, const int32_t* w, uint64_t seed,                \
                                uint32_t sweep, int32_t* z, T* theta, T* phi, int32_t* n_dk,            \
                                int32_t* n_wk) {                                                        \
    return lda_sweep_impl<T>(D, V, K, alpha, beta, doc_off, w, seed, sweep, z, theta, phi, n_dk, n_wk); \
  }                                                                                                     \
  int64_t orc_lda_sweep_phi_observed##SUFFIX(int32_t D, int32_t V, int32_t K, double alpha,             \
                                             const int64_t* doc_off, const int32_t* w, uint64_t seed,   \
                                             uint32_t sweep, int32_t* z, T* theta, const T* phi,        \
                                             int32_t* n_dk, int32_t* n_wk_scratch) {                    \
    return lda_sweep_phi_observed_impl<T>(D, V, K, alpha, doc_off, w, seed, sweep, z, theta, phi, n_dk, \
                                          n_wk_scratch);                                                \
  }                                                                                                     \
  void orc_lda_init##SUFFIX(int32_t D, int32_t V, int32_t K, double alpha, double beta,                 \
                            const int64_t* doc_off, const int32_t* w, uint64_t seed, int32_t* z,        \
                            T* theta, T* phi, int32_t* n_dk, int32_t* n_wk) {                           \
    lda_init_impl<T>(D, V, K, alpha, beta, doc_off, w, seed, z, theta, phi, n_dk, n_wk);                \
  }                                                                                                     \
  void orc_lda_loglik##SUFFIX(int32_t D, int32_t V, int32_t K, double alpha, double beta,               \
                              const int64_t* doc_off, const int32_t* w, const int32_t* z,               \
                              const T* theta, const T* phi, double* log_joint,                          \
                              double* log_marginal_w) {                                                 \
    lda_loglik_impl<T>(D, V, K, alpha, beta, doc_off, w, z, theta, phi, log_joint, log_marginal_w);     \
  }
ORC_LDA_EXPORTS(, float)
ORC_LDA_EXPORTS(_f64, double)
#undef ORC_LDA_EXPORTS

// ------------------------------------------------------------- Gaussian mixture
void orc_gmm_init_z(int64_t N, int32_t K, uint64_t seed, int32_t* z) {
  orc_lda_init_z(N, K, seed, z);
}

int64_t orc_gmm_sample_z(int64_t N, int32_t dim, int32_t K, double sigma, const float* x,
                         const float* pi, const float* mu, uint64_t seed, uint32_t sweep,
                         int32_t* z) {
  std::vector<double> cdf(K);
  int64_t degenerate = 0;
  for (int64_t i = 0; i < N; ++i) {
    gmm_point_cdf(x + i * dim, pi, mu, K, dim, sigma, cdf.data());
    const double S = cdf[K - 1];
    const double u = datum_uniform(seed, (uint64_t)i, sweep, STREAM_Z);
    if (!(S > 0.0) || !std::isfinite(S)) {
      z[i] = (int32_t)(u * (double)K);
      ++degenerate;
    } else {
      z[i] = inverse_cdf(cdf.data(), K, u * S);
    }
  }
  return degenerate;
}

void orc_gmm_point_cdf(int32_t dim, int32_t K, double sigma, const float* x_i, const float* pi,
                       const float* mu, uint64_t seed, uint64_t point, uint32_t sweep,
                       double* cdf, double* t) {
  gmm_point_cdf(x_i, pi, mu, K, dim, sigma, cdf);
  *t = datum_uniform(seed, point, sweep, STREAM_Z) * cdf[K - 1];
}

// Sufficient statistics: n_k and s_k[j] = sum of x_i[j] over points with z_i = k.
void orc_gmm_stats(int64_t N, int32_t dim, int32_t K, const float* x, const int32_t* z,
                   int32_t* n_k, double* s_k) {
  std::memset(n_k, 0, sizeof(int32_t) * (size_t)K);
  for (int64_t e = 0; e < (int64_t)K * dim; ++e) s_k[e] = 0.0;
  for (int64_t i = 0; i < N; ++i) {
    n_k[z[i]] += 1;
    for (int32_t j = 0; j < dim; ++j) s_k[(int64_t)z[i] * dim + j] += (double)x[i * dim + j];
  }
}

// pi ~ Dirichlet(alpha + n); mu_k[j] ~ Normal with precision
// lambda = 1/prior_sd^2 + n_k/sigma^2 and mean (s_k[j]/sigma^2)/lambda
// (Normal-Normal conjugacy, known variance).
int orc_gmm_resample(int32_t dim, int32_t K, double alpha, double prior_sd, double sigma,
                     const int32_t* n_k, const double* s_k, uint64_t seed, uint32_t sweep,
                     float* pi, float* mu) {
  std::vector<double> lg(K);
  int capped = 0;
  for (int32_t k = 0; k < K; ++k)
    lg[k] = gamma_log_draw(alpha + (double)n_k[k], seed, (uint64_t)k, sweep, STREAM_GMM_PI,
                           nullptr, &capped);
  normalise_log_draws(lg.data(), K, 1, pi);
  for (int32_t k = 0; k < K; ++k) {
    const double lambda = 1.0 / (prior_sd * prior_sd) + (double)n_k[k] / (sigma * sigma);
    for (int32_t j = 0; j < dim; ++j) {
      const int64_t e = (int64_t)k * dim + j;
      uint32_t r[4];
      random_block(seed, (uint64_t)e, sweep, STREAM_GMM_MU, 0, r);
      const double mean = (s_k[e] / (sigma * sigma)) / lambda;
      mu[e] = (float)(mean + normal_from(r) / std::sqrt(lambda));
    }
  }
  return capped;
}

int64_t orc_gmm_sweep(int64_t N, int32_t dim, int32_t K, double alpha, double prior_sd,
                      double sigma, const float* x, uint64_t seed, uint32_t sweep, int32_t* z,
                      float* pi, float* mu, int32_t* n_k, double* s_k) {
  const int64_t deg = orc_gmm_sample_z(N, dim, K, sigma, x, pi, mu, seed, sweep, z);
  orc_gmm_stats(N, dim, K, x, z, n_k, s_k);
  orc_gmm_resample(dim, K, alpha, prior_sd, sigma, n_k, s_k, seed, sweep, pi, mu);
  return deg;
}

void orc_gmm_init(int64_t N, int32_t dim, int32_t K, double alpha, double prior_sd,
                  double sigma, const float* x, uint64_t seed, int32_t* z, float* pi, float* mu,
                  int32_t* n_k, double* s_k) {
  orc_gmm_init_z(N, K, seed, z);
  orc_gmm_stats(N, dim, K, x, z, n_k, s_k);
  orc_gmm_resample(dim, K, alpha, prior_sd, sigma, n_k, s_k, seed, 0, pi, mu);
}

// ln p(pi, mu, z, x) = ln Dir(pi; alpha) + sum_kj ln N(mu_kj; 0, prior_sd^2)
//                      + sum_i [ ln pi_{z_i} + ln N(x_i; mu_{z_i}, sigma^2 I) ].
double orc_gmm_loglik(int64_t N, int32_t dim, int32_t K, double alpha, double prior_sd,
                      double sigma, const float* x, const int32_t* z, const float* pi,
                      const float* mu) {
  const double LN_2PI = 1.8378770664093454835606594728112;
  double lj = log_dirichlet_sym(pi, K, 1, alpha);
  for (int64_t e = 0; e < (int64_t)K * dim; ++e) {
    const double m = (double)mu[e];
    lj += -0.5 * LN_2PI - std::log(prior_sd) - m * m / (2.0 * prior_sd * prior_sd);
  }
  for (int64_t i = 0; i < N; ++i) {
    const int32_t k = z[i];
    double q = 0.0;
    for (int32_t j = 0; j < dim; ++j) {
      const double df = (double)x[i * dim + j] - (double)mu[(int64_t)k * dim + j];
      q += df * df;
    }
    lj += std::log((double)pi[k]) - 0.5 * (double)dim * LN_2PI - (double)dim * std::log(sigma) -
          q / (2.0 * sigma * sigma);
  }
  return lj;
}

// ------------------------- Gaussian mixture with unknown component variances
// The supplementary Gaussian mixture as printed: a variance per component with an
// inverse-Gamma prior, var_k ~ InverseGamma(a0, b0) (the listing's
// InverseGamma(1,1)); here for points in R^dim with covariance var_k I.
// Conditionals (all conjugate): z as above with var_k; pi ~ Dirichlet(alpha + n);
// mu_kj ~ N((s_kj / var_k) / lambda_k, 1 / lambda_k), lambda_k = 1/prior_sd^2 +
// n_k / var_k; var_k ~ InverseGamma(a0 + n_k dim / 2, b0 + SS_k / 2) with
// SS_k = sum over points of component k of |x_i - mu_k|^2 (the new mu).
// An inverse-Gamma draw is rate / Gamma(shape) (variance stream, index k).
int64_t orc_gmmuv_sample_z(int64_t N, int32_t dim, int32_t K, const float* x, const float* pi,
                           const float* mu, const float* var, uint64_t seed, uint32_t sweep,
                           int32_t* z) {
  std::vector<double> cdf(K);
  int64_t degenerate = 0;
  for (int64_t i = 0; i < N; ++i) {
    gmmuv_point_cdf(x + i * dim, pi, mu, var, K, dim, cdf.data());
    const double S = cdf[K - 1];
    const double u = datum_uniform(seed, (uint64_t)i, sweep, STREAM_Z);
    if (!(S > 0.0) || !std::isfinite(S)) {
      z[i] = (int32_t)(u * (double)K);
      ++degenerate;
    } else {
      z[i] = inverse_cdf(cdf.data(), K, u * S);
    }
  }
  return degenerate;
}

void orc_gmmuv_point_cdf(int32_t dim, int32_t K, const float* x_i, const float* pi,
                         const float* mu, const float* var, uint64_t seed, uint64_t point,
                         uint32_t sweep, double* cdf, double* t) {
  gmmuv_point_cdf(x_i, pi, mu, var, K, dim, cdf);
  *t = datum_uniform(seed, point, sweep, STREAM_Z) * cdf[K - 1];
}

int orc_gmmuv_resample(int64_t N, int32_t dim, int32_t K, double alpha, double prior_sd, double a0,
                       double b0, const float* x, const int32_t* z, const int32_t* n_k,
                       const double* s_k, uint64_t seed, uint32_t sweep, float* pi, float* mu,
                       float* var) {
  std::vector<double> lg(K);
  int capped = 0;
  for (int32_t k = 0; k < K; ++k)
    lg[k] = gamma_log_draw(alpha + (double)n_k[k], seed, (uint64_t)k, sweep, STREAM_GMM_PI,
                           nullptr, &capped);
  normalise_log_draws(lg.data(), K, 1, pi);
  for (int32_t k = 0; k < K; ++k) {
    const double v = (double)var[k];
    const double lambda = 1.0 / (prior_sd * prior_sd) + (double)n_k[k] / v;
    for (int32_t j = 0; j < dim; ++j) {
      const int64_t e = (int64_t)k * dim + j;
      uint32_t r[4];
      random_block(seed, (uint64_t)e, sweep, STREAM_GMM_MU, 0, r);
      mu[e] = (float)((s_k[e] / v) / lambda + normal_from(r) / std::sqrt(lambda));
    }
  }
  std::vector<double> ss(K, 0.0);
  for (int64_t i = 0; i < N; ++i) {
    const int32_t k = z[i];
    for (int32_t j = 0; j < dim; ++j) {
      const double df = (double)x[i * dim + j] - (double)mu[(int64_t)k * dim + j];
      ss[k] += df * df;
    }
  }
  for (int32_t k = 0; k < K; ++k) {
    const double shape = a0 + 0.5 * (double)n_k[k] * (double)dim;
    const double rate = b0 + 0.5 * ss[k];
    const double lgam = gamma_log_draw(shape, seed, (uint64_t)k, sweep, STREAM_GMM_VAR, nullptr,
                                       &capped);
    double v = std::exp(std::log(rate) - lgam);
    if (v < (double)FLT_MIN) v = (double)FLT_MIN;
    var[k] = (float)v;
  }
  return capped;
}

int64_t orc_gmmuv_sweep(int64_t N, int32_t dim, int32_t K, double alpha, double prior_sd, double a0,
                        double b0, const float* x, uint64_t seed, uint32_t sweep, int32_t* z,
                        float* pi, float* mu, float* var, int32_t* n_k, double* s_k) {
  const int64_t deg = orc_gmmuv_sample_z(N, dim, K, x, pi, mu, var, seed, sweep, z);
  orc_gmm_stats(N, dim, K, x, z, n_k, s_k);
  orc_gmmuv_resample(N, dim, K, alpha, prior_sd, a0, b0, x, z, n_k, s_k, seed, sweep, pi, mu, var);
  return deg;
}

// Initial state: z from the init stream, var_k = b0 / a0, then pi, mu and var
// from their conditionals with sweep index 0.
void orc_gmmuv_init(int64_t N, int32_t dim, int32_t K, double alpha, double prior_sd, double a0,
                    double b0, const float* x, uint64_t seed, int32_t* z, float* pi, float* mu,
                    float* var, int32_t* n_k, double* s_k) {
  orc_gmm_init_z(N, K, seed, z);
  for (int32_t k = 0; k < K; ++k) var[k] = (float)(b0 / a0);
  orc_gmm_stats(N, dim, K, x, z, n_k, s_k);
  orc_gmmuv_resample(N, dim, K, alpha, prior_sd, a0, b0, x, z, n_k, s_k, seed, 0, pi, mu, var);
}

// ln p(pi, mu, var, z, x): Dirichlet, Normal and inverse-Gamma priors plus the
// per-point terms ln pi_z + ln N(x_i; mu_z, var_z I).
double orc_gmmuv_loglik(int64_t N, int32_t dim, int32_t K, double alpha, double prior_sd, double a0,
                        double b0, const float* x, const int32_t* z, const float* pi,
                        const float* mu, const float* var) {
  const double LN_2PI = 1.8378770664093454835606594728112;
  double lj = log_dirichlet_sym(pi, K, 1, alpha);
  for (int64_t e = 0; e < (int64_t)K * dim; ++e) {
    const double m = (double)mu[e];
    lj += -0.5 * LN_2PI - std::log(prior_sd) - m * m / (2.0 * prior_sd * prior_sd);
  }
  for (int32_t k = 0; k < K; ++k) {
    const double v = (double)var[k];
    lj += a0 * std::log(b0) - std::lgamma(a0) - (a0 + 1.0) * std::log(v) - b0 / v;
  }
  for (int64_t i = 0; i < N; ++i) {
    const int32_t k = z[i];
    const double v = (double)var[k];
    double q = 0.0;
    for (int32_t j = 0; j < dim; ++j) {
      const double df = (double)x[i * dim + j] - (double)mu[(int64_t)k * dim + j];
      q += df * df;
    }
    lj += std::log((double)pi[k]) - 0.5 * (double)dim * (LN_2PI + std::log(v)) - q / (2.0 * v);
  }
  return lj;
}

// --------------------------- Metropolis-Hastings on the multivariate regression
// Model (Fig. "regression"): w_k ~ N(0, prior_sd^2), b ~ N(0, prior_sd^2),
// tau ~ InverseGamma(a0, b0), x_nk ~ Uniform(l, u), y_n ~ N(x_n . w + b, tau).
// The second argument of the listing's Gaussian is read as a variance (it is
// what the inverse-Gamma prior is put on).  Parameters are fp64 and ordered
// theta = (w_0 .. w_{K-1}, b, tau); the data are fp32.
//
// ln f (Sect. 4.1): sum of the log prior terms and of the N per-datum terms
// ln p(x_n) + ln N(y_n; x_n . w + b, tau), with ln p(x_n) = -K ln(u - l).
// tau <= 0 has density zero: -infinity.
double orc_mhreg_logf(int64_t N, int32_t K, const float* x, const float* y, const double* theta,
                      double prior_sd, double a0, double b0, double l, double u) {
  const double LN_2PI = 1.8378770664093454835606594728112;
  const double* w = theta;
  const double b = theta[K], tau = theta[K + 1];
  if (!(tau > 0.0)) return -INFINITY;
  double lf = 0.0;
  for (int32_t k = 0; k <= K; ++k)  // w_0 .. w_{K-1} and b
    lf += -0.5 * LN_2PI - std::log(prior_sd) - theta[k] * theta[k] / (2.0 * prior_sd * prior_sd);
  lf += a0 * std::log(b0) - std::lgamma(a0) - (a0 + 1.0) * std::log(tau) - b0 / tau;
  for (int64_t n = 0; n < N; ++n) {
    double mean = b;
    for (int32_t k = 0; k < K; ++k) mean += w[k] * (double)x[n * K + k];
    const double r = (double)y[n] - mean;
    lf += -(double)K * std::log(u - l) - 0.5 * (LN_2PI + std::log(tau)) - r * r / (2.0 * tau);
  }
  return lf;
}

// Proposal of step t (t = 1, 2, ...): every parameter moves at once,
// theta'_e = theta_e + step * n_e, n_e the standard normal of block (index e,
// sweep t) of the proposal stream.
void orc_mhreg_propose(int32_t K, const double* theta, double step, uint64_t seed, uint32_t t,
                       double* proposal) {
  for (int32_t e = 0; e < K + 2; ++e) {
    uint32_t r[4];
    random_block(seed, (uint64_t)e, t, STREAM_MH_PROPOSAL, 0, r);
    proposal[e] = theta[e] + step * normal_from(r);
  }
}

// Uniform of the acceptance test of step t.
double orc_mhreg_accept_uniform(uint64_t seed, uint32_t t) {
  uint32_t r[4];
  random_block(seed, 0, t, STREAM_MH_ACCEPT, 0, r);
  return uniform32(r[0]);
}

// n_steps steps from (theta, *logf), the first with index first_step.  The
// random walk is symmetric, so a proposal is accepted iff ln u < ln f(theta') -
// ln f(theta).  trace (may be NULL) receives theta and ln f after every step,
// K + 3 doubles a row.  Returns the number of accepted proposals.
int64_t orc_mhreg_run(int64_t N, int32_t K, const float* x, const float* y, double prior_sd,
                      double a0, double b0, double l, double u, double step, uint64_t seed,
                      uint32_t first_step, int64_t n_steps, double* theta, double* logf,
                      double* trace) {
  std::vector<double> prop(K + 2);
  int64_t accepted = 0;
  for (int64_t s = 0; s < n_steps; ++s) {
    const uint32_t t = first_step + (uint32_t)s;
    orc_mhreg_propose(K, theta, step, seed, t, prop.data());
    const double lp = orc_mhreg_logf(N, K, x, y, prop.data(), prior_sd, a0, b0, l, u);
    if (std::log(orc_mhreg_accept_uniform(seed, t)) < lp - *logf) {
      for (int32_t e = 0; e < K + 2; ++e) theta[e] = prop[e];
      *logf = lp;
      ++accepted;
    }
    if (trace) {
      for (int32_t e = 0; e < K + 2; ++e) trace[s * (K + 3) + e] = theta[e];
      trace[s * (K + 3) + K + 2] = *logf;
    }
  }
  return accepted;
}

}  // extern "C"

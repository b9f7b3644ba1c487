// Gaussian mixture (the supplementary Gaussian mixture model of arXiv
// 1312.3613): Gibbs sweep over z, the weights pi (Dirichlet-categorical
// conjugacy), the means mu (Normal-Normal conjugacy) and, when the variances
// are unknown, var_k (inverse-Gamma-Normal conjugacy, covariance var_k I), as
// HIP kernels behind the augur_gmm_* C ABI.  With the variance known every
// component has covariance sigma^2 I.
//
// Device layout: x float[N][dim], z int32[N], pi float[K], mu float[K][dim],
// var float[K], n_k int32[K], s_k double[K][dim], q_k double[K] (sum of |x_i|^2,
// unknown variances only).  The z conditional is evaluated in fp64 from the
// fp32 state (N * K * dim fused multiply-adds per sweep is small).
#include "common.hpp"

#include <algorithm>
#include <new>
#include <vector>

using namespace augur;

namespace {

constexpr int kRedBlocks = 512;
// Points per block of the statistics kernel.  Small chunks: a block has only K (dim + 1)
// working threads, so it takes many resident blocks to fill a CU (measured at 10^6 points,
// K dim = 128: 88 us with 1024-point chunks).
constexpr int kStatChunk = 256;     // fp32 staging
constexpr int kStatChunkSq = 256;   // with the sum of squares (fp64 staging)

__global__ __launch_bounds__(256) void gmm_init_z_kernel(int32_t* __restrict__ z, int64_t N, int K,
                                                          uint64_t seed) {
  const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (b * 4 >= N) return;
  const U4 r = random_block(seed, (uint64_t)b, 0, kStreamInitZ, 0);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int64_t i = b * 4 + e;
    if (i < N) z[i] = (int32_t)(((uint64_t)word_of(r, e) * (uint64_t)K) >> 32);
  }
}

// ln pi_k - (dim/2) ln v_k - |x - mu_k|^2 / (2 v_k) for one point; mu, the
// constant part lw_k and 1/(2 v_k) in LDS.  With the variance known the
// (dim/2) ln v term is the same for every k and left out.
// DIM > 0: the dimension is known at compile time and the point is held in registers as
// doubles (converted once, not once per component); DIM == 0: any dimension, read from memory.
template <int DIM>
struct PointOf {
  double v[DIM > 0 ? DIM : 1];
  const float* p;
  __device__ __forceinline__ explicit PointOf(const float* __restrict__ xi) : p(xi) {
    if (DIM > 0) {
#pragma unroll
      for (int j = 0; j < DIM; ++j) v[j] = (double)xi[j];
    }
  }
};
template <int DIM>
__device__ __forceinline__ double gmm_logw(const PointOf<DIM>& x, const double* mu_s,
                                           const double* lw_s, const double* inv2v_s, int k,
                                           int dim) {
  double q = 0.0;
  if (DIM > 0) {
#pragma unroll
    for (int j = 0; j < DIM; ++j) {
      const double df = x.v[j] - mu_s[k * DIM + j];
      q += df * df;
    }
  } else {
    for (int j = 0; j < dim; ++j) {
      const double df = (double)x.p[j] - mu_s[k * dim + j];
      q += df * df;
    }
  }
  return lw_s[k] - q * inv2v_s[k];
}

// Gibbs step for z: p(k) proportional to pi_k N(x_i; mu_k, v_k I), v_k = var[k]
// or sigma^2 for every k when var is NULL, drawn by
// inverse CDF over the weights exp(l_k - max l), running sum in index order.
// One thread per point.  With kCache the K log-weights (then weights) of a
// thread wait in its own LDS column between the three passes (max, total,
// search); without it (K too large for LDS) they are recomputed.  Thread t of a
// group of four computes the Philox block shared by points 4b..4b+3
// redundantly (cheap at this size).
template <bool kCache, int DIM>
__global__ __launch_bounds__(256) void gmm_sample_z_kernel(
    const float* __restrict__ x, const float* __restrict__ pi, const float* __restrict__ mu,
    const float* __restrict__ var, int32_t* __restrict__ z, int64_t N, int dim, int K, double sigma,
    uint64_t seed, SweepRef sweep_ref, unsigned long long* __restrict__ n_degenerate) {
  const uint32_t sweep = sweep_ref.get();
  extern __shared__ double sh[];
  double* mu_s = sh;                // [K][dim]
  double* lw_s = sh + K * dim;      // [K]
  double* inv2v_s = lw_s + K;       // [K]
  double* col = inv2v_s + K + threadIdx.x;  // [K][256]: this thread's column (kCache only)
  for (int e = threadIdx.x; e < K * dim; e += blockDim.x) mu_s[e] = (double)mu[e];
  for (int k = threadIdx.x; k < K; k += blockDim.x) {
    const double lp = log((double)pi[k]);
    if (var != nullptr) {
      const double v = (double)var[k];
      lw_s[k] = lp - 0.5 * (double)dim * log(v);
      inv2v_s[k] = 1.0 / (2.0 * v);
    } else {
      lw_s[k] = lp;
      inv2v_s[k] = 1.0 / (2.0 * sigma * sigma);
    }
  }
  __syncthreads();
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  const PointOf<DIM> xi(x + i * dim);
  double m = -INFINITY;
  bool has_nan = false;
  for (int k = 0; k < K; ++k) {
    const double l = gmm_logw(xi, mu_s, lw_s, inv2v_s, k, dim);
    if (kCache) col[k * 256] = l;
    has_nan = has_nan || !(l == l);
    m = l > m ? l : m;
  }
  const U4 blk = random_block(seed, (uint64_t)(i >> 2), sweep, kStreamZ, 0);
  const uint32_t r = word_of(blk, (uint32_t)(i & 3));
  int zi;
  if (kCache && K <= 32) {
    // Only components within 40 of the largest log-weight get their exponential.  The others
    // weigh less than e^-40 = 4e-18 of the largest term (which is exactly 1): their sum does not
    // reach half an ulp of the total, and none of them can be drawn except where u S lies
    // within that distance of a boundary.  A point typically keeps one to three components, and
    // each lane walks its own list, so a wave takes as many turns as its busiest lane has
    // components instead of K.
    uint32_t live = 0;
    for (int k = 0; k < K; ++k) live |= col[k * 256] - m > -40.0 ? 1u << k : 0u;
    double S = has_nan ? NAN : 0.0;
    for (uint32_t todo = live; __any(todo != 0);) {
      if (todo != 0) {
        const int k = __ffs(todo) - 1;
        todo &= todo - 1;
        const double p = exp(col[k * 256] - m);
        col[k * 256] = p;
        S += p;
      }
    }
    if (!(S > 0.0) || !(S <= DBL_MAX)) {
      zi = u24_times(r, K);
      atomicAdd(n_degenerate, 1ULL);
    } else {
      const double t = (double)u24(r) * S;
      double C = 0.0;
      zi = -1;
      int last = 0;
      for (uint32_t todo = live; __any(todo != 0);) {
        if (todo != 0) {
          const int k = __ffs(todo) - 1;
          todo &= todo - 1;
          const double Cn = C + col[k * 256];
          if (Cn > C) last = k;
          C = Cn;
          if (zi < 0 && C > t) zi = k;
        }
      }
      if (zi < 0) zi = last;
    }
  } else {
    double S = 0.0;
    for (int k = 0; k < K; ++k) {
      const double p = exp((kCache ? col[k * 256] : gmm_logw(xi, mu_s, lw_s, inv2v_s, k, dim)) - m);
      if (kCache) col[k * 256] = p;
      S += p;
    }
    if (!(S > 0.0) || !(S <= DBL_MAX)) {
      zi = u24_times(r, K);
      atomicAdd(n_degenerate, 1ULL);
    } else {
      const double t = (double)u24(r) * S;
      double C = 0.0;
      int last = 0;
      zi = -1;
      for (int k = 0; k < K; ++k) {
        const double p = kCache ? col[k * 256] : exp(gmm_logw(xi, mu_s, lw_s, inv2v_s, k, dim) - m);
        const double Cn = C + p;
        if (Cn > C) last = k;
        C = Cn;
        if (zi < 0 && C > t) zi = k;
      }
      if (zi < 0) zi = last;
    }
  }
  z[i] = zi;
}

// Sufficient statistics, deterministic: a block stages a chunk of points in
// LDS, W values a point: its dim coordinates and, with kSumSq, |x_i|^2 (the
// staged values are then fp64).  Thread (k, j) walks the chunk in index order
// and adds value j of point i when z_i = k (0.0 otherwise, which leaves the sum
// unchanged), thread (k, 0) also counts.  Per-block partials are then added in
// block order, one workgroup per (k, j) pair with a fixed reduction tree.
template <bool kSumSq>
__global__ __launch_bounds__(256) void gmm_stats_partial_kernel(
    const float* __restrict__ x, const int32_t* __restrict__ z, int64_t N, int dim, int K,
    double* __restrict__ part_s, int32_t* __restrict__ part_n) {
  using T = typename std::conditional<kSumSq, double, float>::type;
  extern __shared__ __align__(8) unsigned char raw[];
  constexpr int kChunk = kSumSq ? kStatChunkSq : kStatChunk;
  const int W = dim + (kSumSq ? 1 : 0);
  T* xs = reinterpret_cast<T*>(raw);                                  // [chunk][W]
  int32_t* zs = reinterpret_cast<int32_t*>(xs + (size_t)kChunk * W);  // [chunk]
  const int64_t p0 = (int64_t)blockIdx.x * kChunk;
  const int n = (int)std::min<int64_t>(kChunk, N - p0);
  if (kSumSq) {
    for (int e = threadIdx.x; e < n; e += blockDim.x) {
      double q = 0.0;
      for (int j = 0; j < dim; ++j) {
        const double v = (double)x[(p0 + e) * dim + j];
        xs[e * W + j] = (T)v;
        q += v * v;
      }
      xs[e * W + dim] = (T)q;
    }
  } else {
    for (int e = threadIdx.x; e < n * dim; e += blockDim.x) xs[e] = (T)x[p0 * dim + e];
  }
  for (int e = threadIdx.x; e < n; e += blockDim.x) zs[e] = z[p0 + e];
  __syncthreads();
  for (int pair = threadIdx.x; pair < K * W; pair += blockDim.x) {
    const int k = pair / W, j = pair - k * W;
    double s = 0.0;
    int32_t c = 0;
#pragma unroll 8
    for (int e = 0; e < n; ++e) {
      const bool mine = zs[e] == k;
      s += mine ? (double)xs[e * W + j] : 0.0;
      c += mine ? 1 : 0;
    }
    part_s[(size_t)pair * gridDim.x + blockIdx.x] = s;  // [pair][block]: the merge reads rows
    if (j == 0) part_n[(size_t)k * gridDim.x + blockIdx.x] = c;
  }
}

// The same partial sums for K <= 64 without walking the whole chunk per component: the
// chunk's points are first grouped by component, in index order (a stable counting sort: per
// wave one ballot per component gives every point its rank among the wave's points of that
// component; the four waves' counts are then prefixed), and thread (k, j) adds only the points
// of its component, in the same order as the walk above, so the sums are bit-identical.
// 256 threads, one per point of the chunk.
template <bool kSumSq>
__global__ __launch_bounds__(256) void gmm_stats_grouped_kernel(
    const float* __restrict__ x, const int32_t* __restrict__ z, int64_t N, int dim, int K,
    double* __restrict__ part_s, int32_t* __restrict__ part_n) {
  using T = typename std::conditional<kSumSq, double, float>::type;
  extern __shared__ __align__(8) unsigned char raw[];
  constexpr int kChunk = 256;
  const int W = dim + (kSumSq ? 1 : 0);
  T* xs = reinterpret_cast<T*>(raw);  // [chunk][W]
  __shared__ uint16_t order[kChunk];  // points grouped by component, index order inside a group
  __shared__ int32_t cnt[4][64];      // per wave: points of each component
  __shared__ int32_t first[65];       // start of each component's group in order[]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t p0 = (int64_t)blockIdx.x * kChunk;
  const int n = (int)std::min<int64_t>(kChunk, N - p0);
  if (kSumSq) {
    if (tid < n) {
      double q = 0.0;
      for (int j = 0; j < dim; ++j) {
        const double v = (double)x[(p0 + tid) * dim + j];
        xs[tid * W + j] = (T)v;
        q += v * v;
      }
      xs[tid * W + dim] = (T)q;
    }
  } else {
    for (int e = tid; e < n * dim; e += 256) xs[e] = (T)x[p0 * dim + e];
  }
  const int zi = tid < n ? z[p0 + tid] : -1;
  int rank = 0;
  for (int k = 0; k < K; ++k) {
    const unsigned long long m = __ballot(zi == k);
    if (zi == k) rank = __popcll(m & ((1ULL << lane) - 1ULL));
    if (lane == 0) cnt[wave][k] = __popcll(m);
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int k = 0; k < K; ++k) {
      first[k] = run;
      run += cnt[0][k] + cnt[1][k] + cnt[2][k] + cnt[3][k];
    }
    first[K] = run;
  }
  __syncthreads();
  if (zi >= 0) {
    int at = first[zi] + rank;
    for (int w = 0; w < wave; ++w) at += cnt[w][zi];
    order[at] = (uint16_t)tid;
  }
  __syncthreads();
  for (int pair = tid; pair < K * W; pair += 256) {
    const int k = pair / W, j = pair - k * W;
    const int e0 = first[k], e1 = first[k + 1];
    double s = 0.0;
    for (int e = e0; e < e1; ++e) s += (double)xs[(int)order[e] * W + j];
    part_s[(size_t)pair * gridDim.x + blockIdx.x] = s;  // [pair][block]: the merge reads rows
    if (j == 0) part_n[(size_t)k * gridDim.x + blockIdx.x] = e1 - e0;
  }
}

// W = dim (+ 1 with the sum of squares, whose totals go to q_k).
__global__ __launch_bounds__(256) void gmm_stats_merge_kernel(const double* __restrict__ part_s,
                                                               const int32_t* __restrict__ part_n,
                                                               int nblk, int dim, int W, int K,
                                                               double* __restrict__ s_k,
                                                               double* __restrict__ q_k,
                                                               int32_t* __restrict__ n_k) {
  __shared__ double ss[256];
  __shared__ int32_t sn[256];
  const int pair = blockIdx.x;  // one workgroup per (k, j)
  const int k = pair / W, j = pair - k * W;
  const bool count = j == 0;
  double s = 0.0;
  int32_t c = 0;
  for (int b = threadIdx.x; b < nblk; b += 256) {
    s += part_s[(size_t)pair * nblk + b];
    if (count) c += part_n[(size_t)k * nblk + b];
  }
  ss[threadIdx.x] = s;
  sn[threadIdx.x] = c;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      ss[threadIdx.x] += ss[threadIdx.x + o];
      sn[threadIdx.x] += sn[threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    if (j < dim) s_k[k * dim + j] = ss[0];
    else q_k[k] = ss[0];
    if (count) n_k[k] = sn[0];
  }
}

// pi ~ Dirichlet(alpha + n) from K log-domain Gamma draws normalised in index
// order; mu_kj ~ N(mean, 1/lambda), lambda = 1/prior_sd^2 + n_k/v_k,
// mean = (s_kj / v_k) / lambda, v_k the component's current variance (sigma^2
// when var is NULL).  With unknown variances then
// var_k ~ InverseGamma(a0 + n_k dim / 2, b0 + SS_k / 2), SS_k the sum of
// |x_i - mu_k|^2 over the component's points with the NEW (fp32) mean, taken
// from the sufficient statistics as q_k - 2 mu_k . s_k + n_k |mu_k|^2 in fp64,
// and drawn as exp(ln rate - ln G), G ~ Gamma(shape).  One block.
__global__ __launch_bounds__(256) void gmm_resample_kernel(
    const int32_t* __restrict__ n_k, const double* __restrict__ s_k, const double* __restrict__ q_k,
    float* __restrict__ pi, float* __restrict__ mu, float* __restrict__ var, int dim, int K,
    double alpha, double prior_sd, double sigma, double a0, double b0, uint64_t seed, SweepRef sweep_ref,
    unsigned long long* __restrict__ n_capped) {
  const uint32_t sweep = sweep_ref.get();
  extern __shared__ double lg[];                            // [K]
  float* mu_new = reinterpret_cast<float*>(lg + K);         // [K][dim]
  bool capped = false;
  for (int k = threadIdx.x; k < K; k += blockDim.x)
    lg[k] = gamma_log_draw(alpha + (double)n_k[k], seed, (uint64_t)k, sweep, kStreamGmmPi, capped);
  __syncthreads();
  for (int k = threadIdx.x; k < K; k += blockDim.x) {
    double m = lg[0];
    for (int q = 1; q < K; ++q) m = lg[q] > m ? lg[q] : m;
    double s = 0.0;
    for (int q = 0; q < K; ++q) s += exp(lg[q] - m);
    double p = exp(lg[k] - (m + log(s)));
    p = p < (double)FLT_MIN ? (double)FLT_MIN : p;
    pi[k] = (float)p;
  }
  for (int e = threadIdx.x; e < K * dim; e += blockDim.x) {
    const int k = e / dim;
    const double v = var != nullptr ? (double)var[k] : sigma * sigma;
    const double lambda = 1.0 / (prior_sd * prior_sd) + (double)n_k[k] / v;
    const double mean = (s_k[e] / v) / lambda;
    const U4 b = random_block(seed, (uint64_t)e, sweep, kStreamGmmMu, 0);
    const float m = (float)(mean + normal_from(b) / sqrt(lambda));
    mu[e] = m;
    mu_new[e] = m;
  }
  if (var != nullptr) {
    __syncthreads();  // every mean above read the old variances; the new means are in LDS
    for (int k = threadIdx.x; k < K; k += blockDim.x) {
      const double n = (double)n_k[k];
      double dot = 0.0, sq = 0.0;
      for (int j = 0; j < dim; ++j) {
        const double m = (double)mu_new[k * dim + j];
        dot += m * s_k[k * dim + j];
        sq += m * m;
      }
      double ss = q_k[k] - 2.0 * dot + n * sq;
      ss = ss > 0.0 ? ss : 0.0;
      const double shape = a0 + 0.5 * n * (double)dim;
      const double rate = b0 + 0.5 * ss;
      const double lgam = gamma_log_draw(shape, seed, (uint64_t)k, sweep, kStreamGmmVar, capped);
      double v = exp(log(rate) - lgam);
      v = v < (double)FLT_MIN ? (double)FLT_MIN : v;
      var[k] = (float)v;
    }
  }
  if (capped) atomicAdd(n_capped, 1ULL);
}

// Per-point terms of the log joint: ln pi_z + ln N(x_i; mu_z, v_z I), v_k =
// var[k] or sigma^2 when var is NULL.
__global__ __launch_bounds__(256) void gmm_loglik_kernel(
    const float* __restrict__ x, const int32_t* __restrict__ z, const float* __restrict__ pi,
    const float* __restrict__ mu, const float* __restrict__ var, int64_t N, int dim, double sigma,
    double* __restrict__ part) {
  __shared__ double smem[8];
  const double LN_2PI = 1.8378770664093454835606594728112;
  double s = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int k = z[i];
    double q = 0.0;
    for (int j = 0; j < dim; ++j) {
      const double df = (double)x[i * dim + j] - (double)mu[k * dim + j];
      q += df * df;
    }
    if (var != nullptr) {
      const double v = (double)var[k];
      s += log((double)pi[k]) - 0.5 * (double)dim * (LN_2PI + log(v)) - q / (2.0 * v);
    } else {
      s += log((double)pi[k]) - 0.5 * (double)dim * LN_2PI - (double)dim * log(sigma) -
           q / (2.0 * sigma * sigma);
    }
  }
  block_partial_sum(s, part, smem);
}

__global__ __launch_bounds__(256) void gmm_check_range_kernel(const int32_t* __restrict__ a,
                                                               int64_t n, int32_t hi,
                                                               unsigned long long* __restrict__ bad) {
  unsigned long long c = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x)
    if (a[i] < 0 || a[i] >= hi) ++c;
  if (c) atomicAdd(bad, c);
}

}  // namespace

struct augur_gmm {
  augur_gmm_config cfg{};
  hipStream_t stream = nullptr;
  double alpha = 0, prior_sd = 0, sigma = 0, a0 = 0, b0 = 0;
  bool unknown_var = false;
  float *x = nullptr, *pi = nullptr, *mu = nullptr, *var = nullptr;  // var: unknown variances only
  int32_t *z = nullptr, *n_k = nullptr, *part_n = nullptr;
  double *s_k = nullptr, *q_k = nullptr, *part_s = nullptr, *red = nullptr;
  unsigned long long* counters = nullptr;  // [0] degenerate [1] capped [2] bad input
  int stat_blocks = 0;
  int64_t sweep = 0;
  unsigned long long degenerate_reported = 0;
  // sweep() as a recorded graph
  bool use_graph = true;
  hipGraph_t graph = nullptr;
  hipGraphExec_t graph_exec = nullptr;
  int64_t counter_value = -1;  // what the device's sweep counter (counters[3]) holds once the stream has drained
};

namespace {

bool device_ptrs(const augur_gmm* h) { return (h->cfg.flags & AUGUR_PTRS_DEVICE) != 0; }

void free_all(augur_gmm* h) {
  (void)hipFree(h->x); (void)hipFree(h->pi); (void)hipFree(h->mu); (void)hipFree(h->z);
  (void)hipFree(h->n_k); (void)hipFree(h->part_n); (void)hipFree(h->s_k); (void)hipFree(h->part_s);
  (void)hipFree(h->red); (void)hipFree(h->counters); (void)hipFree(h->var); (void)hipFree(h->q_k);
  if (h->graph_exec) (void)hipGraphExecDestroy(h->graph_exec);
  if (h->graph) (void)hipGraphDestroy(h->graph);
}

int launch_z(augur_gmm* h, SweepRef sweep) {
  const int K = h->cfg.K, dim = h->cfg.dim;
  const int64_t N = h->cfg.N;
  const size_t base_lds = sizeof(double) * ((size_t)K * dim + 2 * (size_t)K);
  const size_t cache_lds = base_lds + sizeof(double) * 256 * (size_t)K;
#define AUGUR_GMM_Z(CACHE, DIMV, LDS)                                                          \
  hipLaunchKernelGGL((gmm_sample_z_kernel<CACHE, DIMV>), dim3((unsigned)((N + 255) / 256)),       \
                     dim3(256), LDS, h->stream, h->x, h->pi, h->mu, h->var, h->z, N, dim, K,      \
                     h->sigma, h->cfg.seed, sweep, h->counters)
  if (cache_lds <= 48 * 1024) {
    switch (dim) {
      case 1: AUGUR_GMM_Z(true, 1, cache_lds); break;
      case 2: AUGUR_GMM_Z(true, 2, cache_lds); break;
      case 3: AUGUR_GMM_Z(true, 3, cache_lds); break;
      case 4: AUGUR_GMM_Z(true, 4, cache_lds); break;
      case 8: AUGUR_GMM_Z(true, 8, cache_lds); break;
      default: AUGUR_GMM_Z(true, 0, cache_lds); break;
    }
  } else {
    AUGUR_GMM_Z(false, 0, base_lds);
  }
#undef AUGUR_GMM_Z
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

int launch_stats(augur_gmm* h) {
  const int K = h->cfg.K, dim = h->cfg.dim;
  // one thread per (component, coordinate) pair; no more waves than that needs
  const int threads = (int)std::min<int64_t>(256, round_up((int64_t)K * (dim + (h->unknown_var ? 1 : 0)), 64));
  if (K <= 64 && kStatChunk == 256 && kStatChunkSq == 256) {
    if (h->unknown_var)
      hipLaunchKernelGGL(gmm_stats_grouped_kernel<true>, dim3(h->stat_blocks), dim3(256),
                         sizeof(double) * 256 * (size_t)(dim + 1), h->stream, h->x, h->z, h->cfg.N,
                         dim, K, h->part_s, h->part_n);
    else
      hipLaunchKernelGGL(gmm_stats_grouped_kernel<false>, dim3(h->stat_blocks), dim3(256),
                         sizeof(float) * 256 * (size_t)dim, h->stream, h->x, h->z, h->cfg.N, dim, K,
                         h->part_s, h->part_n);
  } else if (h->unknown_var) {
    const size_t shm = sizeof(double) * (size_t)kStatChunkSq * (dim + 1) + sizeof(int32_t) * kStatChunkSq;
    hipLaunchKernelGGL(gmm_stats_partial_kernel<true>, dim3(h->stat_blocks), dim3(threads), shm,
                       h->stream, h->x, h->z, h->cfg.N, dim, K, h->part_s, h->part_n);
  } else {
    const size_t shm = sizeof(float) * (size_t)kStatChunk * dim + sizeof(int32_t) * kStatChunk;
    hipLaunchKernelGGL(gmm_stats_partial_kernel<false>, dim3(h->stat_blocks), dim3(threads), shm,
                       h->stream, h->x, h->z, h->cfg.N, dim, K, h->part_s, h->part_n);
  }
  const int W = dim + (h->unknown_var ? 1 : 0);
  hipLaunchKernelGGL(gmm_stats_merge_kernel, dim3(K * W), dim3(256), 0, h->stream, h->part_s,
                     h->part_n, h->stat_blocks, dim, W, K, h->s_k, h->q_k, h->n_k);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

int launch_resample(augur_gmm* h, SweepRef sweep) {
  const size_t shm = sizeof(double) * (size_t)h->cfg.K + sizeof(float) * (size_t)h->cfg.K * h->cfg.dim;
  hipLaunchKernelGGL(gmm_resample_kernel, dim3(1), dim3(256), shm, h->stream, h->n_k, h->s_k, h->q_k,
                     h->pi, h->mu, h->var, h->cfg.dim, h->cfg.K, h->alpha, h->prior_sd, h->sigma,
                     h->a0, h->b0, h->cfg.seed, sweep, h->counters + 1);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

int read_counter(augur_gmm* h, int which, unsigned long long* out) {
  AUGUR_HIP_TRY(hipMemcpyAsync(out, h->counters + which, sizeof(unsigned long long),
                               hipMemcpyDeviceToHost, h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  return AUGUR_OK;
}

#define AUGUR_CHECK_HANDLE(h)                      \
  AUGUR_REQUIRE((h) != nullptr, "handle is NULL"); \
  DeviceGuard guard_((h)->cfg.device);             \
  AUGUR_REQUIRE(guard_.ok, "cannot select device %d", (h)->cfg.device)

#define AUGUR_TRY(expr)              \
  do {                               \
    const int rc_ = (expr);          \
    if (rc_ != AUGUR_OK) return rc_; \
  } while (0)

}  // namespace

extern "C" {

int augur_gmm_create(const augur_gmm_config* cfg, const float* x, augur_gmm** out) {
  AUGUR_REQUIRE(out != nullptr, "out is NULL");
  *out = nullptr;
  AUGUR_REQUIRE(cfg != nullptr && x != nullptr, "config or x is NULL");
  AUGUR_REQUIRE(cfg->N > 0 && cfg->N <= 2147483647LL && cfg->dim > 0 && cfg->K > 0,
                "N, dim, K must be positive and N <= 2^31-1 (got %lld, %d, %d)", (long long)cfg->N,
                cfg->dim, cfg->K);
  AUGUR_REQUIRE((int64_t)cfg->K * cfg->dim <= 4096 && cfg->dim <= 14,
                "supported sizes: dim <= 14 and K * dim <= 4096 (got dim %d, K %d)", cfg->dim,
                cfg->K);
  // the z kernel keeps the means and two K-vectors as doubles in LDS: 8 (K dim + 2 K) bytes,
  // which must fit the 64 KiB a workgroup may ask for
  AUGUR_REQUIRE((int64_t)cfg->K * (cfg->dim + 2) <= 8192,
                "supported sizes: K * (dim + 2) <= 8192 (got dim %d, K %d)", cfg->dim, cfg->K);
  const bool unknown_var = cfg->var_shape > 0.f;
  AUGUR_REQUIRE(std::isfinite(cfg->alpha) && cfg->alpha > 0.f && std::isfinite(cfg->prior_sd) &&
                    cfg->prior_sd > 0.f,
                "alpha and prior_sd must be positive and finite");
  if (unknown_var)
    AUGUR_REQUIRE(std::isfinite(cfg->var_shape) && std::isfinite(cfg->var_scale) &&
                      cfg->var_scale > 0.f,
                  "var_shape and var_scale must be positive and finite for unknown variances");
  else
    AUGUR_REQUIRE(cfg->var_shape == 0.f && std::isfinite(cfg->sigma) && cfg->sigma > 0.f,
                  "known variance: var_shape must be 0 and sigma positive and finite");
  AUGUR_REQUIRE((cfg->flags & ~AUGUR_PTRS_DEVICE) == 0, "unknown flag bits 0x%x", cfg->flags);
  int ndev = 0;
  AUGUR_HIP_TRY(hipGetDeviceCount(&ndev));
  AUGUR_REQUIRE(cfg->device >= 0 && cfg->device < ndev, "device %d out of range (%d present)",
                cfg->device, ndev);
  DeviceGuard guard(cfg->device);
  AUGUR_REQUIRE(guard.ok, "cannot select device %d", cfg->device);

  augur_gmm* h = new (std::nothrow) augur_gmm();
  AUGUR_REQUIRE(h != nullptr, "out of host memory");
  h->cfg = *cfg;
  h->stream = (hipStream_t)cfg->stream;
  h->use_graph = h->stream != nullptr;  // the default stream cannot be recorded
  h->alpha = (double)cfg->alpha;
  h->prior_sd = (double)cfg->prior_sd;
  h->sigma = (double)cfg->sigma;
  h->unknown_var = unknown_var;
  h->a0 = (double)cfg->var_shape;
  h->b0 = (double)cfg->var_scale;
  const int64_t N = cfg->N;
  const int K = cfg->K, dim = cfg->dim;
  const int chunk = unknown_var ? kStatChunkSq : kStatChunk;
  const int W = dim + (unknown_var ? 1 : 0);
  h->stat_blocks = (int)((N + chunk - 1) / chunk);

#define AUGUR_CREATE_TRY(expr)                                                              \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) {                                                                 \
      set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      (void)hipGetLastError(); /* or the runtime hands it to the next caller */ \
      free_all(h);                                                                          \
      delete h;                                                                             \
      return AUGUR_ERR_HIP;                                                                 \
    }                                                                                       \
  } while (0)

  AUGUR_CREATE_TRY(hipMalloc(&h->counters, 4 * sizeof(unsigned long long)));
  AUGUR_CREATE_TRY(hipMemsetAsync(h->counters, 0, 4 * sizeof(unsigned long long), h->stream));
  AUGUR_CREATE_TRY(hipMalloc(&h->x, sizeof(float) * (size_t)N * dim));
  AUGUR_CREATE_TRY(hipMalloc(&h->z, sizeof(int32_t) * (size_t)N));
  AUGUR_CREATE_TRY(hipMalloc(&h->pi, sizeof(float) * (size_t)K));
  AUGUR_CREATE_TRY(hipMalloc(&h->mu, sizeof(float) * (size_t)K * dim));
  AUGUR_CREATE_TRY(hipMalloc(&h->n_k, sizeof(int32_t) * (size_t)K));
  AUGUR_CREATE_TRY(hipMalloc(&h->s_k, sizeof(double) * (size_t)K * dim));
  AUGUR_CREATE_TRY(hipMalloc(&h->part_s, sizeof(double) * (size_t)h->stat_blocks * K * W));
  if (unknown_var) {
    // start from the prior's scale/shape ratio; the first conditional draw replaces it
    std::vector<float> v0((size_t)K, (float)(h->b0 / h->a0));
    AUGUR_CREATE_TRY(hipMalloc(&h->var, sizeof(float) * (size_t)K));
    AUGUR_CREATE_TRY(hipMalloc(&h->q_k, sizeof(double) * (size_t)K));
    AUGUR_CREATE_TRY(hipMemcpy(h->var, v0.data(), sizeof(float) * (size_t)K, hipMemcpyHostToDevice));
  }
  AUGUR_CREATE_TRY(hipMalloc(&h->part_n, sizeof(int32_t) * (size_t)h->stat_blocks * K));
  AUGUR_CREATE_TRY(hipMalloc(&h->red, sizeof(double) * kRedBlocks));
  AUGUR_CREATE_TRY(hipMemcpyAsync(h->x, x, sizeof(float) * (size_t)N * dim,
                                  device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice,
                                  h->stream));
  const int64_t blocks4 = (N + 3) / 4;
  hipLaunchKernelGGL(gmm_init_z_kernel, dim3((unsigned)((blocks4 + 255) / 256)), dim3(256), 0,
                     h->stream, h->z, N, K, cfg->seed);
  AUGUR_CREATE_TRY(hipGetLastError());
  int rc = launch_stats(h);
  if (rc == AUGUR_OK) rc = launch_resample(h, SweepRef{0u, nullptr});
  if (rc == AUGUR_OK && hipStreamSynchronize(h->stream) != hipSuccess) {
    set_error("initial sweep failed: %s", hipGetErrorString(hipGetLastError()));
    (void)hipGetLastError();  // or the runtime hands the error to the next caller
    rc = AUGUR_ERR_HIP;
  }
  if (rc != AUGUR_OK) {
    free_all(h);
    delete h;
    return rc;
  }
  *out = h;
  return AUGUR_OK;
#undef AUGUR_CREATE_TRY
}

void augur_gmm_destroy(augur_gmm* h) {
  if (!h) return;
  DeviceGuard guard(h->cfg.device);
  (void)hipStreamSynchronize(h->stream);
  free_all(h);
  delete h;
}

int augur_gmm_step_sample_z(augur_gmm* h) {
  AUGUR_CHECK_HANDLE(h);
  return launch_z(h, SweepRef{(uint32_t)(h->sweep + 1), nullptr});
}
int augur_gmm_step_stats(augur_gmm* h) {
  AUGUR_CHECK_HANDLE(h);
  return launch_stats(h);
}
int augur_gmm_step_resample(augur_gmm* h) {
  AUGUR_CHECK_HANDLE(h);
  return launch_resample(h, SweepRef{(uint32_t)(h->sweep + 1), nullptr});
}
int augur_gmm_step_finish(augur_gmm* h) {
  AUGUR_REQUIRE(h != nullptr, "handle is NULL");
  h->sweep += 1;
  return AUGUR_OK;
}

int augur_gmm_sweep(augur_gmm* h, int32_t n_sweeps) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(n_sweeps >= 0, "n_sweeps = %d is negative", n_sweeps);
  if (!h->use_graph || n_sweeps == 0) {
    for (int32_t s = 0; s < n_sweeps; ++s) {
      const SweepRef t{(uint32_t)(h->sweep + 1), nullptr};
      AUGUR_TRY(launch_z(h, t));
      AUGUR_TRY(launch_stats(h));
      AUGUR_TRY(launch_resample(h, t));
      h->sweep += 1;
    }
    return AUGUR_OK;
  }
  // One sweep recorded as a HIP graph (its four or five launches, the sweep index read from a
  // counter in device memory that the graph's last kernel advances), then replayed.
  uint32_t* counter = reinterpret_cast<uint32_t*>(h->counters + 3);
  if (h->graph_exec == nullptr) {
    AUGUR_HIP_TRY(hipStreamBeginCapture(h->stream, hipStreamCaptureModeThreadLocal));
    const SweepRef t{0u, counter};
    int rc = launch_z(h, t);
    if (rc == AUGUR_OK) rc = launch_stats(h);
    if (rc == AUGUR_OK) rc = launch_resample(h, t);
    if (rc == AUGUR_OK) {
      hipLaunchKernelGGL(sweep_counter_add_kernel, dim3(1), dim3(1), 0, h->stream, counter, 1u);
      if (hipGetLastError() != hipSuccess) rc = AUGUR_ERR_HIP;
    }
    hipGraph_t g = nullptr;
    const hipError_t e = hipStreamEndCapture(h->stream, &g);  // also ends a failed recording
    if (rc != AUGUR_OK || e != hipSuccess || g == nullptr) {
      if (g) (void)hipGraphDestroy(g);
      if (rc == AUGUR_OK) {
        set_error("recording the sweep as a graph failed: %s", hipGetErrorString(e));
        rc = AUGUR_ERR_HIP;
      }
      (void)hipGetLastError();
      return rc;
    }
    const hipError_t ei = hipGraphInstantiate(&h->graph_exec, g, nullptr, nullptr, 0);
    if (ei != hipSuccess) {
      set_error("hipGraphInstantiate failed: %s", hipGetErrorString(ei));
      (void)hipGetLastError();
      (void)hipGraphDestroy(g);
      h->graph_exec = nullptr;
      return AUGUR_ERR_HIP;
    }
    h->graph = g;
  }
  if (h->counter_value != h->sweep + 1) {
    hipLaunchKernelGGL(sweep_counter_set_kernel, dim3(1), dim3(1), 0, h->stream, counter,
                       (uint32_t)(h->sweep + 1));
    AUGUR_HIP_TRY(hipGetLastError());
    h->counter_value = h->sweep + 1;
  }
  for (int32_t s = 0; s < n_sweeps; ++s) {
    AUGUR_HIP_TRY(hipGraphLaunch(h->graph_exec, h->stream));
    h->sweep += 1;
    h->counter_value += 1;
  }
  return AUGUR_OK;
}

int augur_gmm_set_graph(augur_gmm* h, int32_t on) {
  AUGUR_REQUIRE(h != nullptr, "handle is NULL");
  AUGUR_REQUIRE(on == 0 || h->stream != nullptr,
                "sweeps can only be recorded on a stream of the caller's (config.stream), not on the default stream");
  h->use_graph = on != 0;
  return AUGUR_OK;
}

int augur_gmm_sweep_profile(augur_gmm* h, int32_t n_sweeps, double* ms) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(n_sweeps >= 0 && n_sweeps <= 4096 && ms != nullptr,
                "n_sweeps must lie in [0, 4096] and ms must not be NULL");
  for (int i = 0; i < AUGUR_GMM_NSTEPS; ++i) ms[i] = 0.0;
  // four events per sweep, recorded without a host wait; read back at the end
  std::vector<hipEvent_t> ev((size_t)n_sweeps * 4, nullptr);
  int rc = AUGUR_OK;
  auto fail_hip = [&](hipError_t e, const char* what) {
    if (e != hipSuccess && rc == AUGUR_OK) {
      set_error("%s failed: %s", what, hipGetErrorString(e));
      (void)hipGetLastError();  // or the runtime hands the error to the next caller
      rc = AUGUR_ERR_HIP;
    }
    return e != hipSuccess;
  };
  for (auto& e : ev)
    if (fail_hip(hipEventCreate(&e), "hipEventCreate")) break;
  int done = 0;
  for (int32_t s = 0; s < n_sweeps && rc == AUGUR_OK; ++s) {
    hipEvent_t* e = &ev[(size_t)s * 4];
    const uint32_t t = (uint32_t)(h->sweep + 1);
    if (fail_hip(hipEventRecord(e[0], h->stream), "hipEventRecord")) break;
    rc = launch_z(h, SweepRef{t, nullptr});
    if (rc == AUGUR_OK && fail_hip(hipEventRecord(e[1], h->stream), "hipEventRecord")) break;
    if (rc == AUGUR_OK) rc = launch_stats(h);
    if (rc == AUGUR_OK && fail_hip(hipEventRecord(e[2], h->stream), "hipEventRecord")) break;
    if (rc == AUGUR_OK) rc = launch_resample(h, SweepRef{t, nullptr});
    if (rc == AUGUR_OK && fail_hip(hipEventRecord(e[3], h->stream), "hipEventRecord")) break;
    if (rc == AUGUR_OK) {
      h->sweep += 1;
      ++done;
    }
  }
  fail_hip(hipStreamSynchronize(h->stream), "hipStreamSynchronize");
  for (int s = 0; s < done && rc == AUGUR_OK; ++s) {
    hipEvent_t* e = &ev[(size_t)s * 4];
    for (int i = 0; i < 3; ++i) {
      float x = 0.f;
      if (fail_hip(hipEventElapsedTime(&x, e[i], e[i + 1]), "hipEventElapsedTime")) break;
      ms[i] += (double)x;
    }
    float x = 0.f;
    if (fail_hip(hipEventElapsedTime(&x, e[0], e[3]), "hipEventElapsedTime")) break;
    ms[3] += (double)x;
  }
  for (auto& e : ev)
    if (e) (void)hipEventDestroy(e);
  return rc;
}

int augur_gmm_loglik(augur_gmm* h, double* log_joint) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(log_joint != nullptr, "log_joint is NULL");
  const int K = h->cfg.K, dim = h->cfg.dim;
  hipLaunchKernelGGL(gmm_loglik_kernel, dim3(kRedBlocks), dim3(256), 0, h->stream, h->x, h->z, h->pi,
                     h->mu, h->var, h->cfg.N, dim, h->sigma, h->red);
  AUGUR_HIP_TRY(hipGetLastError());
  std::vector<double> part(kRedBlocks);
  std::vector<float> pi(K), mu((size_t)K * dim), var(h->unknown_var ? K : 0);
  if (h->unknown_var)
    AUGUR_HIP_TRY(hipMemcpyAsync(var.data(), h->var, sizeof(float) * K, hipMemcpyDeviceToHost,
                                 h->stream));
  AUGUR_HIP_TRY(hipMemcpyAsync(part.data(), h->red, sizeof(double) * kRedBlocks,
                               hipMemcpyDeviceToHost, h->stream));
  AUGUR_HIP_TRY(hipMemcpyAsync(pi.data(), h->pi, sizeof(float) * K, hipMemcpyDeviceToHost,
                               h->stream));
  AUGUR_HIP_TRY(hipMemcpyAsync(mu.data(), h->mu, sizeof(float) * mu.size(), hipMemcpyDeviceToHost,
                               h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  // the prior terms are a handful of scalars: summed on the host
  const double LN_2PI = 1.8378770664093454835606594728112;
  double lj = std::lgamma(K * h->alpha) - K * std::lgamma(h->alpha);
  for (int k = 0; k < K; ++k) lj += (h->alpha - 1.0) * std::log((double)pi[k]);
  for (size_t e = 0; e < mu.size(); ++e) {
    const double m = (double)mu[e];
    lj += -0.5 * LN_2PI - std::log(h->prior_sd) - m * m / (2.0 * h->prior_sd * h->prior_sd);
  }
  for (size_t k = 0; k < var.size(); ++k) {  // var_k ~ InverseGamma(a0, b0)
    const double v = (double)var[k];
    lj += h->a0 * std::log(h->b0) - std::lgamma(h->a0) - (h->a0 + 1.0) * std::log(v) - h->b0 / v;
  }
  for (int i = 0; i < kRedBlocks; ++i) lj += part[i];
  *log_joint = lj;
  unsigned long long deg = 0;
  AUGUR_TRY(read_counter(h, 0, &deg));
  if (deg > h->degenerate_reported) {
    set_error("%llu points met a conditional of zero or non-finite mass since the last report",
              deg - h->degenerate_reported);
    h->degenerate_reported = deg;
    return AUGUR_ERR_DEGENERATE;
  }
  return AUGUR_OK;
}

int augur_gmm_get_state(augur_gmm* h, int32_t* z, float* pi, float* mu, int64_t* sweep) {
  AUGUR_CHECK_HANDLE(h);
  const hipMemcpyKind kind = device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost;
  if (z) AUGUR_HIP_TRY(hipMemcpyAsync(z, h->z, sizeof(int32_t) * (size_t)h->cfg.N, kind, h->stream));
  if (pi) AUGUR_HIP_TRY(hipMemcpyAsync(pi, h->pi, sizeof(float) * (size_t)h->cfg.K, kind, h->stream));
  if (mu)
    AUGUR_HIP_TRY(hipMemcpyAsync(mu, h->mu, sizeof(float) * (size_t)h->cfg.K * h->cfg.dim, kind,
                                 h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  if (sweep) *sweep = h->sweep;
  return AUGUR_OK;
}

int augur_gmm_set_state(augur_gmm* h, const int32_t* z, const float* pi, const float* mu,
                        int64_t sweep) {
  AUGUR_CHECK_HANDLE(h);
  const hipMemcpyKind kind = device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
  if (z) {
    if (!device_ptrs(h)) {
      for (int64_t i = 0; i < h->cfg.N; ++i)
        AUGUR_REQUIRE(z[i] >= 0 && z[i] < h->cfg.K, "z[%lld] = %d is outside [0, %d)",
                      (long long)i, z[i], h->cfg.K);
    } else {
      AUGUR_HIP_TRY(hipMemsetAsync(h->counters + 2, 0, sizeof(unsigned long long), h->stream));
      hipLaunchKernelGGL(gmm_check_range_kernel, dim3(512), dim3(256), 0, h->stream, z, h->cfg.N,
                         h->cfg.K, h->counters + 2);
      unsigned long long bad = 0;
      AUGUR_TRY(read_counter(h, 2, &bad));
      AUGUR_REQUIRE(bad == 0, "%llu entries of z are outside [0, %d)", bad, h->cfg.K);
    }
    AUGUR_HIP_TRY(hipMemcpyAsync(h->z, z, sizeof(int32_t) * (size_t)h->cfg.N, kind, h->stream));
    AUGUR_TRY(launch_stats(h));
  }
  if (pi) AUGUR_HIP_TRY(hipMemcpyAsync(h->pi, pi, sizeof(float) * (size_t)h->cfg.K, kind, h->stream));
  if (mu)
    AUGUR_HIP_TRY(hipMemcpyAsync(h->mu, mu, sizeof(float) * (size_t)h->cfg.K * h->cfg.dim, kind,
                                 h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  if (sweep >= 0) h->sweep = sweep;
  return AUGUR_OK;
}

int augur_gmm_get_var(augur_gmm* h, float* var) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(h->unknown_var, "this handle has a known variance (var_shape = 0)");
  AUGUR_REQUIRE(var != nullptr, "var is NULL");
  AUGUR_HIP_TRY(hipMemcpyAsync(var, h->var, sizeof(float) * (size_t)h->cfg.K,
                               device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost,
                               h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  return AUGUR_OK;
}

int augur_gmm_set_var(augur_gmm* h, const float* var) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(h->unknown_var, "this handle has a known variance (var_shape = 0)");
  AUGUR_REQUIRE(var != nullptr, "var is NULL");
  std::vector<float> v((size_t)h->cfg.K);  // K values: checked on the host either way
  if (device_ptrs(h)) {
    AUGUR_HIP_TRY(hipMemcpyAsync(v.data(), var, sizeof(float) * v.size(), hipMemcpyDeviceToHost,
                                 h->stream));
    AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  } else {
    std::copy(var, var + v.size(), v.begin());
  }
  for (int k = 0; k < h->cfg.K; ++k)
    AUGUR_REQUIRE(std::isfinite(v[k]) && v[k] > 0.f, "var[%d] = %g is not positive and finite", k,
                  (double)v[k]);
  AUGUR_HIP_TRY(hipMemcpyAsync(h->var, v.data(), sizeof(float) * v.size(), hipMemcpyHostToDevice,
                               h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  return AUGUR_OK;
}

int augur_gmm_get_stats(augur_gmm* h, int32_t* n_k, double* s_k) {
  AUGUR_CHECK_HANDLE(h);
  const hipMemcpyKind kind = device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost;
  if (n_k) AUGUR_HIP_TRY(hipMemcpyAsync(n_k, h->n_k, sizeof(int32_t) * (size_t)h->cfg.K, kind, h->stream));
  if (s_k)
    AUGUR_HIP_TRY(hipMemcpyAsync(s_k, h->s_k, sizeof(double) * (size_t)h->cfg.K * h->cfg.dim, kind,
                                 h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  return AUGUR_OK;
}

int augur_gmm_get_degenerate(augur_gmm* h, int64_t* count) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(count != nullptr, "count is NULL");
  unsigned long long c = 0;
  AUGUR_TRY(read_counter(h, 0, &c));
  *count = (int64_t)c;
  return AUGUR_OK;
}

int augur_gmm_sync(augur_gmm* h) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  return AUGUR_OK;
}

}  // extern "C"

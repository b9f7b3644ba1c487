// Data-parallel random-walk Metropolis-Hastings on the multivariate regression
// model of arXiv 1312.3613 (Fig. "regression"; Sect. 4.1): the function f
// proportional to the posterior is the product of the priors of w, b, tau and
// of one term per datum, evaluated in log space with the per-datum terms
// computed in parallel and summed; a symmetric Gaussian random walk over all
// parameters at once proposes, and the usual ratio test accepts.
//
//   w_k ~ N(0, prior_sd^2), b ~ N(0, prior_sd^2), tau ~ InverseGamma(a0, b0),
//   x_nk ~ Uniform(lo, hi), y_n ~ N(x_n . w + b, tau)      (tau a variance)
//
// theta = (w_0 .. w_{K-1}, b, tau) is fp64; x float[N][K] and y float[N] stay
// in HBM (or LDS, below).  The only data-dependent part of ln f is the sum of
// squared residuals SSR(w, b); everything else is a handful of scalars.
//
// SSR has one summation order whatever the launch shape: points are grouped in
// chunks of 1024; in a chunk, thread j of 256 adds points j, j+256, j+512,
// j+768 in that order, each wave adds its 64 lanes with an xor butterfly, the
// four wave sums are added in wave order; the chunk sums are then added the
// same way (thread j takes chunks j, j+256, ...).
//
// Two schedules:
//  * chain kernel (N <= 65536): ONE workgroup of 1024 threads runs all the
//    requested steps in a single launch; the data sit in LDS (transposed,
//    conflict-free) when they fit, else they come from L2 every step.  At the
//    sizes of the paper's regression tables (hundreds to thousands of rows) a
//    launch per step would cost several times the arithmetic.
//  * step kernel (any N): one launch per step over min(chunks, 2048) workgroups;
//    the workgroup that finishes last (a ticket from one device-scope atomic, no
//    waiting) adds the chunk sums and takes the decision.
#include "common.hpp"

#include <algorithm>
#include <new>
#include <vector>

using namespace augur;

namespace {

constexpr int kChunk = 1024;
constexpr int kMaxK = 64;
constexpr int kMaxChainChunks = 64;        // chain kernel: N <= 64 * 1024
constexpr int kMaxStepBlocks = 2048;
constexpr size_t kLdsDataBytes = 128 * 1024;  // data cached in LDS up to this size
constexpr double kLn2Pi = 1.8378770664093454835606594728112;

struct MhParams {
  int64_t N;
  int K;
  double prior_sd, a0, b0, step;
  double ln_prior_const;  // -(K+1)(ln 2pi / 2 + ln prior_sd) + a0 ln b0 - lgamma(a0)
  double ln_x_const;      // -N K ln(hi - lo)
  uint64_t seed;
};

struct MhState {
  double theta[kMaxK + 2];
  double logf;
  unsigned long long accepted;
  unsigned int ticket;
};

// theta'_e = theta_e + step * n_e: block (index e, step t) of the proposal stream.
__device__ __forceinline__ double propose_one(const MhParams& p, double theta_e, int e, uint32_t t) {
  return theta_e + p.step * normal_from(random_block(p.seed, (uint64_t)e, t, kStreamMhProposal, 0));
}

// Squared residual of point n.  kLds: x is stored [K][ld] and y [ld] in LDS.
template <bool kLds>
__device__ __forceinline__ double sq_residual(const float* __restrict__ x, const float* __restrict__ y,
                                              int64_t n, int K, int64_t ld, const double* th) {
  double mean = th[K];
  if (kLds) {
    for (int k = 0; k < K; ++k) mean += th[k] * (double)x[(int64_t)k * ld + n];
  } else {
    for (int k = 0; k < K; ++k) mean += th[k] * (double)x[n * K + k];
  }
  const double r = (double)y[n] - mean;
  return r * r;
}

// Sum over one chunk by a group of 256 consecutive threads (four waves); g = index in the
// group.  Returns the wave's sum in every lane; the caller adds the four waves in order.
template <bool kLds>
__device__ __forceinline__ double chunk_wave_sum(const float* __restrict__ x, const float* __restrict__ y,
                                                 int64_t N, int K, int64_t ld, int64_t base,
                                                 const double* th, int g) {
  double s = 0.0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t n = base + g + 256 * i;
    if (n < N) s += sq_residual<kLds>(x, y, n, K, ld, th);
  }
  return wave_allreduce_sum(s);
}

// ln f at the proposal from its SSR; -inf outside the support of tau.
__device__ __forceinline__ double logf_from_ssr(const MhParams& p, const double* th, double ssr) {
  const int K = p.K;
  const double tau = th[K + 1];
  if (!(tau > 0.0)) return -INFINITY;
  double sq = 0.0;
  for (int k = 0; k <= K; ++k) sq += th[k] * th[k];
  const double ln_tau = log(tau);
  return p.ln_prior_const - sq / (2.0 * p.prior_sd * p.prior_sd) - (p.a0 + 1.0) * ln_tau - p.b0 / tau +
         p.ln_x_const - 0.5 * (double)p.N * (kLn2Pi + ln_tau) - ssr / (2.0 * tau);
}

__device__ __forceinline__ bool accept_test(const MhParams& p, uint32_t t, double lp, double lf) {
  const double u = u32d(random_block(p.seed, 0, t, kStreamMhAccept, 0).x);
  return log(u) < lp - lf;
}

// Adds n chunk sums (LDS or global) in the fixed order; first 256 threads of the block.
// smem4: four doubles.  Result valid in thread 0.
__device__ __forceinline__ double final_sum(const double* part, int n, int tid, double* smem4) {
  double s = 0.0;
  if (tid < 256) {
    for (int c = tid; c < n; c += 256) s += part[c];
    s = wave_allreduce_sum(s);
    if ((tid & 63) == 0) smem4[tid >> 6] = s;
  }
  __syncthreads();
  return ((smem4[0] + smem4[1]) + smem4[2]) + smem4[3];
}

// ---------------------------------------------------------------- chain kernel
// One workgroup, all steps.  Thread group q (256 threads) takes chunks q, q+4, ...
template <bool kLds>
__global__ __launch_bounds__(1024) void mhreg_chain_kernel(
    const float* __restrict__ x, const float* __restrict__ y, MhParams p, MhState* __restrict__ st,
    int64_t n_steps, uint32_t first_step, double* __restrict__ trace, int64_t ld) {
  extern __shared__ __align__(16) float data[];  // kLds: x as [K][ld], then y [ld]
  __shared__ double th[kMaxK + 2], prop[kMaxK + 2];
  __shared__ double wsum[16], part[kMaxChainChunks], smem4[4];
  __shared__ double lf_s;
  __shared__ unsigned long long acc_s;
  const int tid = threadIdx.x, K = p.K;
  const int q = tid >> 8, g = tid & 255, wave = tid >> 6;
  const int nchunks = (int)((p.N + kChunk - 1) / kChunk);
  if (kLds) {
    for (int64_t e = tid; e < p.N * K; e += 1024) data[(e % K) * ld + e / K] = x[e];
    for (int64_t n = tid; n < p.N; n += 1024) data[(int64_t)K * ld + n] = y[n];
  }
  const float* xd = kLds ? data : x;
  const float* yd = kLds ? data + (int64_t)K * ld : y;
  if (tid < K + 2) th[tid] = st->theta[tid];
  if (tid == 0) {
    lf_s = st->logf;
    acc_s = st->accepted;
  }
  __syncthreads();
  for (int64_t s = 0; s < n_steps; ++s) {
    const uint32_t t = first_step + (uint32_t)s;
    if (tid < K + 2) prop[tid] = propose_one(p, th[tid], tid, t);
    __syncthreads();
    const bool in_support = prop[K + 1] > 0.0;
    double ssr = 0.0;
    if (in_support) {
      for (int c0 = 0; c0 < nchunks; c0 += 4) {
        const int c = c0 + q;
        const double w = c < nchunks
                             ? chunk_wave_sum<kLds>(xd, yd, p.N, K, ld, (int64_t)c * kChunk, prop, g)
                             : 0.0;
        if ((tid & 63) == 0) wsum[wave] = w;
        __syncthreads();
        if (g == 0 && c < nchunks)
          part[c] = ((wsum[4 * q] + wsum[4 * q + 1]) + wsum[4 * q + 2]) + wsum[4 * q + 3];
        __syncthreads();
      }
      ssr = final_sum(part, nchunks, tid, smem4);
    }
    if (tid == 0) {
      const double lp = in_support ? logf_from_ssr(p, prop, ssr) : -INFINITY;
      const bool take = accept_test(p, t, lp, lf_s);
      if (take) {
        lf_s = lp;
        acc_s += 1;
      }
      wsum[0] = take ? 1.0 : 0.0;
    }
    __syncthreads();
    const bool take = wsum[0] != 0.0;
    if (tid < K + 2) {
      if (take) th[tid] = prop[tid];
      if (trace) trace[s * (K + 3) + tid] = th[tid];
    }
    if (tid == 0 && trace) trace[s * (K + 3) + K + 2] = lf_s;
    __syncthreads();
  }
  if (tid < K + 2) st->theta[tid] = th[tid];
  if (tid == 0) {
    st->logf = lf_s;
    st->accepted = acc_s;
  }
}

// ----------------------------------------------------------------- step kernel
// One step.  With decide = false only ln f at st->theta is computed (into st->logf).
__global__ __launch_bounds__(256) void mhreg_step_kernel(
    const float* __restrict__ x, const float* __restrict__ y, MhParams p, MhState* __restrict__ st,
    double* __restrict__ part, uint32_t t, bool decide, double* __restrict__ trace_row) {
  __shared__ double prop[kMaxK + 2];
  __shared__ double wsum[4], smem4[4];
  __shared__ bool last_s;
  const int tid = threadIdx.x, K = p.K;
  const int nchunks = (int)((p.N + kChunk - 1) / kChunk);
  if (tid < K + 2) prop[tid] = decide ? propose_one(p, st->theta[tid], tid, t) : st->theta[tid];
  __syncthreads();
  const bool in_support = prop[K + 1] > 0.0;
  if (in_support) {
    for (int c = blockIdx.x; c < nchunks; c += gridDim.x) {
      const double w = chunk_wave_sum<false>(x, y, p.N, K, 0, (int64_t)c * kChunk, prop, tid);
      if ((tid & 63) == 0) wsum[tid >> 6] = w;
      __syncthreads();
      if (tid == 0) part[c] = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
      __syncthreads();
    }
  }
  if (tid == 0) {
    __threadfence();  // this workgroup's chunk sums before its ticket
    const unsigned int ticket = atomicAdd(&st->ticket, 1u);
    last_s = ticket == gridDim.x - 1;
    if (last_s) __threadfence();  // the others' chunk sums after their tickets
  }
  __syncthreads();
  if (!last_s) return;
  // the workgroup that drew the last ticket: every chunk sum is in memory
  __shared__ double part_s[256];
  double s = 0.0;
  if (in_support)
    for (int c = tid; c < nchunks; c += 256)
      s += __longlong_as_double((long long)__hip_atomic_load(
          reinterpret_cast<unsigned long long*>(part) + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  part_s[tid] = s;  // thread j holds chunks j, j+256, ... : the fixed order's first level
  __syncthreads();
  s = wave_allreduce_sum(part_s[tid]);
  if ((tid & 63) == 0) smem4[tid >> 6] = s;
  __syncthreads();
  const double ssr = ((smem4[0] + smem4[1]) + smem4[2]) + smem4[3];
  __shared__ bool take_s;
  if (tid == 0) {
    const double lp = in_support ? logf_from_ssr(p, prop, ssr) : -INFINITY;
    if (decide) {
      take_s = accept_test(p, t, lp, st->logf);
      if (take_s) {
        st->logf = lp;
        st->accepted += 1;
      }
    } else {
      take_s = false;
      st->logf = lp;
    }
    st->ticket = 0;  // for the next launch
  }
  __syncthreads();
  if (tid < K + 2) {
    const double v = take_s ? prop[tid] : st->theta[tid];
    if (take_s) st->theta[tid] = v;
    if (trace_row) trace_row[tid] = v;
  }
  if (tid == 0 && trace_row) trace_row[K + 2] = st->logf;
}

// Counts values outside [lo, hi] (or not finite) in x and non-finite values in y.
__global__ __launch_bounds__(256) void mhreg_check_kernel(const float* __restrict__ x,
                                                           const float* __restrict__ y, int64_t N,
                                                           int K, float lo, float hi,
                                                           unsigned long long* __restrict__ bad) {
  unsigned long long c = 0;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (int64_t e = first; e < N * K; e += stride)
    if (!(x[e] >= lo && x[e] <= hi)) ++c;
  for (int64_t n = first; n < N; n += stride)
    if (!(fabsf(y[n]) <= FLT_MAX)) ++c;
  if (c) atomicAdd(bad, c);
}

}  // namespace

struct augur_mhreg {
  augur_mhreg_config cfg{};
  hipStream_t stream = nullptr;
  MhParams p{};
  float *x = nullptr, *y = nullptr;
  MhState* st = nullptr;
  double* part = nullptr;
  unsigned long long* bad = nullptr;
  int nchunks = 0, step_blocks = 0;
  int schedule = 0;  // 0 automatic, 1 chain kernel, 2 step kernel
  bool lds_attr_set = false;
  int64_t step_index = 0;
};

namespace {

bool device_ptrs(const augur_mhreg* h) { return (h->cfg.flags & AUGUR_PTRS_DEVICE) != 0; }

void free_all(augur_mhreg* h) {
  (void)hipFree(h->x); (void)hipFree(h->y); (void)hipFree(h->st); (void)hipFree(h->part);
  (void)hipFree(h->bad);
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

bool use_chain(const augur_mhreg* h) {
  if (h->schedule == 1) return true;
  if (h->schedule == 2) return false;
  return h->cfg.N <= 16384;
}

// ln f at the current theta into the state.
int launch_evaluate(augur_mhreg* h) {
  hipLaunchKernelGGL(mhreg_step_kernel, dim3(h->step_blocks), dim3(256), 0, h->stream, h->x, h->y,
                     h->p, h->st, h->part, 0u, false, (double*)nullptr);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

int launch_steps(augur_mhreg* h, int64_t n_steps, double* trace_dev) {
  const int K = h->cfg.K;
  const uint32_t first = (uint32_t)(h->step_index + 1);
  if (use_chain(h)) {
    const int64_t ld = round_up(h->cfg.N, 64);
    const size_t data_bytes = sizeof(float) * (size_t)ld * (K + 1);
    if (data_bytes <= kLdsDataBytes) {
      if (!h->lds_attr_set) {
        AUGUR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&mhreg_chain_kernel<true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)kLdsDataBytes));
        h->lds_attr_set = true;
      }
      hipLaunchKernelGGL(mhreg_chain_kernel<true>, dim3(1), dim3(1024), data_bytes, h->stream, h->x,
                         h->y, h->p, h->st, n_steps, first, trace_dev, ld);
    } else {
      hipLaunchKernelGGL(mhreg_chain_kernel<false>, dim3(1), dim3(1024), 0, h->stream, h->x, h->y,
                         h->p, h->st, n_steps, first, trace_dev, (int64_t)0);
    }
    AUGUR_HIP_TRY(hipGetLastError());
  } else {
    for (int64_t s = 0; s < n_steps; ++s) {
      hipLaunchKernelGGL(mhreg_step_kernel, dim3(h->step_blocks), dim3(256), 0, h->stream, h->x,
                         h->y, h->p, h->st, h->part, first + (uint32_t)s, true,
                         trace_dev ? trace_dev + s * (K + 3) : (double*)nullptr);
    }
    AUGUR_HIP_TRY(hipGetLastError());
  }
  h->step_index += n_steps;
  return AUGUR_OK;
}

int upload_theta(augur_mhreg* h, const double* theta) {
  const int K = h->cfg.K;
  std::vector<double> th((size_t)K + 2);
  if (device_ptrs(h)) {
    AUGUR_HIP_TRY(hipMemcpyAsync(th.data(), theta, sizeof(double) * th.size(), hipMemcpyDeviceToHost,
                                 h->stream));
    AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  } else {
    std::copy(theta, theta + th.size(), th.begin());
  }
  for (int e = 0; e < K + 2; ++e)
    AUGUR_REQUIRE(std::isfinite(th[e]), "theta[%d] = %g is not finite", e, th[e]);
  AUGUR_REQUIRE(th[K + 1] > 0.0, "tau = %g is outside the support (tau > 0)", th[K + 1]);
  AUGUR_HIP_TRY(hipMemcpyAsync(h->st->theta, th.data(), sizeof(double) * th.size(),
                               hipMemcpyHostToDevice, h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));  // th leaves scope
  return launch_evaluate(h);
}

}  // namespace

extern "C" {

int augur_mhreg_create(const augur_mhreg_config* cfg, const float* x, const float* y,
                       const double* theta0, augur_mhreg** out) {
  AUGUR_REQUIRE(out != nullptr, "out is NULL");
  *out = nullptr;
  AUGUR_REQUIRE(cfg != nullptr && x != nullptr && y != nullptr, "config, x or y is NULL");
  AUGUR_REQUIRE(cfg->N > 0 && cfg->N <= 2147483647LL && cfg->K > 0 && cfg->K <= kMaxK,
                "N must be in [1, 2^31-1] and K in [1, %d] (got %lld, %d)", kMaxK, (long long)cfg->N,
                cfg->K);
  AUGUR_REQUIRE(std::isfinite(cfg->prior_sd) && cfg->prior_sd > 0.f && std::isfinite(cfg->tau_shape) &&
                    cfg->tau_shape > 0.f && std::isfinite(cfg->tau_scale) && cfg->tau_scale > 0.f &&
                    std::isfinite(cfg->step) && cfg->step > 0.f,
                "prior_sd, tau_shape, tau_scale and step must be positive and finite");
  AUGUR_REQUIRE(std::isfinite(cfg->x_lo) && std::isfinite(cfg->x_hi) && cfg->x_lo < cfg->x_hi,
                "x_lo < x_hi required (got %g, %g)", (double)cfg->x_lo, (double)cfg->x_hi);
  AUGUR_REQUIRE((cfg->flags & ~AUGUR_PTRS_DEVICE) == 0, "unknown flag bits 0x%x", cfg->flags);
  int ndev = 0;
  AUGUR_HIP_TRY(hipGetDeviceCount(&ndev));
  AUGUR_REQUIRE(cfg->device >= 0 && cfg->device < ndev, "device %d out of range (%d present)",
                cfg->device, ndev);
  DeviceGuard guard(cfg->device);
  AUGUR_REQUIRE(guard.ok, "cannot select device %d", cfg->device);

  augur_mhreg* h = new (std::nothrow) augur_mhreg();
  AUGUR_REQUIRE(h != nullptr, "out of host memory");
  h->cfg = *cfg;
  h->stream = (hipStream_t)cfg->stream;
  const int64_t N = cfg->N;
  const int K = cfg->K;
  MhParams& p = h->p;
  p.N = N;
  p.K = K;
  p.prior_sd = (double)cfg->prior_sd;
  p.a0 = (double)cfg->tau_shape;
  p.b0 = (double)cfg->tau_scale;
  p.step = (double)cfg->step;
  p.seed = cfg->seed;
  p.ln_prior_const = -(double)(K + 1) * (0.5 * kLn2Pi + std::log(p.prior_sd)) + p.a0 * std::log(p.b0) -
                     std::lgamma(p.a0);
  p.ln_x_const = -(double)N * (double)K * std::log((double)cfg->x_hi - (double)cfg->x_lo);
  h->nchunks = (int)((N + kChunk - 1) / kChunk);
  h->step_blocks = std::min(h->nchunks, kMaxStepBlocks);

#define AUGUR_CREATE_TRY(expr)                                                              \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) {                                                                 \
      set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      free_all(h);                                                                          \
      delete h;                                                                             \
      return AUGUR_ERR_HIP;                                                                 \
    }                                                                                       \
  } while (0)

  const hipMemcpyKind in_kind = device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
  AUGUR_CREATE_TRY(hipMalloc(&h->x, sizeof(float) * (size_t)N * K));
  AUGUR_CREATE_TRY(hipMalloc(&h->y, sizeof(float) * (size_t)N));
  AUGUR_CREATE_TRY(hipMalloc(&h->st, sizeof(MhState)));
  AUGUR_CREATE_TRY(hipMalloc(&h->part, sizeof(double) * (size_t)h->nchunks));
  AUGUR_CREATE_TRY(hipMalloc(&h->bad, sizeof(unsigned long long)));
  AUGUR_CREATE_TRY(hipMemsetAsync(h->st, 0, sizeof(MhState), h->stream));
  AUGUR_CREATE_TRY(hipMemsetAsync(h->bad, 0, sizeof(unsigned long long), h->stream));
  AUGUR_CREATE_TRY(hipMemcpyAsync(h->x, x, sizeof(float) * (size_t)N * K, in_kind, h->stream));
  AUGUR_CREATE_TRY(hipMemcpyAsync(h->y, y, sizeof(float) * (size_t)N, in_kind, h->stream));
  hipLaunchKernelGGL(mhreg_check_kernel, dim3(512), dim3(256), 0, h->stream, h->x, h->y, N, K,
                     cfg->x_lo, cfg->x_hi, h->bad);
  AUGUR_CREATE_TRY(hipGetLastError());
  unsigned long long bad = 0;
  AUGUR_CREATE_TRY(hipMemcpyAsync(&bad, h->bad, sizeof(bad), hipMemcpyDeviceToHost, h->stream));
  AUGUR_CREATE_TRY(hipStreamSynchronize(h->stream));
  int rc = AUGUR_OK;
  if (bad != 0) {
    set_error("%llu values of x lie outside [x_lo, x_hi] or are not finite (x or y)", bad);
    rc = AUGUR_ERR_INVALID_ARG;
  }
  if (rc == AUGUR_OK) {
    if (theta0 != nullptr) {
      rc = upload_theta(h, theta0);
    } else {  // w = 0, b = 0, tau = 1
      std::vector<double> th((size_t)K + 2, 0.0);
      th[K + 1] = 1.0;
      if (hipMemcpy(h->st->theta, th.data(), sizeof(double) * th.size(), hipMemcpyHostToDevice) !=
          hipSuccess) {
        set_error("initial state upload failed");
        rc = AUGUR_ERR_HIP;
      } else {
        rc = launch_evaluate(h);
      }
    }
  }
  if (rc == AUGUR_OK && hipStreamSynchronize(h->stream) != hipSuccess) {
    set_error("initial evaluation failed: %s", hipGetErrorString(hipGetLastError()));
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

void augur_mhreg_destroy(augur_mhreg* h) {
  if (!h) return;
  DeviceGuard guard(h->cfg.device);
  (void)hipStreamSynchronize(h->stream);
  free_all(h);
  delete h;
}

int augur_mhreg_run(augur_mhreg* h, int64_t n_steps, double* trace) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(n_steps >= 0, "n_steps = %lld is negative", (long long)n_steps);
  AUGUR_REQUIRE(h->step_index + n_steps < 4294967295LL, "step index would pass 2^32 - 1");
  if (n_steps == 0) return AUGUR_OK;
  const int K = h->cfg.K;
  if (trace == nullptr || device_ptrs(h)) return launch_steps(h, n_steps, trace);
  double* dev = nullptr;
  const size_t bytes = sizeof(double) * (size_t)n_steps * (K + 3);
  AUGUR_HIP_TRY(hipMalloc(&dev, bytes));
  int rc = launch_steps(h, n_steps, dev);
  if (rc == AUGUR_OK && (hipMemcpyAsync(trace, dev, bytes, hipMemcpyDeviceToHost, h->stream) != hipSuccess ||
                         hipStreamSynchronize(h->stream) != hipSuccess)) {
    set_error("trace download failed: %s", hipGetErrorString(hipGetLastError()));
    rc = AUGUR_ERR_HIP;
  }
  (void)hipStreamSynchronize(h->stream);
  (void)hipFree(dev);
  return rc;
}

int augur_mhreg_get_state(augur_mhreg* h, double* theta, double* logf, int64_t* step_index,
                          int64_t* accepted) {
  AUGUR_CHECK_HANDLE(h);
  MhState st;
  AUGUR_HIP_TRY(hipMemcpyAsync(&st, h->st, sizeof(MhState), hipMemcpyDeviceToHost, h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  if (theta) {
    if (device_ptrs(h)) {
      AUGUR_HIP_TRY(hipMemcpyAsync(theta, h->st->theta, sizeof(double) * ((size_t)h->cfg.K + 2),
                                   hipMemcpyDeviceToDevice, h->stream));
      AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
    } else {
      std::copy(st.theta, st.theta + h->cfg.K + 2, theta);
    }
  }
  if (logf) *logf = st.logf;
  if (step_index) *step_index = h->step_index;
  if (accepted) *accepted = (int64_t)st.accepted;
  return AUGUR_OK;
}

int augur_mhreg_set_state(augur_mhreg* h, const double* theta, int64_t step_index) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(step_index < 4294967295LL, "step_index = %lld is too large", (long long)step_index);
  if (theta) AUGUR_TRY(upload_theta(h, theta));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  if (step_index >= 0) h->step_index = step_index;
  return AUGUR_OK;
}

int augur_mhreg_set_schedule(augur_mhreg* h, int32_t schedule) {
  AUGUR_REQUIRE(h != nullptr, "handle is NULL");
  AUGUR_REQUIRE(schedule >= 0 && schedule <= 2, "schedule = %d (0 automatic, 1 chain, 2 step)", schedule);
  AUGUR_REQUIRE(schedule != 1 || h->nchunks <= kMaxChainChunks,
                "the chain kernel takes at most %d points", kMaxChainChunks * kChunk);
  h->schedule = schedule;
  return AUGUR_OK;
}

int augur_mhreg_sync(augur_mhreg* h) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  return AUGUR_OK;
}

}  // extern "C"

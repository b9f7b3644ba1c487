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
// theta = (w_0 .. w_{K-1}, b, tau) is fp64.  The library keeps its own copy of
// the data, transposed and zero-padded: xt float[K][ld] and y float[ld] (ld = N
// rounded up to 64), so that a thread reads four consecutive points of every
// predictor with one 16-byte load, at unit stride across the wave.  The only data-dependent part of ln f is the sum of squared
// residuals SSR(w, b); everything else is a handful of scalars.
//
// SSR has one summation order whatever the launch shape: points are grouped in
// chunks of 1024; in a chunk, thread j of 256 adds points 4j, 4j+1, 4j+2,
// 4j+3 in that order; each wave adds its 64 lanes by wave_sum's fixed tree
// (pairs, quads, eights and sixteens inside a row of 16 lanes, then the four
// rows in order); the four wave sums are added in wave order; the chunk sums
// are then added the same way (thread j takes chunks j, j+256, ...).
//
// Two schedules:
//  * chain kernel (N <= 65536): ONE workgroup of 1024 threads runs all the
//    requested steps in a single launch; the data sit in LDS when they fit,
//    else they come from L2 every step.  The random numbers (they do not
//    depend on the state) are drawn for a batch of steps at a time by all 1024
//    threads.  At the sizes of the paper's
//    regression tables (hundreds to thousands of rows) a launch per step would
//    cost several times the arithmetic.
//  * step kernel (any N): one launch per step over min(chunks, 256) workgroups
//    (one a compute unit: each workgroup pays one device-scope release, a cache
//    write-back, before its ticket, and that cost grows with their number);
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
constexpr int kMaxStepBlocks = 256;
constexpr int kStepBatch = 32;            // chunks a workgroup sums between two barriers
constexpr size_t kLdsDataBytes = 144 * 1024;  // data cached in LDS up to this size (160 KB a CU)
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

// n_e of step t: block (index e, step t) of the proposal stream; theta'_e = theta_e + step n_e.
__device__ __forceinline__ double proposal_normal(const MhParams& p, int e, uint32_t t) {
  return normal_from(random_block(p.seed, (uint64_t)e, t, kStreamMhProposal, 0));
}
// ln u of the acceptance test of step t.
__device__ __forceinline__ double accept_log_uniform(const MhParams& p, uint32_t t) {
  return log(u32d(random_block(p.seed, 0, t, kStreamMhAccept, 0).x));
}

// Sum over the 64 lanes of a wave (all active), the same value in every lane.  Data-parallel
// primitive moves inside a row of 16 lanes: lane i adds lane i^1, then i^2 (quad permutes),
// then 7-i of its half row, then 15-i of its row; after each move every lane of the group
// holds the bit-identical group sum (addition commutes).  The four row sums are then read
// from lanes 0, 16, 32, 48 and added in that order.
template <int kCtrl>
__device__ __forceinline__ double dpp_move(double v) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)b, kCtrl, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), kCtrl, 0xF, 0xF, false);
  return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned int)lo);
}
__device__ __forceinline__ double read_lane(double v, int lane) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_readlane((int)b, lane);
  const int hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
  return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned int)lo);
}
__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);  // row_half_mirror
  v += dpp_move<0x140>(v);  // row_mirror
  return ((read_lane(v, 0) + read_lane(v, 16)) + read_lane(v, 32)) + read_lane(v, 48);
}

// Sum over one chunk by a group of 256 consecutive threads (four waves); g = index in the
// group.  xt is stored [K][ld] and y [ld] (HBM or LDS alike), 16-byte aligned, zero beyond N.
// Returns the wave's sum in every lane; the caller adds the four waves in order.
__device__ __forceinline__ double chunk_wave_sum(const float* __restrict__ xt, const float* __restrict__ y,
                                                 int64_t N, int K, int64_t ld, int64_t base,
                                                 const double* th, int g) {
  const int64_t m = base + 4 * g;
  const int64_t at = m < ld ? m : base;  // a valid address; the values are dropped below
  double mean[4];
  const double b = th[K];
#pragma unroll
  for (int i = 0; i < 4; ++i) mean[i] = b;
#pragma unroll 8
  for (int k = 0; k < K; ++k) {
    const float4 v = *reinterpret_cast<const float4*>(xt + (int64_t)k * ld + at);
    const double w = th[k];
    mean[0] += w * (double)v.x;
    mean[1] += w * (double)v.y;
    mean[2] += w * (double)v.z;
    mean[3] += w * (double)v.w;
  }
  const float4 yv = *reinterpret_cast<const float4*>(y + at);
  const double r[4] = {(double)yv.x - mean[0], (double)yv.y - mean[1], (double)yv.z - mean[2],
                       (double)yv.w - mean[3]};
  double s = 0.0;
#pragma unroll
  for (int i = 0; i < 4; ++i) s += m + i < N ? r[i] * r[i] : 0.0;
  return wave_sum(s);
}

// ln f at the proposal from its SSR and ln tau; -inf outside the support of tau.
__device__ __forceinline__ double logf_from_ssr(const MhParams& p, const double* th, double ln_tau,
                                                double ssr) {
  const int K = p.K;
  const double tau = th[K + 1];
  if (!(tau > 0.0)) return -INFINITY;
  double sq = 0.0;
  for (int k = 0; k <= K; ++k) sq += th[k] * th[k];
  return p.ln_prior_const - sq / (2.0 * p.prior_sd * p.prior_sd) - (p.a0 + 1.0) * ln_tau - p.b0 / tau +
         p.ln_x_const - 0.5 * (double)p.N * (kLn2Pi + ln_tau) - ssr / (2.0 * tau);
}

// Adds n chunk sums (LDS or global) in the fixed order; first 256 threads of the block.
// smem4: four doubles.  Result valid in thread 0.
__device__ __forceinline__ double final_sum(const double* part, int n, int tid, double* smem4) {
  double s = 0.0;
  if (tid < 256) {
    for (int c = tid; c < n; c += 256) s += part[c];
    s = wave_sum(s);
    if ((tid & 63) == 0) smem4[tid >> 6] = s;
  }
  __syncthreads();
  return ((smem4[0] + smem4[1]) + smem4[2]) + smem4[3];
}

// ---------------------------------------------------------------- chain kernel
// One workgroup, all steps.  Thread group q (256 threads) takes chunks q, q+4, ...
// The last K + 2 threads each own one parameter (in a register).  The normals
// and ln u of a batch of B = 1024 / (K + 3) steps are drawn by all threads at
// once into LDS tables.  A step has three phases, with a barrier after each:
// (1) chunk sums; (2) thread 0 decides; (3) the owners update theta, write the
// trace row and publish the next proposal (with ln tau', which the otherwise
// idle owner computes while the next step's chunk sums are under way).
constexpr int kTableSlots = 1024;
template <bool kLds>
__global__ __launch_bounds__(1024) void mhreg_chain_kernel(
    const float* __restrict__ xt, const float* __restrict__ y, MhParams p, MhState* __restrict__ st,
    int64_t n_steps, uint32_t first_step, double* __restrict__ trace, int64_t ld) {
  extern __shared__ __align__(16) float data[];  // kLds: xt [K][ld], then y [ld]
  __shared__ double prop[kMaxK + 2];
  __shared__ double wsum[16], part[kMaxChainChunks], smem4[4];
  __shared__ double table[kTableSlots];  // [B][K + 3]: normals of the K + 2 parameters, ln u
  __shared__ double ln_tau_s;
  __shared__ int take_s;
  const int tid = threadIdx.x, K = p.K;
  const int q = tid >> 8, g = tid & 255, wave = tid >> 6;
  const int nchunks = (int)((p.N + kChunk - 1) / kChunk);
  const int e = tid - (1024 - (K + 2));  // parameter owned by this thread, if >= 0
  const bool owner = e >= 0;
  const int row = K + 3, B = kTableSlots / row;
  const int my_step = tid / row, my_item = tid - my_step * row;
  // draws of steps t0 .. t0 + B - 1
  auto fill_table = [&](uint32_t t0) {
    if (my_step < B)
      table[tid] = my_item < K + 2 ? proposal_normal(p, my_item, t0 + (uint32_t)my_step)
                                   : accept_log_uniform(p, t0 + (uint32_t)my_step);
  };
  if (kLds) {
    for (int64_t i = tid; i < (int64_t)(K + 1) * ld; i += 1024) data[i] = i < (int64_t)K * ld ? xt[i] : y[i - (int64_t)K * ld];
  }
  const float* xd = kLds ? data : xt;
  const float* yd = kLds ? data + (int64_t)K * ld : y;
  fill_table(first_step);
  __syncthreads();
  double th_e = 0.0, lf = 0.0;
  unsigned long long acc = 0;
  if (owner) {
    th_e = st->theta[e];
    const double v = th_e + p.step * table[e];
    prop[e] = v;
    if (e == K + 1) ln_tau_s = v > 0.0 ? log(v) : 0.0;
  }
  if (tid == 0) {
    lf = st->logf;
    acc = st->accepted;
  }
  __syncthreads();
  for (int64_t s = 0; s < n_steps; ++s) {
    const int sb = (int)(s % B);  // slot of step s in the table
    const bool in_support = prop[K + 1] > 0.0;
    // (1) sum of squared residuals at the proposal, valid in thread 0
    double ssr = 0.0;
    if (in_support) {
      if (nchunks <= 4) {
        const double w = q < nchunks ? chunk_wave_sum(xd, yd, p.N, K, ld, (int64_t)q * kChunk, prop, g)
                                     : 0.0;
        if ((tid & 63) == 0) wsum[wave] = w;
        __syncthreads();
        if (tid == 0) {
          // what final_sum gives for up to four chunk sums (absent ones are 0.0): lanes 0..3 of
          // wave 0 hold them, the quad moves add (c0 + c1) + (c2 + c3), everything else adds 0.0
          double c[4];
          for (int i = 0; i < 4; ++i)
            c[i] = ((wsum[4 * i] + wsum[4 * i + 1]) + wsum[4 * i + 2]) + wsum[4 * i + 3];
          ssr = (c[0] + c[1]) + (c[2] + c[3]);
        }
      } else {
        for (int c0 = 0; c0 < nchunks; c0 += 4) {
          const int c = c0 + q;
          const double w = c < nchunks
                               ? chunk_wave_sum(xd, yd, p.N, K, ld, (int64_t)c * kChunk, prop, g)
                               : 0.0;
          if ((tid & 63) == 0) wsum[wave] = w;
          __syncthreads();
          if (g == 0 && c < nchunks)
            part[c] = ((wsum[4 * q] + wsum[4 * q + 1]) + wsum[4 * q + 2]) + wsum[4 * q + 3];
          __syncthreads();
        }
        ssr = final_sum(part, nchunks, tid, smem4);
      }
    }
    // (2) the decision of step s
    if (tid == 0) {
      const double lp = in_support ? logf_from_ssr(p, prop, ln_tau_s, ssr) : -INFINITY;
      const bool take = table[sb * row + K + 2] < lp - lf;
      if (take) {
        lf = lp;
        acc += 1;
      }
      take_s = take ? 1 : 0;
    }
    __syncthreads();
    if (sb == B - 1) {  // the table is used up: draw the next batch
      fill_table(first_step + (uint32_t)(s + 1));
      __syncthreads();
    }
    // (3) new state, trace row, next proposal
    if (owner) {
      if (take_s) th_e = prop[e];
      if (trace) trace[s * (K + 3) + e] = th_e;
      const double v = th_e + p.step * table[(sb == B - 1 ? 0 : sb + 1) * row + e];
      prop[e] = v;
      if (e == K + 1) ln_tau_s = v > 0.0 ? log(v) : 0.0;
    }
    if (tid == 0 && trace) trace[s * (K + 3) + K + 2] = lf;
    __syncthreads();
  }
  if (owner) st->theta[e] = th_e;
  if (tid == 0) {
    st->logf = lf;
    st->accepted = acc;
  }
}

// ----------------------------------------------------------------- step kernel
// One step.  With decide = false only ln f at st->theta is computed (into st->logf).
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(6, 8))) void mhreg_step_kernel(
    const float* __restrict__ xt, const float* __restrict__ y, int64_t ld, MhParams p,
    MhState* __restrict__ st, double* part, uint32_t t, bool decide,
    double* __restrict__ trace_row) {
  __shared__ double prop[kMaxK + 2];
  __shared__ double wsum[kStepBatch][4], smem4[4];
  __shared__ bool last_s;
  const int tid = threadIdx.x, K = p.K;
  const int nchunks = (int)((p.N + kChunk - 1) / kChunk);
  if (tid < K + 2)
    prop[tid] = decide ? st->theta[tid] + p.step * proposal_normal(p, tid, t) : st->theta[tid];
  __syncthreads();
  const bool in_support = prop[K + 1] > 0.0;
  if (in_support) {
    // this workgroup's chunks, kStepBatch at a time; no barrier between the chunks of a batch,
    // so the waves of a workgroup run ahead of one another and keep loads in flight
    for (int c0 = blockIdx.x; c0 < nchunks; c0 += kStepBatch * gridDim.x) {
      int j = 0;
      for (int c = c0; j < kStepBatch && c < nchunks; ++j, c += gridDim.x) {
        const double w = chunk_wave_sum(xt, y, p.N, K, ld, (int64_t)c * kChunk, prop, tid);
        if ((tid & 63) == 0) wsum[j][tid >> 6] = w;
      }
      __syncthreads();
      if (tid < j)
        part[c0 + tid * (int)gridDim.x] = ((wsum[tid][0] + wsum[tid][1]) + wsum[tid][2]) + wsum[tid][3];
      __syncthreads();
    }
  }
  if (tid < 64) {
    // the chunk sums above were stored by this wave: release them device-wide (one cache
    // write-back a workgroup, no invalidate), then take the ticket
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    if (tid == 0) {
      const unsigned int ticket = atomicAdd(&st->ticket, 1u);
      last_s = ticket == gridDim.x - 1;
    }
  }
  __syncthreads();
  if (!last_s) return;
  // The workgroup that drew the last ticket: every other workgroup released its chunk sums
  // before its ticket.  Acquire (drops stale cache lines; this workgroup only), then ordinary
  // loads, which unlike atomic ones can all be in flight together.
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  double s = 0.0;
  if (in_support)
    for (int c = tid; c < nchunks; c += 256) s += part[c];  // chunks j, j+256, ...: first level
  s = wave_sum(s);
  if ((tid & 63) == 0) smem4[tid >> 6] = s;
  __syncthreads();
  const double ssr = ((smem4[0] + smem4[1]) + smem4[2]) + smem4[3];
  __shared__ bool take_s;
  if (tid == 0) {
    const double lp = in_support ? logf_from_ssr(p, prop, log(prop[K + 1]), ssr) : -INFINITY;
    if (decide) {
      take_s = accept_log_uniform(p, t) < lp - st->logf;
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

// xt[k][n] = x[n][k]; the padding columns n >= N are zero.
__global__ __launch_bounds__(256) void mhreg_transpose_kernel(const float* __restrict__ x,
                                                               float* __restrict__ xt, int64_t N,
                                                               int K, int64_t ld) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < (int64_t)K * ld; e += stride) {
    const int64_t k = e / ld, n = e - k * ld;
    xt[e] = n < N ? x[n * K + k] : 0.f;
  }
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
  float *xt = nullptr, *y = nullptr;  // xt [K][ld]
  int64_t ld = 0;
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
  (void)hipFree(h->xt); (void)hipFree(h->y); (void)hipFree(h->st); (void)hipFree(h->part);
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
  return h->cfg.N <= 4096;
}

// ln f at the current theta into the state.
int launch_evaluate(augur_mhreg* h) {
  hipLaunchKernelGGL(mhreg_step_kernel, dim3(h->step_blocks), dim3(256), 0, h->stream, h->xt, h->y,
                     h->ld, h->p, h->st, h->part, 0u, false, (double*)nullptr);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

int launch_steps(augur_mhreg* h, int64_t n_steps, double* trace_dev) {
  const int K = h->cfg.K;
  const uint32_t first = (uint32_t)(h->step_index + 1);
  if (use_chain(h)) {
    const int64_t ld = h->ld;
    const size_t data_bytes = sizeof(float) * (size_t)ld * (K + 1);
    if (data_bytes <= kLdsDataBytes) {
      if (!h->lds_attr_set) {
        AUGUR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&mhreg_chain_kernel<true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)kLdsDataBytes));
        h->lds_attr_set = true;
      }
      hipLaunchKernelGGL(mhreg_chain_kernel<true>, dim3(1), dim3(1024), data_bytes, h->stream, h->xt,
                         h->y, h->p, h->st, n_steps, first, trace_dev, ld);
    } else {
      hipLaunchKernelGGL(mhreg_chain_kernel<false>, dim3(1), dim3(1024), 0, h->stream, h->xt, h->y,
                         h->p, h->st, n_steps, first, trace_dev, ld);
    }
    AUGUR_HIP_TRY(hipGetLastError());
  } else {
    for (int64_t s = 0; s < n_steps; ++s) {
      hipLaunchKernelGGL(mhreg_step_kernel, dim3(h->step_blocks), dim3(256), 0, h->stream, h->xt,
                         h->y, h->ld, h->p, h->st, h->part, first + (uint32_t)s, true,
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
      (void)hipGetLastError(); /* or the runtime hands it to the next caller */ \
      free_all(h);                                                                          \
      delete h;                                                                             \
      return AUGUR_ERR_HIP;                                                                 \
    }                                                                                       \
  } while (0)

  const hipMemcpyKind in_kind = device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
  h->ld = round_up(N, 64);
  float* x_in = nullptr;  // the caller's layout, on the device; only needed until the transpose
  if (device_ptrs(h)) {
    x_in = const_cast<float*>(x);
  } else {
    AUGUR_CREATE_TRY(hipMalloc(&x_in, sizeof(float) * (size_t)N * K));
    hipError_t e_up = hipMemcpyAsync(x_in, x, sizeof(float) * (size_t)N * K, hipMemcpyHostToDevice, h->stream);
    if (e_up != hipSuccess) {
      (void)hipFree(x_in);
      AUGUR_CREATE_TRY(e_up);
    }
  }
  struct StagingGuard {
    float* p;
    hipStream_t s;
    ~StagingGuard() {
      if (p) {
        (void)hipStreamSynchronize(s);
        (void)hipFree(p);
      }
    }
  } staging{device_ptrs(h) ? nullptr : x_in, h->stream};
  AUGUR_CREATE_TRY(hipMalloc(&h->xt, sizeof(float) * (size_t)h->ld * K));
  AUGUR_CREATE_TRY(hipMalloc(&h->y, sizeof(float) * (size_t)h->ld));
  AUGUR_CREATE_TRY(hipMemsetAsync(h->y, 0, sizeof(float) * (size_t)h->ld, h->stream));
  AUGUR_CREATE_TRY(hipMalloc(&h->st, sizeof(MhState)));
  AUGUR_CREATE_TRY(hipMalloc(&h->part, sizeof(double) * (size_t)h->nchunks));
  AUGUR_CREATE_TRY(hipMalloc(&h->bad, sizeof(unsigned long long)));
  AUGUR_CREATE_TRY(hipMemsetAsync(h->st, 0, sizeof(MhState), h->stream));
  AUGUR_CREATE_TRY(hipMemsetAsync(h->bad, 0, sizeof(unsigned long long), h->stream));
  AUGUR_CREATE_TRY(hipMemcpyAsync(h->y, y, sizeof(float) * (size_t)N, in_kind, h->stream));
  hipLaunchKernelGGL(mhreg_transpose_kernel, dim3(1024), dim3(256), 0, h->stream, x_in, h->xt, N, K,
                     h->ld);
  hipLaunchKernelGGL(mhreg_check_kernel, dim3(512), dim3(256), 0, h->stream, x_in, h->y, N, K,
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
    (void)hipGetLastError();  // or the runtime hands the error to the next caller
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

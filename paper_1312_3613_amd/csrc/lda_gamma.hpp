// The theta and phi steps (Sect. 4.3, Alg. 1 and 2): Dirichlet draws from normalised Gamma draws.
// Part of the LDA translation unit (lda.hip includes these files in order; they share one
// anonymous namespace's worth of helpers and are not meant to be included anywhere else).
#pragma once

namespace {

// ------------------------------------------------------------ resample theta
// theta_d ~ Dirichlet(alpha + n_dk[d][.]) for every document in parallel
// (Sect. 4.3; App. B, Alg. 2): K Gamma draws in the log domain, normalised by
// their sum (log-sum-exp in fp64), stored as fp32 floored at FLT_MIN (fp64 state: as doubles
// floored at DBL_MIN).
//
// One wave owns `rows` consecutive documents (rows * K variables, about 25 per
// lane).  Rejection sampling diverges, so each lane walks its own variables:
// every trip of the loop is one attempt on the lane's current variable, and an
// accepted lane moves on without waiting for the others.  The draws wait in the
// wave's LDS strip; then each row is normalised by the whole wave.
template <typename T>
__global__ __launch_bounds__(256) void lda_resample_theta_kernel(
    const int32_t* __restrict__ n_dk, T* __restrict__ theta, int D, int K, int ldk, int rows,
    double alpha, const GammaShape* __restrict__ shapes, const double2* __restrict__ log_table,
    const double* __restrict__ exp_table, uint64_t seed, SweepRef sweep_ref,
    unsigned long long* __restrict__ n_capped) {
  extern __shared__ double lg_all[];
  const uint32_t sweep = sweep_ref.get();
  __shared__ double2 lt[kLogTableSize];
  __shared__ double et[kExpTableSize];
  for (int i = threadIdx.x; i < kLogTableSize; i += blockDim.x) lt[i] = log_table[i];
  for (int i = threadIdx.x; i < kExpTableSize; i += blockDim.x) et[i] = exp_table[i];
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int d0 = (blockIdx.x * 4 + wave) * rows;
  if (d0 >= D) return;
  const int nrows = min(rows, D - d0);
  const int total = nrows * K;
  double* lg = lg_all + (size_t)wave * rows * K;

  // Variable e of the wave = row e / K, topic e % K.  The lanes do not own fixed lists: a lane
  // whose draw is accepted takes the first variable that nobody has taken yet (the lanes that
  // finish in the same trip take consecutive ones, in lane order), so that the wave runs dry
  // only in its last trips, however the rejections fall.  Every variable's random numbers are
  // keyed by its own index: which lane draws it does not matter.
  const float inv_K = 1.0f / (float)K;
  auto row_of = [&](int e_) {  // e_ / K for 0 <= e_ < 16384 (the quotient of the rounded floats is off by one at most)
    int q = (int)(((float)e_ + 0.5f) * inv_K);
    q -= q * K > e_ ? 1 : 0;
    q += (q + 1) * K <= e_ ? 1 : 0;
    return q;
  };
  int e = lane, r = row_of(lane), k = lane - r * K;
  int next = 64;  // the first variable not yet taken (the same in every lane)
  uint32_t attempt = 0;
  bool capped = false;
  GammaShape g = gamma_shape_count(shapes, alpha, e < total ? n_dk[(size_t)(d0 + r) * ldk + k] : 0);
  while (__any(e < total)) {
    bool done = false;
    if (e < total) {
      const uint64_t index = (uint64_t)(d0 + r) * (uint64_t)K + (uint64_t)k;
      double x;
      done = gamma_attempt(g, random_block(seed, index, sweep, kStreamTheta, attempt), x, lt);
      if (!done && ++attempt == (uint32_t)kGammaAttemptCap) {
        done = true;
        capped = true;
        x = g.ln_d;
      }
      if (done) lg[e] = x;
    }
    const uint64_t finished = __ballot(done);
    if (done) {
      e = next + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(finished >> 32),
                                                __builtin_amdgcn_mbcnt_lo((uint32_t)finished, 0u));
      r = row_of(e);
      k = e - r * K;
      attempt = 0;
      if (e < total) g = gamma_shape_count(shapes, alpha, n_dk[(size_t)(d0 + r) * ldk + k]);
    }
    next += __popcll(finished);
  }
  wave_lds_fence();
  for (int rr = 0; rr < nrows; ++rr) {
    double* row = lg + (size_t)rr * K;
    double m = -INFINITY;
    for (int kk = lane; kk < K; kk += 64) m = row[kk] > m ? row[kk] : m;
    m = wave_allreduce_max(m);
    double sum = 0.0;
    for (int kk = lane; kk < K; kk += 64) {  // each lane revisits only its own entries
      const double ex = exp_tab(row[kk] - m, et);
      row[kk] = ex;
      sum += ex;
    }
    sum = wave_allreduce_sum(sum);
    const double inv = 1.0 / sum;
    for (int kk = lane; kk < K; kk += 64) {
      double p = row[kk] * inv;
      p = p < state_floor<T>() ? state_floor<T>() : p;
      theta[(size_t)(d0 + rr) * ldk + kk] = (T)p;
    }
  }
  if (capped) atomicAdd(n_capped, 1ULL);
}

// -------------------------------------------------------------- resample phi
// phi_k ~ Dirichlet(beta + n_wk[.][k]) for every topic (Sect. 4.3, Alg. 1): a
// V x K matrix of Gamma draws, element-parallel because K is small, then one
// normaliser per topic.  Here the normaliser is a column log-sum-exp: pass 1
// draws and keeps a running (max, sum) per column per block of rows, pass 2
// merges the blocks, pass 3 writes exp(lg - L_k).  In pass 1 a thread owns one
// column of its block of rows and retries on its own variable (see theta).
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(6, 6))) void lda_phi_draw_kernel(
    const int32_t* __restrict__ n_wk, double* __restrict__ lg, double2* __restrict__ partial, int V,
    int K, int ldk, int rows_per_block, int groups, int n_row_blocks, int col_w, double beta,
    const GammaShape* __restrict__ shapes, const double2* __restrict__ log_table,
    const double* __restrict__ exp_table, uint64_t seed, SweepRef sweep_ref,
    unsigned long long* __restrict__ n_capped) {
  __shared__ double2 lt[kLogTableSize];
  const uint32_t sweep = sweep_ref.get();
  __shared__ double et[kExpTableSize];
  __shared__ GammaShape small_shapes[kShapeLds];  // the constants of the smallest counts: most entries of the table
  for (int i = threadIdx.x; i < kLogTableSize; i += blockDim.x) lt[i] = log_table[i];
  for (int i = threadIdx.x; i < kExpTableSize; i += blockDim.x) et[i] = exp_table[i];
  for (int i = threadIdx.x; i < kShapeLds; i += blockDim.x) small_shapes[i] = shapes[i];
  __syncthreads();
  // The workgroup covers columns [blockIdx.y col_w, +col_w) (all K of them unless K > 512).
  // thread t: column t % col_w of that range, row block blockIdx.x * groups + t / col_w.
  // Several row blocks share a workgroup so that K need not be a multiple of the wave size
  // to keep the lanes busy.
  const int gi = (int)threadIdx.x / col_w;
  const int k = (int)blockIdx.y * col_w + ((int)threadIdx.x - gi * col_w);
  const int rb = blockIdx.x * groups + gi;
  const bool active = gi < groups && rb < n_row_blocks && k < K;
  const int v0 = active ? rb * rows_per_block : 0;
  const int v1 = active ? min(V, v0 + rows_per_block) : 0;
  bool capped = false;
  int v = v0;
  double m = -INFINITY, s = 0.0;
  uint32_t attempt = 0;
  GammaShape g = gamma_shape_count(shapes, beta, v < v1 ? n_wk[(size_t)v * ldk + k] : 0);
  // the count of the variable after the current one, asked for one variable ahead: when a draw
  // is accepted the next one's constants are a table look-up away, not two dependent loads
  int n_next = v + 1 < v1 ? n_wk[(size_t)(v + 1) * ldk + k] : 0;
  while (__any(v < v1)) {
    if (v < v1) {
      const size_t e = (size_t)v * ldk + k;
      double x;
      bool done = gamma_attempt(
          g, random_block(seed, (uint64_t)v * (uint64_t)K + (uint64_t)k, sweep, kStreamPhi, attempt),
          x, lt);
      if (!done && ++attempt == (uint32_t)kGammaAttemptCap) {
        done = true;
        capped = true;
        x = g.ln_d;
      }
      if (done) {
        lg[e] = x;
        // running (max, sum of exp(. - max)); one exp and no branch, so lanes that raise
        // their maximum and lanes that do not share the instructions
        const double dx = x - m;               // +inf on the first row: e = 0, s = 1
        const double ex = exp_tab(-fabs(dx), et);
        s = dx > 0.0 ? fma(s, ex, 1.0) : s + ex;
        m = dx > 0.0 ? x : m;
        ++v;
        attempt = 0;
        if (v < v1) g = n_next < kShapeLds ? small_shapes[n_next] : gamma_shape_count(shapes, beta, n_next);
        if (v + 1 < v1) n_next = n_wk[(size_t)(v + 1) * ldk + k];
      }
    }
  }
  if (active) partial[(size_t)k * n_row_blocks + rb] = make_double2(m, s);  // [K][row blocks]
  if (capped) atomicAdd(n_capped, 1ULL);
}

// One block per topic: merge the per-block (max, sum) pairs in a fixed order.
__global__ __launch_bounds__(1024) void lda_phi_norm_kernel(const double2* __restrict__ partial,
                                                             double* __restrict__ logZ, int nblk,
                                                             int K) {
  __shared__ double sm[1024], ss[1024];
  const int k = blockIdx.x;
  double m = -INFINITY, s = 0.0;
  for (int b = threadIdx.x; b < nblk; b += 1024) {
    const double2 p = partial[(size_t)k * nblk + b];
    if (p.x > m) {
      s = s * exp(m - p.x) + p.y;
      m = p.x;
    } else {
      s += p.y * exp(p.x - m);
    }
  }
  sm[threadIdx.x] = m;
  ss[threadIdx.x] = s;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      const double m2 = sm[threadIdx.x + o], s2 = ss[threadIdx.x + o];
      double m1 = sm[threadIdx.x], s1 = ss[threadIdx.x];
      if (m2 > m1) {
        s1 = s1 * exp(m1 - m2) + s2;
        m1 = m2;
      } else if (m2 > -INFINITY) {
        s1 += s2 * exp(m2 - m1);
      }
      sm[threadIdx.x] = m1;
      ss[threadIdx.x] = s1;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) logZ[k] = sm[0] + log(ss[0]);
}

template <typename T>
__global__ __launch_bounds__(256) void lda_phi_write_kernel(const double* __restrict__ lg,
                                                             const double* __restrict__ logZ,
                                                             T* __restrict__ phi, int V, int K,
                                                             int ldk) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)V * ldk) return;
  const int k = (int)(e % ldk);
  if (k >= K) return;
  double p = exp(lg[e] - logZ[k]);
  p = p < state_floor<T>() ? state_floor<T>() : p;
  phi[e] = (T)p;
}

}  // namespace

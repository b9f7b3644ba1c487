// The log joint and the log marginal (Sect. 4.1), Gamma shape tables and input validation.
// Part of the LDA translation unit (lda.hip includes these files in order; they share one
// anonymous namespace's worth of helpers and are not meant to be included anywhere else).
#pragma once

namespace {

// -------------------------------------------------------------------- loglik
// Per-token terms of the log joint (Sect. 4.1: log space, terms evaluated in
// parallel and summed): ln theta[d][z_i] + ln phi[w_i][z_i], and
// ln sum_k theta[d][k] phi[w_i][k] for the marginal.  One wave per segment
// slot (a whole document unless it is split) with theta_d as doubles in LDS and a quad
// per token, 64 contiguous bytes of the phi row per load: the load shape of the
// sampler.  Every product is formed in fp64 from its two fp32 factors (exact: 24 + 24
// bits) and all sums are fp64, so the result differs from a sum in any other order by
// fp64 rounding only.  The three logarithms of a token are taken side by side by three
// lanes of its quad with the table logarithm.
//
// NS16 > 0: that many stripes of 16 topics, unrolled (K <= 256); NS16 = 0: the
// number of stripes is read at run time (K <= 1024).  Columns k >= K of theta and
// phi rows (padding up to the row stride) are never used, whatever they hold.
// Word ids and topics are clamped into their tables, so that arrays that were
// never validated cannot make the kernel read outside them.
__device__ __forceinline__ double log_any(double x, const double2* __restrict__ lt) {
  // the table logarithm needs a positive, finite, normal argument; zero, negative,
  // non-finite and subnormal ones (degenerate states only) take the general routine
  if (__builtin_expect(!(x >= DBL_MIN && x <= DBL_MAX), 0)) return log(x);
  return log_tab(x, lt);
}
template <int NS16>
__global__ __launch_bounds__(256) void lda_loglik_tokens_kernel(
    const int32_t* __restrict__ w, const int32_t* __restrict__ z,
    const int64_t* __restrict__ doc_off, const int32_t* __restrict__ seg_base, int n_segs,
    const float* __restrict__ theta, const float* __restrict__ phi, int D, int V, int K, int ldk,
    const double2* __restrict__ log_table, double* __restrict__ part_lik,
    double* __restrict__ part_marg) {
  extern __shared__ __align__(16) double theta_lds[];  // [4][16 * stripes]
  __shared__ double2 lt[kLogTableSize];
  __shared__ double smem[8];
  for (int i = threadIdx.x; i < kLogTableSize; i += blockDim.x) lt[i] = log_table[i];
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tq = lane >> 2, q = lane & 3;
  const int stripes = NS16 > 0 ? NS16 : (ldk + 15) >> 4;
  double* th = theta_lds + (size_t)wave * 16 * stripes;
  const uint32_t row_bytes = 4u * (uint32_t)ldk;
  const uint32_t lane_off = 16u * (uint32_t)q;
  const char* phi_bytes = reinterpret_cast<const char*>(phi);
  // the lane's chunk of stripe c: 16 bytes of the row at 64 c + 16 q, pulled back into the row
  // where the last stripe overhangs it; entries at or past column K count as zero
  auto chunk = [&](uint32_t row_off, int c) {
    const uint32_t off = min(64u * (uint32_t)c + lane_off, row_bytes - 16u);
    float4 y = *reinterpret_cast<const float4*>(phi_bytes + (row_off + off));
    const int col = 16 * c + 4 * q;
    if (16 * c + 16 > K) {  // the same for the whole wave
      y.x = col + 0 < K ? y.x : 0.f;
      y.y = col + 1 < K ? y.y : 0.f;
      y.z = col + 2 < K ? y.z : 0.f;
      y.w = col + 3 < K ? y.w : 0.f;
    }
    return y;
  };
  double lik = 0.0, marg = 0.0;
  for (int seg = blockIdx.x * 4 + wave; seg < n_segs; seg += gridDim.x * 4) {
    const Segment sg = segment_of(doc_off, seg_base, D, seg);
    const int d = sg.d;
    wave_lds_fence();  // the previous document's reads are done
    for (int k = lane; k < 16 * stripes; k += 64)
      th[k] = k < K ? (double)theta[(size_t)d * ldk + k] : 0.0;
    wave_lds_fence();
    const int64_t a = sg.first > sg.a ? sg.first : sg.a, b = sg.end;
    for (int64_t i0 = a; i0 < b; i0 += 16) {
      // theta_d does not change inside the loop; an offset the compiler cannot see through
      // keeps it from reading the whole row once and holding it in registers
      int theta_off = 4 * q;
      asm volatile("" : "+v"(theta_off));
      const double* th_q = th + theta_off;
      const int64_t i = i0 + tq;
      const bool valid = i < b;
      const int64_t ii = valid ? i : a;  // a quad past the end redoes the first token; not counted
      const int wi = min(max(w[ii], 0), V - 1);
      const int zi = min(max(z[ii], 0), K - 1);
      const uint32_t row_off = (uint32_t)wi * row_bytes;
      double s = 0.0;
      if constexpr (NS16 > 0) {
        float4 y[NS16];
#pragma unroll
        for (int c = 0; c < NS16; ++c) y[c] = chunk(row_off, c);
#pragma unroll
        for (int c = 0; c < NS16; ++c) {
          const double2 x01 = *reinterpret_cast<const double2*>(th_q + 16 * c);
          const double2 x23 = *reinterpret_cast<const double2*>(th_q + 16 * c + 2);
          s = fma(x01.x, (double)y[c].x, s);
          s = fma(x01.y, (double)y[c].y, s);
          s = fma(x23.x, (double)y[c].z, s);
          s = fma(x23.y, (double)y[c].w, s);
        }
      } else {
#pragma unroll 4
        for (int c = 0; c < stripes; ++c) {
          const float4 y = chunk(row_off, c);
          const double2 x01 = *reinterpret_cast<const double2*>(th_q + 16 * c);
          const double2 x23 = *reinterpret_cast<const double2*>(th_q + 16 * c + 2);
          s = fma(x01.x, (double)y.x, s);
          s = fma(x01.y, (double)y.y, s);
          s = fma(x23.x, (double)y.z, s);
          s = fma(x23.y, (double)y.w, s);
        }
      }
      s += __shfl_xor(s, 1, 64);
      s += __shfl_xor(s, 2, 64);
      // lane 0 of the quad: ln of the sum; lane 1: ln theta[d][z]; lane 2: ln phi[w][z]
      const double th_z = th[zi];
      const double ph_z =
          (double)*reinterpret_cast<const float*>(phi_bytes + (row_off + 4u * (uint32_t)zi));
      const double arg = q == 0 ? s : q == 1 ? th_z : q == 2 ? ph_z : 1.0;
      const double lg = log_any(arg, lt);
      marg += valid && q == 0 ? lg : 0.0;
      lik += valid && (q == 1 || q == 2) ? lg : 0.0;
    }
  }
  block_partial_sum(lik, part_lik, smem);
  block_partial_sum(marg, part_marg, smem);
}

// The same terms with the phi rows of the most frequent words read from LDS: the workgroup
// shape, the cache, the processing order (wz, ord) and the LDS budget of the resident z kernel
// (lda_sample_z_hot_kernel); per wave theta_d as doubles, then the chunk's wz and ord strips.
// One trip of the inner loop issues the row loads of a 16-token iteration that reads memory,
// runs an iteration that reads LDS only while they are on their way, then consumes them.
// Blocks past the grid's size in the partial arrays are cleared here (the finishing kernel adds
// all kRedBlocks of them).
template <int NS16>
__global__ __launch_bounds__(64 * kHotWaves) void lda_loglik_hot_kernel(
    const int32_t* __restrict__ wz, const uint8_t* __restrict__ ord, const int32_t* __restrict__ z,
    const int64_t* __restrict__ doc_off, const int32_t* __restrict__ seg_base, int n_segs,
    const float* __restrict__ theta, const float* __restrict__ phi, int D, int K, int ldk,
    const double2* __restrict__ log_table, double* __restrict__ part_lik,
    double* __restrict__ part_marg, const int32_t* __restrict__ hot_words, int n_hot) {
  extern __shared__ __align__(16) unsigned char lds[];
  __shared__ double2 lt[kLogTableSize];
  __shared__ double smem[kHotWaves];
  constexpr int kRowLds = 64 * NS16 + hot_row_pad_bytes(NS16);
  constexpr int kWaveBytes = hot_wave_bytes(NS16, true);  // the z kernel's strip: 128 NS16 + 1280 bytes are used
  static_assert(128 * NS16 + 1024 + 256 <= kWaveBytes, "the strips of a wave must fit the z kernel's");
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t row_bytes = 4u * (uint32_t)ldk;  // 64 NS16
  for (int i = threadIdx.x; i < kLogTableSize; i += blockDim.x) lt[i] = log_table[i];
  {
    const int pieces = 4 * NS16;
    for (int e = threadIdx.x; e < n_hot * pieces; e += blockDim.x) {
      const int s = e / pieces, pc = e - s * pieces;
      const float4 v = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(phi) +
                                                       ((size_t)(uint32_t)hot_words[s] * row_bytes + 16u * pc));
      *reinterpret_cast<float4*>(lds + (size_t)s * kRowLds + 16 * pc) = v;
    }
  }
  for (int i = (int)(gridDim.x + blockIdx.x * blockDim.x + threadIdx.x); i < kRedBlocks;
       i += (int)(blockDim.x * gridDim.x)) {
    part_lik[i] = 0.0;
    part_marg[i] = 0.0;
  }
  __syncthreads();
  unsigned char* mine = lds + (size_t)n_hot * kRowLds + (size_t)wave * kWaveBytes;
  double* th = reinterpret_cast<double*>(mine);                          // [16 NS16]
  uint32_t* strip_w = reinterpret_cast<uint32_t*>(mine + 128 * NS16);    // wz of the j-th token in order
  uint8_t* strip_o = mine + 128 * NS16 + 1024;                           // its position in the chunk
  const int tq = lane >> 2, q = lane & 3;
  const char* phi_bytes = reinterpret_cast<const char*>(phi);
  const uint32_t lane_off = 16u * (uint32_t)q;
  double lik = 0.0, marg = 0.0;

  // the three logarithms of a token, by three lanes of its quad
  auto add_terms = [&](double s, int zi, double ph_z, bool valid) {
    s += __shfl_xor(s, 1, 64);
    s += __shfl_xor(s, 2, 64);
    const double arg = q == 0 ? s : q == 1 ? th[zi] : q == 2 ? ph_z : 1.0;
    const double lg = log_any(arg, lt);
    marg += valid && q == 0 ? lg : 0.0;
    lik += valid && (q == 1 || q == 2) ? lg : 0.0;
  };

  for (int seg = blockIdx.x * kHotWaves + wave; seg < n_segs; seg += gridDim.x * kHotWaves) {
    const Segment sg = segment_of(doc_off, seg_base, D, seg);
    wave_lds_fence();  // the previous segment's reads of theta are done
    for (int k = lane; k < 16 * NS16; k += 64) th[k] = k < K ? (double)theta[(size_t)sg.d * ldk + k] : 0.0;
    const int32_t* z_seg = z + sg.first;
    const int rel_a = (int)(sg.a - sg.first);
    const int rel_b = (int)(sg.end - sg.first);
    for (int rbase = 0; rbase < rel_b; rbase += 256) {
      const int lo = max(rel_a, rbase);
      const int hi = min(rel_b, rbase + 256);
      const int n_valid = hi - lo;
      int n_cached = 0;
      {
        const int32_t* wz_c = wz + (sg.first + lo);
        const uint8_t* ord_c = ord + (sg.first + lo);
        uint32_t wv[4];
        uint8_t ov[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = lane + 64 * e;
          wv[e] = j < n_valid ? (uint32_t)wz_c[j] : 0u;
          ov[e] = j < n_valid ? ord_c[j] : (uint8_t)0;
        }
        wave_lds_fence();  // earlier reads of the strips are done
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          strip_w[lane + 64 * e] = wv[e];
          strip_o[lane + 64 * e] = ov[e];
          n_cached += __popcll(__ballot((wv[e] >> 24) != 0u));
        }
        wave_lds_fence();
      }
      const int n_hot_iters = __builtin_amdgcn_readfirstlane(n_cached) >> 4;
      const int cold0 = 16 * n_hot_iters;
      const int n_cold_iters = (n_valid - cold0 + 15) >> 4;
      const int n_trips = max(n_hot_iters, n_cold_iters);
      for (int it = 0; it < n_trips; ++it) {
        const bool do_cold = it < n_cold_iters, do_hot = it < n_hot_iters;
        float4 ph[NS16];
        float ph_z_c = 1.f;
        int zi_c = 0;
        bool valid_c = false;
        if (do_cold) {
          const int j0 = cold0 + 16 * it;
          const int j = j0 + tq;
          valid_c = j < n_valid;
          const int jj = valid_c ? j : j0;  // a quad past the end redoes the iteration's first token; not counted
          const uint32_t row_off = __umul24(strip_w[jj] & 0xFFFFFFu, row_bytes);
          zi_c = min(max(z_seg[rbase + (int)strip_o[jj]], 0), K - 1);
          const char* rowp = phi_bytes + (size_t)(row_off + lane_off);
#pragma unroll
          for (int c = 0; c < NS16; ++c) ph[c] = *reinterpret_cast<const float4*>(rowp + 64 * c);
          ph_z_c = *reinterpret_cast<const float*>(phi_bytes + (size_t)(row_off + 4u * (uint32_t)zi_c));
        }
        asm volatile("" ::: "memory");  // the loads above are issued before anything below starts
        if (do_hot) {
          const int j = 16 * it + tq;
          const uint32_t wv = strip_w[j];
          const int zi = min(max(z_seg[rbase + (int)strip_o[j]], 0), K - 1);
          const unsigned char* crow = lds + (size_t)((wv >> 24) - 1u) * kRowLds;
          int theta_off = 4 * q;
          asm volatile("" : "+v"(theta_off));  // or theta_d is read once and held in registers
          const double* th_q = th + theta_off;
          double s = 0.0;
#pragma unroll
          for (int c = 0; c < NS16; ++c) {
            const float4 y = *reinterpret_cast<const float4*>(crow + 64 * c + 16 * q);
            const double2 x01 = *reinterpret_cast<const double2*>(th_q + 16 * c);
            const double2 x23 = *reinterpret_cast<const double2*>(th_q + 16 * c + 2);
            s = fma(x01.x, (double)y.x, s);
            s = fma(x01.y, (double)y.y, s);
            s = fma(x23.x, (double)y.z, s);
            s = fma(x23.y, (double)y.w, s);
          }
          add_terms(s, zi, (double)*reinterpret_cast<const float*>(crow + 4 * zi), true);
        }
        if (do_cold) {
          int theta_off = 4 * q;
          asm volatile("" : "+v"(theta_off));
          const double* th_q = th + theta_off;
          double s = 0.0;
#pragma unroll
          for (int c = 0; c < NS16; ++c) {
            const double2 x01 = *reinterpret_cast<const double2*>(th_q + 16 * c);
            const double2 x23 = *reinterpret_cast<const double2*>(th_q + 16 * c + 2);
            s = fma(x01.x, (double)ph[c].x, s);
            s = fma(x01.y, (double)ph[c].y, s);
            s = fma(x23.x, (double)ph[c].z, s);
            s = fma(x23.y, (double)ph[c].w, s);
          }
          add_terms(s, zi_c, (double)ph_z_c, valid_c);
        }
      }
    }
  }
  // (the sum over a workgroup of 16 waves)
  lik = wave_allreduce_sum(lik);
  marg = wave_allreduce_sum(marg);
  if (lane == 0) smem[wave] = lik;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int i = 0; i < kHotWaves; ++i) t += smem[i];
    part_lik[blockIdx.x] = t;
  }
  __syncthreads();
  if (lane == 0) smem[wave] = marg;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int i = 0; i < kHotWaves; ++i) t += smem[i];
    part_marg[blockIdx.x] = t;
  }
}

// The same per-token terms for the fp64 state: theta and phi are doubles, nothing is converted.
__global__ __launch_bounds__(256) void lda_loglik_tokens_f64_kernel(
    const int32_t* __restrict__ w, const int32_t* __restrict__ z,
    const int64_t* __restrict__ doc_off, const int32_t* __restrict__ seg_base, int n_segs,
    const double* __restrict__ theta, const double* __restrict__ phi, int D, int V, int K, int ldk,
    const double2* __restrict__ log_table, double* __restrict__ part_lik,
    double* __restrict__ part_marg) {
  extern __shared__ __align__(16) double theta_lds[];  // [4][ldk16]
  __shared__ double2 lt[kLogTableSize];
  __shared__ double smem[8];
  for (int i = threadIdx.x; i < kLogTableSize; i += blockDim.x) lt[i] = log_table[i];
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tq = lane >> 2, q = lane & 3;
  const int ldk16 = (ldk + 15) & ~15;
  const int stripes = ldk16 >> 4;
  double* th = theta_lds + (size_t)wave * ldk16;
  double lik = 0.0, marg = 0.0;
  for (int seg = blockIdx.x * 4 + wave; seg < n_segs; seg += gridDim.x * 4) {
    const Segment sg = segment_of(doc_off, seg_base, D, seg);
    wave_lds_fence();
    for (int k = lane; k < ldk16; k += 64) th[k] = k < K ? theta[(size_t)sg.d * ldk + k] : 0.0;
    wave_lds_fence();
    const int64_t a = sg.first > sg.a ? sg.first : sg.a, b = sg.end;
    for (int64_t i0 = a; i0 < b; i0 += 16) {
      const int64_t i = i0 + tq;
      const bool valid = i < b;
      const int64_t ii = valid ? i : a;
      const int wi = min(max(w[ii], 0), V - 1);
      const int zi = min(max(z[ii], 0), K - 1);
      const double* row = phi + (size_t)wi * ldk;
      double s = 0.0;
      for (int c = 0; c < stripes; ++c) {
        const int col = 16 * c + 4 * q;
#pragma unroll
        for (int e = 0; e < 4; ++e) s = fma(th[col + e], col + e < K ? row[col + e] : 0.0, s);
      }
      s = quad_sum_f64(s);
      const double arg = q == 0 ? s : q == 1 ? th[zi] : q == 2 ? row[zi] : 1.0;
      const double lg = log_any(arg, lt);
      marg += valid && q == 0 ? lg : 0.0;
      lik += valid && (q == 1 || q == 2) ? lg : 0.0;
    }
  }
  block_partial_sum(lik, part_lik, smem);
  block_partial_sum(marg, part_marg, smem);
}

// Sum of ln x over the K real columns of a [rows][ldk] matrix (ldk a multiple of 4: a
// thread takes four entries of one row at a time).
template <typename T>
__global__ __launch_bounds__(256) void sum_log_kernel(const T* __restrict__ x, int64_t rows,
                                                       int K, int ldk,
                                                       const double2* __restrict__ log_table,
                                                       double* __restrict__ part) {
  __shared__ double2 lt[kLogTableSize];
  __shared__ double smem[8];
  for (int i = threadIdx.x; i < kLogTableSize; i += blockDim.x) lt[i] = log_table[i];
  __syncthreads();
  double s = 0.0;
  const int per_row = ldk >> 2;
  const int64_t total = rows * per_row;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
       e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = e / per_row;
    const int col = 4 * (int)(e - r * per_row);
    // rows are padded to a multiple of 16 entries: four at a time stay inside the row
    T v[4];
    if constexpr (sizeof(T) == sizeof(float)) {
      const float4 f = *reinterpret_cast<const float4*>(x + r * ldk + col);
      v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
    } else {
      const double2 lo = *reinterpret_cast<const double2*>(x + r * ldk + col);
      const double2 hi = *reinterpret_cast<const double2*>(x + r * ldk + col + 2);
      v[0] = lo.x; v[1] = lo.y; v[2] = hi.x; v[3] = hi.y;
    }
    if (col + 0 < K) s += log_any((double)v[0], lt);
    if (col + 1 < K) s += log_any((double)v[1], lt);
    if (col + 2 < K) s += log_any((double)v[2], lt);
    if (col + 3 < K) s += log_any((double)v[3], lt);
  }
  block_partial_sum(s, part, smem);
}

// Adds the block partials of the three kernels above in a fixed order and forms the two
// outputs: out[0] = log joint = prior terms + token terms, out[1] = log marginal.
// red = [4][kRedBlocks]: token terms, marginal terms, sum ln theta, sum ln phi.
// c_theta, c_phi: the normalising constants of the two Dirichlet priors summed over
// documents and topics; am1 = alpha - 1, bm1 = beta - 1.
__global__ __launch_bounds__(256) void lda_loglik_finish_kernel(const double* __restrict__ red,
                                                                 double c_theta, double am1,
                                                                 double c_phi, double bm1,
                                                                 double* __restrict__ out) {
  __shared__ double sh[4][256];
  const int t = threadIdx.x;
  for (int g = 0; g < 4; ++g) {
    double s = 0.0;
    for (int i = t; i < kRedBlocks; i += 256) s += red[(size_t)g * kRedBlocks + i];
    sh[g][t] = s;
  }
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (t < o)
      for (int g = 0; g < 4; ++g) sh[g][t] += sh[g][t + o];
    __syncthreads();
  }
  if (t == 0) {
    out[0] = (c_theta + am1 * sh[2][0]) + (c_phi + bm1 * sh[3][0]) + sh[0][0];
    out[1] = sh[1][0];
  }
}

// Per-handle tables of Gamma shape constants for a0 + n, n = 0 .. kShapeTable - 1.
__global__ __launch_bounds__(256) void shape_table_kernel(GammaShape* __restrict__ table, double a0) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n < kShapeTable) table[n] = gamma_shape(a0 + (double)n);
}

// --------------------------------------------------------------- validation
__global__ __launch_bounds__(256) void check_range_kernel(const int32_t* __restrict__ a, int64_t n,
                                                           int32_t lo, int32_t hi,
                                                           unsigned long long* __restrict__ bad) {
  unsigned long long c = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x)
    if (a[i] < lo || a[i] >= hi) ++c;
  if (c) atomicAdd(bad, c);
}

// doc_off[d+1] = inclusive prefix of doc_len on the host for host pointers; for
// device pointers a single block scans (D is at most a few 10^5).
__global__ __launch_bounds__(1024) void doc_offsets_kernel(const int32_t* __restrict__ doc_len,
                                                            int64_t* __restrict__ doc_off, int D,
                                                            unsigned long long* __restrict__ bad) {
  __shared__ int64_t chunk_sum[1024];
  const int t = threadIdx.x;
  const int per = (D + 1023) / 1024;
  const int lo = min(D, t * per), hi = min(D, lo + per);
  int64_t s = 0;
  unsigned long long neg = 0;
  // bad == NULL: nobody reads a count of negative entries; they are taken as 0, so that the
  // offsets never decrease
  const bool clamp = bad == nullptr;
  for (int d = lo; d < hi; ++d) {
    if (doc_len[d] < 0) ++neg;
    s += clamp ? max(doc_len[d], 0) : doc_len[d];
  }
  chunk_sum[t] = s;
  __syncthreads();
  if (t == 0) {
    int64_t run = 0;
    for (int c = 0; c < 1024; ++c) {
      const int64_t x = chunk_sum[c];
      chunk_sum[c] = run;
      run += x;
    }
    doc_off[0] = 0;
  }
  __syncthreads();
  int64_t run = chunk_sum[t];
  for (int d = lo; d < hi; ++d) {
    run += clamp ? max(doc_len[d], 0) : doc_len[d];
    doc_off[d + 1] = run;
  }
  if (neg && !clamp) atomicAdd(bad, neg);
}

// The table of log_tab built on the device (fill_log_table is its host twin; the two may
// differ in the last bit of an entry).
__global__ __launch_bounds__(256) void log_table_kernel(double2* __restrict__ t) {
  const int i = threadIdx.x;
  if (i >= kLogTableSize) return;
  const double inv = 1.0 / (1.0 + (double)i / 128.0);
  // from the fold on the entry is -ln(inv) - ln 2 = -ln(2 inv); 2 inv is exact, so no cancellation
  double l = i >= kLogTableFold ? -log(2.0 * inv) : -log(inv);
  if (i == 0 || i == kLogTableSize - 1) l = 0.0;
  t[i] = make_double2(inv, l);
}

}  // namespace

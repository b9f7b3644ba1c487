// LDA (Fig. 1 of arXiv 1312.3613): the uncollapsed Gibbs sweep of Sect. 4.2 as
// HIP kernels for gfx950, behind the augur_lda_* C ABI.
//
// Device layout (all row strides are ldk = K rounded up to a multiple of 16, or of 64
// above 256 topics, so every row starts 64- or 256-byte aligned; padding columns hold 0):
//   w, z      int32[N]     doc-major
//   doc_off   int64[D+1]
//   theta     float[D][ldk]     n_dk int32[D][ldk]
//   phi       float[V][ldk]     n_wk int32[V][ldk]
//   perm      int32[N]     token indices sorted by word (built once: w never changes)
//   zb        uint8[N]     copy of z in one byte a token (K <= 256), for the word table's gathers
//   word_off  int32[V+1]   start of each word's run in perm
//   slice_desc int4[slices] a word's run is cut into slices: first, end (in perm), word, mode;
//   item_off  int32[items+1] the slices a wave visits in one go (its "item")
#include "common.hpp"

#include <hipcub/hipcub.hpp>

#include <algorithm>
#include <exception>
#include <mutex>
#include <new>
#include <vector>

using namespace augur;

namespace {

constexpr int kRedBlocks = 2048;       // partial sums of the log-likelihood reductions

// theta and phi are stored as fp32 (the benchmark's state) or, in the fp64 state mode, as fp64;
// a stored probability is never below the type's smallest positive normal number, so that its
// logarithm stays finite.
template <typename T>
__host__ __device__ constexpr double state_floor() {
  return sizeof(T) == sizeof(float) ? (double)FLT_MIN : DBL_MIN;
}
constexpr int kPhiRowsMax = 32;  // most rows of the Gamma matrix handled by one block

// ------------------------------------------------------------------ DPP rows
// A "row" is 16 consecutive lanes; DPP moves data inside rows at VALU speed.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {  // out-of-row sources read 0
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ float dpp_mov_f32(float x) {  // plain move, out-of-row sources read 0
  return __builtin_bit_cast(float,
                            __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i32_keep(int x) {  // out-of-row sources keep x
  return __builtin_amdgcn_update_dpp(x, x, CTRL, 0xF, 0xF, false);
}
constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kRowRor1 = 0x121, kRowRor2 = 0x122, kRowRor4 = 0x124, kRowRor8 = 0x128;
constexpr int kRowBcast15 = 0x15F;  // lane 15 of the row to the whole row

__device__ __forceinline__ int row_allreduce_min(int x) {
  x = min(x, dpp_i32_keep<kRowRor8>(x));
  x = min(x, dpp_i32_keep<kRowRor4>(x));
  x = min(x, dpp_i32_keep<kRowRor2>(x));
  x = min(x, dpp_i32_keep<kRowRor1>(x));
  return x;
}
__device__ __forceinline__ int row_allreduce_max(int x) {
  x = max(x, dpp_i32_keep<kRowRor8>(x));
  x = max(x, dpp_i32_keep<kRowRor4>(x));
  x = max(x, dpp_i32_keep<kRowRor2>(x));
  x = max(x, dpp_i32_keep<kRowRor1>(x));
  return x;
}

// ------------------------------------------------------- document segments
// The sampler gives one wave a whole document.  Documents longer than
// kSegTokens positions are cut into segments of that length (counted from the
// document's first 4-aligned position, so segments are whole Philox strips), one
// wave each, so that a few very long documents do not serialise the launch.
// seg_base[d] = id of document d's first segment; NULL when every document is a
// single segment (then segment id = document id).
constexpr int kSegTokens = 1024;
struct Segment {
  int d;                // document
  int64_t a, b;         // the document's tokens
  int64_t first, end;   // this segment: chunk bases first, first + 256, ... below end
};
__device__ __forceinline__ Segment segment_of(const int64_t* __restrict__ doc_off,
                                              const int32_t* __restrict__ seg_base, int D, int s) {
  Segment g;
  if (seg_base == nullptr) {
    g.d = s;
    g.a = doc_off[s];
    g.b = doc_off[s + 1];
    g.first = g.a & ~(int64_t)3;
    g.end = g.b;
    return g;
  }
  int lo = 0, hi = D;  // largest d with seg_base[d] <= s
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (seg_base[mid] <= s) lo = mid; else hi = mid;
  }
  g.d = lo;
  g.a = doc_off[lo];
  g.b = doc_off[lo + 1];
  g.first = (g.a & ~(int64_t)3) + (int64_t)(s - seg_base[lo]) * kSegTokens;
  g.end = g.b < g.first + kSegTokens ? g.b : g.first + kSegTokens;
  return g;
}
// True when document d is cut into more than one segment: then no single wave
// sees all of its tokens, and its row of n_dk is zeroed first and every segment
// adds its own histogram to it (integer adds: the result does not depend on the
// order).
__device__ __forceinline__ bool is_split(const int32_t* __restrict__ seg_base, int d) {
  return seg_base != nullptr && seg_base[d + 1] - seg_base[d] > 1;
}
__global__ __launch_bounds__(256) void zero_split_rows_kernel(const int32_t* __restrict__ seg_base,
                                                               int32_t* __restrict__ n_dk, int D,
                                                               int ldk) {
  const int lane = threadIdx.x & 63;
  const int d = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (d >= D || !is_split(seg_base, d)) return;
  for (int k = lane; k < ldk; k += 64) n_dk[(size_t)d * ldk + k] = 0;
}
// Stores (whole document) or adds (segment of a split document) a wave's LDS
// histogram into the document's row.
__device__ __forceinline__ void flush_doc_histogram(const int32_t* hist, int32_t* __restrict__ row,
                                                    int ldk, bool split, int lane) {
  if (!split) {
    for (int k = lane; k < ldk; k += 64) row[k] = hist[k];
  } else {
    for (int k = lane; k < ldk; k += 64)
      if (hist[k] != 0) atomicAdd(&row[k], hist[k]);
  }
}
__global__ __launch_bounds__(256) void segment_counts_kernel(const int64_t* __restrict__ doc_off,
                                                              int D, int32_t* __restrict__ ns) {
  const int d = blockIdx.x * blockDim.x + threadIdx.x;
  if (d > D) return;
  if (d == D) { ns[d] = 0; return; }
  const int64_t a = doc_off[d], b = doc_off[d + 1];
  const int64_t span = b - (a & ~(int64_t)3);
  ns[d] = (int32_t)(span <= kSegTokens ? 1 : (span + kSegTokens - 1) / kSegTokens);
}

// ------------------------------------------------------------------- init z
// z_i = floor(K r / 2^32), r = word (i & 3) of block i >> 2 of the init stream.
__global__ __launch_bounds__(256) void lda_init_z_kernel(int32_t* __restrict__ z, int64_t N, int K,
                                                          uint64_t seed) {
  const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one Philox block each
  if (b * 4 >= N) return;
  const U4 r = random_block(seed, (uint64_t)b, 0, kStreamInitZ, 0);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int64_t i = b * 4 + e;
    if (i < N) z[i] = (int32_t)(((uint64_t)word_of(r, e) * (uint64_t)K) >> 32);
  }
}

// ----------------------------------------------------------------- sample z
// Gibbs step for the assignments (Sect. 4.2): token i of document d with word v
// draws z_i = first k with C_k > u_i * S, C_k the running sum of
// theta[d][k] * phi[v][k] and S = C_{K-1}; fp32 throughout.
//
// One wave owns one document.  The wave is four 16-lane rows; each row draws one
// token per iteration.  A row covers the K topics in NS stripes of 64: lane j
// holds topics 64 m + 4 j + {0,1,2,3} of stripe m (its "chunk" of the stripe), so a
// row reads 256 contiguous bytes of the phi row per load.  theta_d is staged in LDS
// once per document (zero beyond the last topic).
//
// Pass 1 keeps one number per chunk, the sum of its four products.  The row scans
// the chunk sums of each stripe with DPP and carries the stripe totals, which gives
// every chunk the running sum before it.  Each lane then finds the first of its
// chunks that the threshold falls into (a chunk of zero mass never qualifies).
// Pass 2 takes that one chunk again (16 bytes of the phi row: from the registers that
// still hold the row up to ten stripes, by a second load, a cache hit, beyond; and of
// theta from LDS), repeats the same three multiply-adds, which give the same bits, and locates the
// topic inside it; the row takes the minimum candidate index.  Keeping the products of
// all stripes instead (and theta in registers) needs 256 registers a lane, one wave
// per SIMD; this form needs half and the loads of several waves overlap.
//
// Random numbers: lane L computes the Philox block of tokens
// base + 4 L .. base + 4 L + 3 (base a multiple of 4), parks the four words in
// the wave's LDS strip, and each row then picks the word of its token: one
// Philox evaluation per wave serves 256 tokens.
//
// Registers: up to 14 stripes the kernel is held to 128 registers (four waves per SIMD); with
// 15 or 16 stripes that limit makes the compiler serialise the row loads, and three waves
// with all loads of a row in flight are faster (K = 1000 on 10M tokens: 2.28 against 2.86 ms).
template <int NS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NS >= 15 ? 3 : 4, NS >= 15 ? 3 : 8)))
void lda_sample_z_kernel(
    const int32_t* __restrict__ w, const int64_t* __restrict__ doc_off,
    const int32_t* __restrict__ seg_base, int n_segs, const float* __restrict__ theta,
    const float* __restrict__ phi, int32_t* __restrict__ z, int D, int K, int ldk, uint64_t seed,
    SweepRef sweep_ref, unsigned long long* __restrict__ n_degenerate) {
  __shared__ uint32_t rnd[4][256];
  const uint32_t sweep = sweep_ref.get();
  __shared__ __align__(16) float theta_s[4][NS * 64];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int seg = blockIdx.x * 4 + wave;
  if (seg >= n_segs) return;
  const Segment sg = segment_of(doc_off, seg_base, D, seg);
  const int d = sg.d;
  const int row = lane >> 4, j = lane & 15;

  // theta_d into the wave's LDS strip; chunks past the last topic hold 0.  Every lane's
  // byte offset inside a phi row is fixed: full stripes sit 256 B apart, and the last
  // stripe's lanes beyond the row are pointed at the row's last chunk (their theta is 0),
  // so all loads are unconditional and stay inside the row.
  float* th = theta_s[wave];
#pragma unroll
  for (int c = 4 * lane; c < NS * 64; c += 256) {
    *reinterpret_cast<float4*>(th + c) =
        c < ldk ? *reinterpret_cast<const float4*>(theta + (size_t)d * ldk + c)
                : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  wave_lds_fence();
  const float* th_lane = th + 4 * j;
  // With five stripes there are registers to spare for a second set of row loads: the next
  // group's rows are requested while pass 2 of this one waits for its chunk (K = 300, 3.2M
  // tokens: 0.305 against 0.338 ms; with six to eight stripes the same costs more than it hides).
  constexpr bool kPipelined = NS <= 5;
  const uint32_t lane_off = 16u * (uint32_t)j;
  const uint32_t last_off = 4u * (uint32_t)min(64 * (NS - 1) + 4 * j, ldk - 4);
  const char* phi_bytes = reinterpret_cast<const char*>(phi);
  const uint32_t row_bytes = 4u * (uint32_t)ldk;

  const int64_t a = sg.a, b = sg.end;
  for (int64_t base = sg.first; base < b; base += 256) {
    {
      const U4 r = random_block(seed, (uint64_t)(base >> 2) + (uint64_t)lane, sweep, kStreamZ, 0);
      wave_lds_fence();  // earlier reads of the strip are done
      *reinterpret_cast<uint4*>(&rnd[wave][4 * lane]) = make_uint4(r.x, r.y, r.z, r.w);
      wave_lds_fence();
    }
    const int64_t lo = a > base ? a : base;
    const int64_t hi = b < base + 256 ? b : base + 256;
    // The token of this row in the group of four starting at i0 (a row past the end of the
    // chunk reads word 0's row, in bounds, and stores nothing), and its phi row's loads.
    struct Token {
      int64_t i;
      bool valid;
      uint32_t r;
      const char *rowp, *lastp;
    };
    auto fetch = [&](int64_t i0, Token& T, float4 (&q)[NS]) {
      T.i = i0 + row;
      T.valid = T.i < hi;
      const uint32_t v = T.valid ? (uint32_t)w[T.i] : 0u;
      T.r = rnd[wave][T.valid ? (int)(T.i - base) : 0];
      const uint32_t row_off = v * row_bytes;  // < 2^32: checked when the handle is created
      T.rowp = phi_bytes + (size_t)(row_off + lane_off);  // constant offsets fold into the loads
      T.lastp = phi_bytes + (size_t)(row_off + last_off);
#pragma unroll
      for (int m = 0; m < NS - 1; ++m) q[m] = *reinterpret_cast<const float4*>(T.rowp + 256 * m);
      q[NS - 1] = *reinterpret_cast<const float4*>(T.lastp);
    };
    Token T, Tn;
    float4 q[NS], qn[kPipelined ? NS : 1];
    if (kPipelined) fetch(lo, T, q);
    for (int64_t i0 = lo; i0 < hi; i0 += 4) {
      if (!kPipelined) fetch(i0, T, q);
      const int64_t i = T.i;
      const bool valid = T.valid;
      const uint32_t r = T.r;
      const char* rowp = T.rowp;
      const char* lastp = T.lastp;

      // ls[m] = sum of the lane's chunk of stripe m; inc[m] its inclusive row scan; cbase[m] =
      // sum of everything before the chunk.  The NS row scans are independent until the
      // carries, so they are issued side by side.
      float ls[NS], inc[NS], cbase[NS];
#pragma unroll
      for (int m = 0; m < NS; ++m) {
        const float4 t4 = *reinterpret_cast<const float4*>(th_lane + 64 * m);
        float l = t4.x * q[m].x;
        l = fmaf(t4.y, q[m].y, l);
        l = fmaf(t4.z, q[m].z, l);
        l = fmaf(t4.w, q[m].w, l);
        ls[m] = l;
        inc[m] = l;
      }
#pragma unroll
      for (int m = 0; m < NS; ++m) inc[m] += dpp_f32<kRowShr1>(inc[m]);
#pragma unroll
      for (int m = 0; m < NS; ++m) inc[m] += dpp_f32<kRowShr2>(inc[m]);
#pragma unroll
      for (int m = 0; m < NS; ++m) inc[m] += dpp_f32<kRowShr4>(inc[m]);
#pragma unroll
      for (int m = 0; m < NS; ++m) inc[m] += dpp_f32<kRowShr8>(inc[m]);
      float carry = 0.f;
#pragma unroll
      for (int m = 0; m < NS; ++m) {
        cbase[m] = carry + dpp_mov_f32<kRowShr1>(inc[m]);
        carry += dpp_mov_f32<kRowBcast15>(inc[m]);
      }
      const float S = carry;
      const float t = u24(r) * S;

      // the first of this lane's chunks whose running sum exceeds t and whose mass is positive
      int cm = -1;
      float ctt = 0.f;
#pragma unroll
      for (int m = NS - 1; m >= 0; --m) {
        const float tt = fmaxf(t - cbase[m], 0.f);
        const bool hit = ls[m] > tt;
        cm = hit ? m : cm;
        ctt = hit ? tt : ctt;
      }
      if constexpr (kPipelined) fetch(i0 + 4, Tn, qn);
      // pass 2 on that chunk (stripe 0 for a lane without one; its result is not used)
      int cand = 0x7FFFFFFF;
      {
        const int mm = cm < 0 ? 0 : cm;
        // Up to ten stripes the chunk is taken from the registers that still hold the row
        // (no second load, no wait for it: K = 500 on 3.2M tokens 0.39 against 0.43 ms); with
        // more stripes keeping the row alive spills, and loading the chunk again is faster.
        float4 q2;
        if constexpr (NS <= 10) {
          q2 = q[0];
#pragma unroll
          for (int m = 1; m < NS; ++m) {
            const bool sel = mm == m;
            q2.x = sel ? q[m].x : q2.x;
            q2.y = sel ? q[m].y : q2.y;
            q2.z = sel ? q[m].z : q2.z;
            q2.w = sel ? q[m].w : q2.w;
          }
        } else {
          q2 = *reinterpret_cast<const float4*>(mm == NS - 1 ? lastp : rowp + 256 * mm);
        }
        const float4 t4 = *reinterpret_cast<const float4*>(th_lane + 64 * mm);
        const float l0 = t4.x * q2.x;
        const float l1 = fmaf(t4.y, q2.y, l0);
        const float l2 = fmaf(t4.z, q2.z, l1);
        const int e = (l0 <= ctt) + (l1 <= ctt) + (l2 <= ctt);
        cand = cm >= 0 ? 64 * cm + 4 * j + e : cand;
      }
      int k = row_allreduce_min(cand);

      const bool ok = S > 0.f && S <= FLT_MAX;  // false for 0, inf and NaN
      if (__builtin_expect(__any(valid && (!ok || k == 0x7FFFFFFF)), 0)) {
        if (!ok) {
          // zero or non-finite mass: z = floor(u K)
          k = u24_times(r, K);
          if (valid && j == 0) atomicAdd(n_degenerate, 1ULL);
        } else if (k == 0x7FFFFFFF) {
          // rounding pushed t to S: the last topic of positive mass
          int last = -1;
          for (int m = 0; m < NS; ++m) {
            const float4 q2 = *reinterpret_cast<const float4*>(m == NS - 1 ? lastp : rowp + 256 * m);
            const float4 t4 = *reinterpret_cast<const float4*>(th_lane + 64 * m);
            const float l0 = t4.x * q2.x;
            const float l1 = fmaf(t4.y, q2.y, l0);
            const float l2 = fmaf(t4.z, q2.z, l1);
            const float l3 = fmaf(t4.w, q2.w, l2);
            const int kk = 64 * m + 4 * j;
            if (l0 > 0.f) last = kk;
            if (l1 > l0) last = kk + 1;
            if (l2 > l1) last = kk + 2;
            if (l3 > l2) last = kk + 3;
          }
          k = row_allreduce_max(last);
        }
      }
      // garbage parameters (negative or NaN entries) must not yield an index outside the tables
      if (valid && j == 0) z[i] = min(max(k, 0), K - 1);
      if constexpr (kPipelined) {
        T = Tn;
#pragma unroll
        for (int m = 0; m < NS; ++m) q[m] = qn[m];
      }
    }
  }
}

// ------------------------------------------------- sample z, up to 256 topics
// Same draw as lda_sample_z_kernel with a finer grain: a QUAD (4 lanes) per
// token, 16 tokens per wave and iteration.  The topics are cut into stripes of
// 16; quad lane q holds topics 16 c + 4 q + {0..3} of stripe c, so a quad reads
// 64 contiguous bytes of the phi row per load.
//
// Pass 1 is one chain of multiply-adds per lane over all its topics; the value of the
// chain after stripe c, a[c], is the lane's share of the running sum C at the end of
// that stripe, and the sum of a[c] over the quad (two DPP adds; all four lanes get the
// same bits) is C itself.  Only the last of these sums is formed outright: S, and
// t = u S.  The crossing stripe c* = #{c : C(c) <= t} is then found by bisection over
// c, which needs the quad sum of one a[.] per level (four levels for 16 stripes); the
// a[.] wanted at a level is picked by the comparison masks of the levels before it.
// The sums are non-decreasing in c (every product is >= 0 and rounding is monotone),
// so bisection finds the same c* as a scan would.
//
// Pass 2 needs the 64 bytes of stripe c* of the row again, and theta's from LDS: it
// rebuilds that stripe's running sums and finds the topic.  Those bytes are asked for
// again (a cache hit or an L2 hit) as soon as c* is known, but not waited for: pass 2 of
// an iteration runs in the next iteration, after the loads of that one have been
// issued and before they are waited for.  So the row's registers die with pass 1, and no
// wave waits for a second load.  (Keeping the row alive and selecting the chunk from the
// registers cost 48 conditional moves a lane and iteration and the registers of a wave
// per SIMD; loading it again and waiting on the spot cost one more wait.)
//
// The wave's LDS strip holds, for the 256 tokens of the current chunk, the
// Philox word and the word id of each token, and theta_d padded with zeros to a
// whole number of stripes.
constexpr int kQpSwap1 = 0xB1;   // quad_perm [1,0,3,2]
constexpr int kQpSwap2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int kQpDown1 = 0x90;   // quad_perm [0,0,1,2]: lane q reads lane q - 1 (lane 0 itself)
constexpr int kQpDown2 = 0x44;   // quad_perm [0,1,0,1]: lane q reads lane q - 2 (lanes 0, 1 themselves)
constexpr int kNoTopic = 0x7FFFFFFF;

__device__ __forceinline__ float quad_sum(float s) {
  s += dpp_f32<kQpSwap1>(s);
  s += dpp_f32<kQpSwap2>(s);
  return s;
}

// Bisection over the M = NS16 - 1 stripe ends before the last one (if none of them
// exceeds t the crossing stripe is the last).  A level has a step s (a power of two);
// with p the number of stripes already known to lie at or below t, it tests stripe
// p + s - 1.  p is different in every quad, so the value is picked from the
// compile-time candidates {s - 1, 3 s - 1, 5 s - 1, ...} by the masks of the levels above
// (m[j] belongs to step 2^j): a tree of conditional moves, one fewer than candidates.
// Candidates past the end count as +infinity (never at or below t).
template <int NS16, int STEP, int HS, int P>
__device__ __forceinline__ float pick_stripe_end(const float (&a)[NS16], const bool (&m)[5]) {
  if constexpr (HS == STEP) {
    constexpr int idx = P + STEP - 1;
    if constexpr (idx < NS16 - 1) return a[idx];
    else return INFINITY;
  } else {
    constexpr int idx_lo = P + STEP - 1;  // the smallest candidate below this node
    if constexpr (idx_lo >= NS16 - 1) {
      return INFINITY;  // every candidate of this subtree is past the end
    } else {
      constexpr int bit = HS == 16 ? 4 : HS == 8 ? 3 : HS == 4 ? 2 : 1;  // log2(HS); HS >= 2 here
      const float lo = pick_stripe_end<NS16, STEP, HS / 2, P>(a, m);
      const float hi = pick_stripe_end<NS16, STEP, HS / 2, P + HS>(a, m);
      return m[bit] ? hi : lo;
    }
  }
}
template <int NS16, int STEP, int TOP>
__device__ __forceinline__ void bisect_level(const float (&a)[NS16], float t, bool (&m)[5], int& pos,
                                             float& cprev) {
  constexpr int bit = STEP == 16 ? 4 : STEP == 8 ? 3 : STEP == 4 ? 2 : STEP == 2 ? 1 : 0;
  float x;
  if constexpr (STEP == TOP) x = pick_stripe_end<NS16, STEP, STEP, 0>(a, m);
  else x = pick_stripe_end<NS16, STEP, TOP, 0>(a, m);
  const float qs = quad_sum(x);
  const bool below = qs <= t;
  m[bit] = below;
  pos += below ? STEP : 0;
  cprev = below ? qs : cprev;
  if constexpr (STEP > 1) bisect_level<NS16, STEP / 2, TOP>(a, t, m, pos, cprev);
}

//
// With kCountDocs the wave also builds its document's row of n_dk in LDS while it
// draws and stores it at the end (the document half of the counting phase, for
// free: the wave already owns the document; a segment of a split document adds
// to the row, which the host zeroes before the launch).
//
// The kernel comes in two forms that draw the same bits.  The plain form gives every wave one
// segment and takes every phi row from memory.  The kernel is bound by the texture addresser
// (96 % busy at K = 200: about 21 cycles for every 64-lane load of 16 bytes a lane, whatever
// the cache level that answers), so the second form takes the rows of the most frequent words
// from LDS instead, which has a path of its own: workgroups of 16 waves stay resident, one per
// CU, copy the rows of the H most frequent words (H as many as fit beside the waves' own
// strips: about 100 at K = 200) into LDS once per launch, and walk the tokens of every
// 256-token chunk in an order fixed at create time: tokens of cached words first.  An
// iteration whose 16 tokens are all cached reads its rows from LDS and issues no load.
//
// Waves per SIMD (plain form): the kernel waits on its row loads, so a wave more per SIMD pays.
template <int NS16>
constexpr int quad_waves_per_simd() { return NS16 > 10 ? 4 : NS16 > 6 ? 5 : NS16 > 3 ? 6 : 8; }

// What pass 2 of a token needs, carried from the iteration that ran its pass 1.
struct QuadPending {
  float4 p2;          // the lane's chunk of the crossing stripe (load in flight)
  float t, cprev;     // threshold; running sum before the crossing stripe
  int cs;             // crossing stripe
  uint32_t r, row_off;
  int pos;            // position of the token in its chunk (0..255), or -1 for a quad without a token
  bool ok, in_row;    // S positive and finite; t < S
  __device__ __forceinline__ void idle() {  // a quad without a token, which pass 2 runs through idly
    p2 = make_float4(0.f, 0.f, 0.f, 0.f);
    t = 0.f;
    cprev = 0.f;
    cs = 0;
    r = 0u;
    row_off = 0u;
    pos = -1;
    ok = true;
    in_row = true;
  }
};
// The lane-constant part of a quad's view of the tables.
struct QuadLane {
  int q;                 // lane within the quad
  uint32_t lane_off;     // 16 q: the lane's byte offset inside a 64-byte piece of a row
  uint32_t row_bytes;    // 4 ldk
  float from1, from2;    // 1 for lanes that have a neighbour one / two lanes down in the quad, else 0
  const char* phi_bytes;
  const float* theta_q;  // the wave's copy of theta_d in LDS, + 4 q
};

// Pass 1 and the bisection: from the row's chunks to S, t = u S, the crossing stripe and the
// running sum before it.  theta_p1 is theta_q behind an offset the compiler cannot see through
// (theta_d does not change inside the token loop, so it would otherwise be read once and
// held in registers, at the price of a wave per SIMD).
template <int NS16>
__device__ __forceinline__ void quad_pass1(const float4 (&ph)[NS16], const float* theta_p1, uint32_t r,
                                           float& S, float& t, int& cs, float& cprev) {
  float ac[NS16];
  float acc = 0.f;
#pragma unroll
  for (int c = 0; c < NS16; ++c) {
    const float4 tc = *reinterpret_cast<const float4*>(theta_p1 + 16 * c);
    acc = c == 0 ? tc.x * ph[c].x : fmaf(tc.x, ph[c].x, acc);
    acc = fmaf(tc.y, ph[c].y, acc);
    acc = fmaf(tc.z, ph[c].z, acc);
    acc = fmaf(tc.w, ph[c].w, acc);
    ac[c] = acc;
  }
  S = quad_sum(ac[NS16 - 1]);
  t = u24(r) * S;
  cs = 0;
  cprev = 0.f;
  if constexpr (NS16 > 1) {
    constexpr int M = NS16 - 1;
    constexpr int TOP = M >= 8 ? 8 : M >= 4 ? 4 : M >= 2 ? 2 : 1;
    bool m[5] = {false, false, false, false, false};
    bisect_level<NS16, TOP, TOP>(ac, t, m, cs, cprev);
  }
}

// Pass 2: the topic inside the crossing stripe; the drawn topic goes to the chunk's stage
// (and the document histogram).
template <int NS16, bool kCountDocs>
__device__ __forceinline__ void quad_finish(const QuadPending& P, const QuadLane& L, int K,
                                            unsigned long long* __restrict__ n_degenerate,
                                            uint8_t* zstage, int32_t* hist) {
  const bool valid = P.pos >= 0;
  const int cs = P.cs;
  const int q = L.q;
  const float4 t2 = *reinterpret_cast<const float4*>(L.theta_q + 16 * cs);
  const float l0 = t2.x * P.p2.x;
  const float l1 = fmaf(t2.y, P.p2.y, l0);
  const float l2 = fmaf(t2.z, P.p2.z, l1);
  const float l3 = fmaf(t2.w, P.p2.w, l2);
  // sum of the chunks of the quad's lower lanes: an inclusive scan over the quad in two
  // steps (a lane takes the value one, then two, lanes down; lanes without such a neighbour
  // multiply what they get by 0), then moved up by one lane
  float incl = fmaf(dpp_mov_f32<kQpDown1>(l3), L.from1, l3);
  incl = fmaf(dpp_mov_f32<kQpDown2>(incl), L.from2, incl);
  const float excl = dpp_mov_f32<kQpDown1>(incl) * L.from1;
  const float tt = fmaxf(P.t - (P.cprev + excl), 0.f);
  const int e = (l0 <= tt) + (l1 <= tt) + (l2 <= tt);
  int cand = l3 > tt ? 4 * q + e : kNoTopic;
  cand = min(cand, dpp_i32_keep<kQpSwap1>(cand));
  cand = min(cand, dpp_i32_keep<kQpSwap2>(cand));
  int k = 16 * cs + cand;

  const bool found = P.in_row && cand != kNoTopic;
  if (__builtin_expect(__any(valid && !(P.ok && found)), 0)) {
    if (!P.ok) {
      // zero or non-finite mass: z = floor(u K)
      k = u24_times(P.r, K);
      if (valid && q == 0) atomicAdd(n_degenerate, 1ULL);
    } else if (!found) {
      // rounding put t at or past the running sum that should exceed it: the
      // last topic of positive mass in the crossing stripe (or overall)
      const int limit = P.in_row ? 16 * (cs + 1) : 16 * NS16;
      int last = -1;
#pragma unroll 1
      for (int c = 0; c < NS16; ++c) {  // rare: kept small, nothing precomputed outside
        const uint32_t o = min(64u * (uint32_t)c + L.lane_off, L.row_bytes - 16u);
        const float4 pp = *reinterpret_cast<const float4*>(L.phi_bytes + (P.row_off + o));
        const float4 tp = *reinterpret_cast<const float4*>(L.theta_q + 16 * c);
        const int kk = 16 * c + 4 * q;
        if (kk < limit) {
          if (tp.x * pp.x > 0.f) last = kk;
          if (tp.y * pp.y > 0.f) last = kk + 1;
          if (tp.z * pp.z > 0.f) last = kk + 2;
          if (tp.w * pp.w > 0.f) last = kk + 3;
        }
      }
      last = max(last, dpp_i32_keep<kQpSwap1>(last));
      last = max(last, dpp_i32_keep<kQpSwap2>(last));
      k = last;
    }
  }
  // garbage parameters (negative or NaN entries) must not yield an index outside the tables
  k = min(max(k, 0), K - 1);
  if (valid && q == 0) {
    zstage[P.pos] = (uint8_t)k;  // K <= 256 here; stored to z and zb a chunk at a time
    if (kCountDocs) atomicAdd(&hist[k], 1);
  }
}

// Stores the staged topics of the chunk at rbase (tokens lo..hi-1 of the segment): lane L takes
// tokens rbase + 4 L .. + 3, so z leaves as one 16-byte and zb as one 4-byte store per lane
// instead of a 4-byte and a 1-byte store per token (a store instruction of 16 lanes costs the
// address path as much as one of 64).  Tokens outside lo..hi-1 belong to other waves: the
// lanes at the two ends store element by element.
__device__ __forceinline__ void quad_flush_chunk(const uint8_t* zstage, int32_t* z_seg, uint8_t* zb_seg,
                                                 int rbase, int lo, int hi, int lane) {
  wave_lds_fence();
  const int r0 = rbase + 4 * lane;
  const uint32_t four = *reinterpret_cast<const uint32_t*>(zstage + 4 * lane);
  const int k0 = (int)(four & 255u), k1 = (int)((four >> 8) & 255u), k2 = (int)((four >> 16) & 255u),
            k3 = (int)(four >> 24);
  if (r0 >= lo && r0 + 4 <= hi) {
    *reinterpret_cast<int4*>(z_seg + r0) = make_int4(k0, k1, k2, k3);
    *reinterpret_cast<uint32_t*>(zb_seg + r0) = four;
  } else {
    if (r0 + 0 >= lo && r0 + 0 < hi) { z_seg[r0 + 0] = k0; zb_seg[r0 + 0] = (uint8_t)k0; }
    if (r0 + 1 >= lo && r0 + 1 < hi) { z_seg[r0 + 1] = k1; zb_seg[r0 + 1] = (uint8_t)k1; }
    if (r0 + 2 >= lo && r0 + 2 < hi) { z_seg[r0 + 2] = k2; zb_seg[r0 + 2] = (uint8_t)k2; }
    if (r0 + 3 >= lo && r0 + 3 < hi) { z_seg[r0 + 3] = k3; zb_seg[r0 + 3] = (uint8_t)k3; }
  }
  wave_lds_fence();  // before the next chunk's topics overwrite the stage
}

// theta_d into the wave's LDS strip, zero past the last topic.  Pass 1 reads it from there
// (all quads read the same 16 bytes per lane: a broadcast), which keeps the registers for
// the row loads in flight.
template <int NS16>
__device__ __forceinline__ void quad_stage_theta(const float* __restrict__ theta, int d, int ldk,
                                                 float* theta_s, int tq, int q) {
#pragma unroll
  for (int c = 0; c < NS16; ++c) {
    const int col = 16 * c + 4 * q;
    const float4 v = col < ldk ? *reinterpret_cast<const float4*>(theta + (size_t)d * ldk + col)
                               : make_float4(0.f, 0.f, 0.f, 0.f);
    if (tq == 0) *reinterpret_cast<float4*>(theta_s + col) = v;
  }
}

template <int NS16, bool kCountDocs>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(quad_waves_per_simd<NS16>())))
void lda_sample_z_quad_kernel(
    const int32_t* __restrict__ w, const int64_t* __restrict__ doc_off,
    const int32_t* __restrict__ seg_base, int n_segs, const float* __restrict__ theta,
    const float* __restrict__ phi, int32_t* __restrict__ z, int32_t* __restrict__ n_dk, int D, int K,
    int ldk, uint64_t seed, SweepRef sweep_ref, unsigned long long* __restrict__ n_degenerate,
    uint8_t* __restrict__ zb) {
  __shared__ uint2 strip_all[4][256];            // {Philox word, word id} per token of the chunk
  const uint32_t sweep = sweep_ref.get();
  __shared__ __align__(16) float theta_all[4][16 * NS16];
  __shared__ int32_t hist_all[kCountDocs ? 4 : 1][kCountDocs ? 16 * NS16 : 1];
  __shared__ __align__(4) uint8_t zstage_all[4][256];  // the topics drawn for the current chunk
  const int lane = threadIdx.x & 63;
  // the wave's number is the same in all its lanes: saying so keeps everything that follows
  // from it (the segment, its offsets, the loop bounds) in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int seg = blockIdx.x * 4 + wave;
  if (seg >= n_segs) return;
  const Segment sg = segment_of(doc_off, seg_base, D, seg);
  const int d = sg.d;
  const int tq = lane >> 2, q = lane & 3;  // token slot of this quad, lane within the quad
  uint2* strip = strip_all[wave];
  float* theta_s = theta_all[wave];
  int32_t* hist = hist_all[kCountDocs ? wave : 0];
  uint8_t* zstage = zstage_all[wave];
  if (kCountDocs)
    for (int k = lane; k < 16 * NS16; k += 64) hist[k] = 0;
  quad_stage_theta<NS16>(theta, d, ldk, theta_s, tq, q);
  QuadLane L;
  L.q = q;
  L.lane_off = 16u * (uint32_t)q;
  L.row_bytes = 4u * (uint32_t)ldk;
  L.from1 = q >= 1 ? 1.f : 0.f;
  L.from2 = q >= 2 ? 1.f : 0.f;
  L.phi_bytes = reinterpret_cast<const char*>(phi);
  L.theta_q = theta_s + 4 * q;
  const uint32_t last_off = min(64u * (NS16 - 1) + L.lane_off, L.row_bytes - 16u);
  // Tokens are addressed relative to the segment's first chunk base (an int: a segment has at
  // most kSegTokens + 3 positions).
  const int32_t* w_seg = w + sg.first;
  int32_t* z_seg = z + sg.first;
  uint8_t* zb_seg = zb + sg.first;
  const int rel_a = (int)(sg.a - sg.first);  // 0..3: the first token of the document
  const int rel_b = (int)(sg.end - sg.first);

  QuadPending P;
  for (int rbase = 0; rbase < rel_b; rbase += 256) {
    P.idle();
    {
      // tokens rbase + 4 lane .. + 3 of the segment: one Philox block and four word ids (w is
      // padded by 256 entries, so the vector load never leaves the allocation)
      const U4 r = random_block(seed, (uint64_t)((sg.first + rbase) >> 2) + (uint64_t)lane, sweep,
                                kStreamZ, 0);
      const int4 wv = *reinterpret_cast<const int4*>(w_seg + rbase + 4 * lane);
      wave_lds_fence();  // earlier reads of the strip are done
      uint4* dst = reinterpret_cast<uint4*>(strip + 4 * lane);
      dst[0] = make_uint4(r.x, (uint32_t)wv.x, r.y, (uint32_t)wv.y);
      dst[1] = make_uint4(r.z, (uint32_t)wv.z, r.w, (uint32_t)wv.w);
      wave_lds_fence();
    }
    const int lo = max(rel_a, rbase);
    const int hi = min(rel_b, rbase + 256);

    for (int i0 = lo; i0 < hi; i0 += 16) {
      // this iteration's token of the quad and the loads of its row
      const int i = i0 + tq;
      const bool valid = i < hi;
      const uint2 rw = strip[(valid ? i : lo) - rbase];
      const uint32_t row_off = __umul24(rw.y, L.row_bytes);  // both below 2^24; product below 2^32
      const char* rowp = L.phi_bytes + (size_t)(row_off + L.lane_off);  // constant offsets fold into the loads
      float4 ph[NS16];
#pragma unroll
      for (int c = 0; c < NS16 - 1; ++c) ph[c] = *reinterpret_cast<const float4*>(rowp + 64 * c);
      ph[NS16 - 1] = *reinterpret_cast<const float4*>(L.phi_bytes + (row_off + last_off));

      // pass 2 of the previous iteration, while those loads are on their way.  The empty asm
      // statement keeps the compiler from starting it (and waiting for its chunk) before the
      // loads above have been issued: everything in pass 2 follows from the stripe number.
      asm volatile("" : "+v"(P.cs)::"memory");
      quad_finish<NS16, kCountDocs>(P, L, K, n_degenerate, zstage, hist);

      int theta_off = 4 * q;
      asm volatile("" : "+v"(theta_off));
      float S, t, cprev;
      int cs;
      quad_pass1<NS16>(ph, theta_s + theta_off, rw.x, S, t, cs, cprev);
      // the chunk of stripe cs again, for pass 2 in the next iteration
      P.p2 = *reinterpret_cast<const float4*>(
          L.phi_bytes + (row_off + min(64u * (uint32_t)cs + L.lane_off, L.row_bytes - 16u)));
      P.t = t;
      P.cprev = cprev;
      P.cs = cs;
      P.r = rw.x;
      P.row_off = row_off;
      P.pos = valid ? i - rbase : -1;
      P.ok = S > 0.f && S <= FLT_MAX;  // false for 0, inf and NaN
      P.in_row = S > t;
    }
    quad_finish<NS16, kCountDocs>(P, L, K, n_degenerate, zstage, hist);  // the chunk's last iteration
    quad_flush_chunk(zstage, z_seg, zb_seg, rbase, lo, hi, lane);
  }
  if (kCountDocs) {
    wave_lds_fence();
    flush_doc_histogram(hist, n_dk + (size_t)d * ldk, ldk, is_split(seg_base, d), lane);
  }
}

// ---- the resident form, with the rows of the most frequent words in LDS ----
// wz / ord: for every 256-token chunk of every segment, its tokens in processing order (cached
// words first, each group in position order): wz = word id | (cache slot + 1) << 24 (0: not
// cached), ord = position in the chunk; both indexed from the chunk's first token.  Built once
// (lda_build_order_kernel): words never change.
constexpr int kHotWaves = 16;              // waves of a resident workgroup
constexpr int kHotMinStripes = 5;          // shortest rows for which the library picks this form itself
// Cached rows lie 64 NS16 (+ pad) bytes apart.  A quad reads 64 contiguous bytes, half of the
// LDS banks; two quads served together do not collide when their pieces start half the banks
// apart, which random rows do half of the time if the row pitch is an odd multiple of 64 bytes,
// and never if it is an even one.
__host__ __device__ constexpr int hot_row_pad_bytes(int ns16) { return ns16 % 2 == 0 ? 64 : 0; }
__host__ __device__ constexpr int hot_wave_bytes(int ns16, bool count_docs) {
  // Philox words by position, wz by order, ord by order, theta_d, [document histogram], stage
  return 1024 + 1024 + 256 + 64 * ns16 + (count_docs ? 64 * ns16 : 0) + 256;
}
template <int NS16, bool kCountDocs>
__global__ __launch_bounds__(64 * kHotWaves) void lda_sample_z_hot_kernel(
    const int32_t* __restrict__ wz, const uint8_t* __restrict__ ord, const int64_t* __restrict__ doc_off,
    const int32_t* __restrict__ seg_base, int n_segs, const float* __restrict__ theta,
    const float* __restrict__ phi, int32_t* __restrict__ z, int32_t* __restrict__ n_dk, int D, int K,
    int ldk, uint64_t seed, SweepRef sweep_ref, unsigned long long* __restrict__ n_degenerate,
    uint8_t* __restrict__ zb, const int32_t* __restrict__ hot_words, int n_hot) {
  extern __shared__ __align__(16) unsigned char lds[];
  const uint32_t sweep = sweep_ref.get();
  constexpr int kRowLds = 64 * NS16 + hot_row_pad_bytes(NS16);  // bytes between cached rows
  constexpr int kWaveBytes = hot_wave_bytes(NS16, kCountDocs);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t row_bytes = 4u * (uint32_t)ldk;  // 64 NS16: rows of tables with up to 256 topics are whole stripes
  // the cache: row s = phi row of hot_words[s], 16 bytes a thread and trip
  {
    const int pieces = 4 * NS16;  // 16-byte pieces of a row
    for (int e = threadIdx.x; e < n_hot * pieces; e += blockDim.x) {
      const int s = e / pieces, pc = e - s * pieces;
      const float4 v = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(phi) +
                                                       ((size_t)(uint32_t)hot_words[s] * row_bytes + 16u * pc));
      *reinterpret_cast<float4*>(lds + (size_t)s * kRowLds + 16 * pc) = v;
    }
  }
  __syncthreads();  // the only barrier: every wave passes it before it looks for work
  unsigned char* mine = lds + (size_t)n_hot * kRowLds + (size_t)wave * kWaveBytes;
  uint32_t* strip_r = reinterpret_cast<uint32_t*>(mine);           // Philox word of position p
  uint32_t* strip_w = reinterpret_cast<uint32_t*>(mine + 1024);    // wz of the j-th token in order
  uint8_t* strip_o = mine + 2048;                                  // its position
  float* theta_s = reinterpret_cast<float*>(mine + 2304);
  int32_t* hist = reinterpret_cast<int32_t*>(mine + 2304 + 64 * NS16);
  uint8_t* zstage = mine + 2304 + 64 * NS16 + (kCountDocs ? 64 * NS16 : 0);
  const int tq = lane >> 2, q = lane & 3;
  QuadLane L;
  L.q = q;
  L.lane_off = 16u * (uint32_t)q;
  L.row_bytes = row_bytes;
  L.from1 = q >= 1 ? 1.f : 0.f;
  L.from2 = q >= 2 ? 1.f : 0.f;
  L.phi_bytes = reinterpret_cast<const char*>(phi);
  L.theta_q = theta_s + 4 * q;
  const unsigned char* cache_q = lds + 16 * q;

  for (int seg = blockIdx.x * kHotWaves + wave; seg < n_segs; seg += gridDim.x * kHotWaves) {
    const Segment sg = segment_of(doc_off, seg_base, D, seg);
    const int d = sg.d;
    wave_lds_fence();  // the previous segment's reads of theta and the histogram are done
    if (kCountDocs)
      for (int k = lane; k < 16 * NS16; k += 64) hist[k] = 0;
    quad_stage_theta<NS16>(theta, d, ldk, theta_s, tq, q);
    int32_t* z_seg = z + sg.first;
    uint8_t* zb_seg = zb + sg.first;
    const int rel_a = (int)(sg.a - sg.first);
    const int rel_b = (int)(sg.end - sg.first);

    QuadPending P;
    for (int rbase = 0; rbase < rel_b; rbase += 256) {
      P.idle();
      const int lo = max(rel_a, rbase);
      const int hi = min(rel_b, rbase + 256);
      const int n_valid = hi - lo;
      int n_cached = 0;
      {
        const U4 r = random_block(seed, (uint64_t)((sg.first + rbase) >> 2) + (uint64_t)lane, sweep,
                                  kStreamZ, 0);
        // the chunk's order: entries lane, lane + 64, ... of the lists that start at its first token
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
        *reinterpret_cast<uint4*>(strip_r + 4 * lane) = make_uint4(r.x, r.y, r.z, r.w);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          strip_w[lane + 64 * e] = wv[e];
          strip_o[lane + 64 * e] = ov[e];
          n_cached += __popcll(__ballot((wv[e] >> 24) != 0u));
        }
        wave_lds_fence();
      }
      // The first 16 * n_hot_iters tokens of the order are cached: whole iterations that read
      // LDS only.  The rest read memory.  One trip of the loop takes an iteration of each kind:
      // it issues the row loads of the memory one, runs the LDS one from start to end while
      // they are on their way, then pass 2 of the previous memory iteration and pass 1 of this
      // one.  (Both counts are the same for the whole wave.)
      const int n_hot_iters = __builtin_amdgcn_readfirstlane(n_cached) >> 4;
      const int cold0 = 16 * n_hot_iters;
      const int n_cold_iters = (n_valid - cold0 + 15) >> 4;
      const int n_trips = max(n_hot_iters, n_cold_iters);
      for (int it = 0; it < n_trips; ++it) {
        const bool do_cold = it < n_cold_iters, do_hot = it < n_hot_iters;
        float4 ph[NS16];
        uint32_t r_c = 0u, row_off_c = 0u;
        int pos_c = -1;
        if (do_cold) {
          const int j0 = cold0 + 16 * it;
          const int j = j0 + tq;
          const bool valid = j < n_valid;
          const int jj = valid ? j : j0;  // a quad past the end redoes the iteration's first token
          const uint32_t wv = strip_w[jj];
          const int pos = (int)strip_o[jj];
          r_c = strip_r[pos];
          row_off_c = __umul24(wv & 0xFFFFFFu, row_bytes);
          pos_c = valid ? pos : -1;
          const char* rowp = L.phi_bytes + (size_t)(row_off_c + L.lane_off);
#pragma unroll
          for (int c = 0; c < NS16; ++c) ph[c] = *reinterpret_cast<const float4*>(rowp + 64 * c);
        }
        asm volatile("" ::: "memory");  // the loads above are issued before anything below starts
        if (do_hot) {
          const int j = 16 * it + tq;
          const uint32_t wv = strip_w[j];
          const int pos = (int)strip_o[j];
          const uint32_t r = strip_r[pos];
          const unsigned char* crow = cache_q + (size_t)((wv >> 24) - 1u) * kRowLds;
          int theta_off = 4 * q;
          asm volatile("" : "+v"(theta_off));
          const float* theta_p1 = theta_s + theta_off;
          // pass 1 with the row's pieces read from LDS as they are needed
          float ac[NS16];
          float acc = 0.f;
#pragma unroll
          for (int c = 0; c < NS16; ++c) {
            const float4 tc = *reinterpret_cast<const float4*>(theta_p1 + 16 * c);
            const float4 pc = *reinterpret_cast<const float4*>(crow + 64 * c);
            acc = c == 0 ? tc.x * pc.x : fmaf(tc.x, pc.x, acc);
            acc = fmaf(tc.y, pc.y, acc);
            acc = fmaf(tc.z, pc.z, acc);
            acc = fmaf(tc.w, pc.w, acc);
            ac[c] = acc;
          }
          QuadPending H;
          const float S = quad_sum(ac[NS16 - 1]);
          H.t = u24(r) * S;
          // t is a rounded fp32 product everywhere else (it crosses an iteration in a register);
          // here pass 2 follows at once, and the compiler would fuse this product into pass 2's
          // subtraction, unrounded: another threshold in the last bit, and other draws than the
          // plain form's once in a million tokens
          asm volatile("" : "+v"(H.t));
          H.cs = 0;
          H.cprev = 0.f;
          if constexpr (NS16 > 1) {
            constexpr int M = NS16 - 1;
            constexpr int TOP = M >= 8 ? 8 : M >= 4 ? 4 : M >= 2 ? 2 : 1;
            bool m[5] = {false, false, false, false, false};
            bisect_level<NS16, TOP, TOP>(ac, H.t, m, H.cs, H.cprev);
          }
          H.p2 = *reinterpret_cast<const float4*>(crow + 64 * H.cs);
          H.r = r;
          H.row_off = __umul24(wv & 0xFFFFFFu, row_bytes);
          H.pos = pos;
          H.ok = S > 0.f && S <= FLT_MAX;
          H.in_row = S > H.t;
          quad_finish<NS16, kCountDocs>(H, L, K, n_degenerate, zstage, hist);
        }
        if (do_cold) {
          asm volatile("" : "+v"(P.cs)::"memory");
          quad_finish<NS16, kCountDocs>(P, L, K, n_degenerate, zstage, hist);
          int theta_off = 4 * q;
          asm volatile("" : "+v"(theta_off));
          float S, t, cprev;
          int cs;
          quad_pass1<NS16>(ph, theta_s + theta_off, r_c, S, t, cs, cprev);
          // the chunk of stripe cs again, for pass 2 in the next trip
          P.p2 = *reinterpret_cast<const float4*>(L.phi_bytes + (row_off_c + 64u * (uint32_t)cs + L.lane_off));
          P.t = t;
          P.cprev = cprev;
          P.cs = cs;
          P.r = r_c;
          P.row_off = row_off_c;
          P.pos = pos_c;
          P.ok = S > 0.f && S <= FLT_MAX;
          P.in_row = S > t;
        }
      }
      quad_finish<NS16, kCountDocs>(P, L, K, n_degenerate, zstage, hist);
      quad_flush_chunk(zstage, z_seg, zb_seg, rbase, lo, hi, lane);
    }
    if (kCountDocs) {
      wave_lds_fence();
      flush_doc_histogram(hist, n_dk + (size_t)d * ldk, ldk, is_split(seg_base, d), lane);
    }
  }
}

// The processing order of the resident form: one wave per segment; for every 256-token chunk
// a stable partition of its tokens into cached and other words.  slot_of[v] = cache slot + 1
// of word v, or 0.
__global__ __launch_bounds__(256) void lda_build_order_kernel(
    const int32_t* __restrict__ w, const int64_t* __restrict__ doc_off,
    const int32_t* __restrict__ seg_base, int n_segs, int D, const uint8_t* __restrict__ slot_of,
    int32_t* __restrict__ wz, uint8_t* __restrict__ ord) {
  const int lane = threadIdx.x & 63;
  const int seg = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (seg >= n_segs) return;
  const Segment sg = segment_of(doc_off, seg_base, D, seg);
  const int rel_a = (int)(sg.a - sg.first), rel_b = (int)(sg.end - sg.first);
  for (int rbase = 0; rbase < rel_b; rbase += 256) {
    const int lo = max(rel_a, rbase), hi = min(rel_b, rbase + 256);
    int word[4], slot[4];
    bool valid[4];
    int n_c = 0, n_o = 0;  // this lane's cached / other tokens
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int rel = rbase + 4 * lane + e;
      valid[e] = rel >= lo && rel < hi;
      word[e] = valid[e] ? w[sg.first + rel] : 0;
      slot[e] = valid[e] ? (int)slot_of[word[e]] : 0;
      n_c += valid[e] && slot[e] != 0;
      n_o += valid[e] && slot[e] == 0;
    }
    // exclusive sums over the lower lanes, and the wave's number of cached tokens
    int before_c = n_c, before_o = n_o;
    for (int o = 1; o < 64; o <<= 1) {
      const int uc = __shfl_up(before_c, o, 64), uo = __shfl_up(before_o, o, 64);
      if (lane >= o) { before_c += uc; before_o += uo; }
    }
    const int total_c = __shfl(before_c, 63, 64);
    before_c -= n_c;
    before_o -= n_o;
    int32_t* wz_c = wz + (sg.first + lo);
    uint8_t* ord_c = ord + (sg.first + lo);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (!valid[e]) continue;
      const int j = slot[e] != 0 ? before_c++ : total_c + before_o++;
      wz_c[j] = word[e] | (slot[e] << 24);
      ord_c[j] = (uint8_t)(4 * lane + e);
    }
  }
}

// ------------------------------------------------- gather probe (measurement)
// The memory side of the z step alone: the same walk over documents and tokens, the same
// word-id stream and the same loads of phi rows (a quad per token reading 64 bytes a load
// up to 256 topics, a 16-lane row reading 256 bytes a load beyond), with no random
// numbers, no arithmetic and no stores.  Its duration is the floor that the memory
// system sets for any z kernel of this load shape on this corpus; the sampler is held
// against it.  The loaded registers are handed to an empty asm statement, which makes
// the compiler wait for every load without spending an instruction on the values.
template <int NS16>
__global__ __launch_bounds__(256) void lda_gather_probe_quad_kernel(
    const int32_t* __restrict__ w, const int64_t* __restrict__ doc_off,
    const int32_t* __restrict__ seg_base, int n_segs, const float* __restrict__ phi, int D, int ldk) {
  __shared__ uint32_t strip_all[4][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int seg = blockIdx.x * 4 + wave;
  if (seg >= n_segs) return;
  const Segment sg = segment_of(doc_off, seg_base, D, seg);
  const int tq = lane >> 2, q = lane & 3;
  uint32_t* strip = strip_all[wave];
  const uint32_t row_bytes = 4u * (uint32_t)ldk;
  const uint32_t lane_off = 16u * (uint32_t)q;
  const uint32_t last_off = min(64u * (NS16 - 1) + lane_off, row_bytes - 16u);
  const char* phi_bytes = reinterpret_cast<const char*>(phi);
  const int64_t a = sg.a, b = sg.end;
  for (int64_t base = sg.first; base < b; base += 256) {
    const int4 wv = *reinterpret_cast<const int4*>(w + base + 4 * lane);
    wave_lds_fence();
    *reinterpret_cast<int4*>(strip + 4 * lane) = wv;
    wave_lds_fence();
    const int64_t lo = a > base ? a : base;
    const int64_t hi = b < base + 256 ? b : base + 256;
    for (int64_t i0 = lo; i0 < hi; i0 += 16) {
      const int64_t i = i0 + tq;
      const uint32_t v = strip[i < hi ? (int)(i - base) : (int)(lo - base)];
      const uint32_t row_off = __umul24(v, row_bytes);
      const char* rowp = phi_bytes + (size_t)(row_off + lane_off);
      float4 ph[NS16];
#pragma unroll
      for (int c = 0; c < NS16 - 1; ++c) ph[c] = *reinterpret_cast<const float4*>(rowp + 64 * c);
      ph[NS16 - 1] = *reinterpret_cast<const float4*>(phi_bytes + (row_off + last_off));
#pragma unroll
      for (int c = 0; c < NS16; ++c)
        asm volatile("" ::"v"(ph[c].x), "v"(ph[c].y), "v"(ph[c].z), "v"(ph[c].w));
    }
  }
}
template <int NS>
__global__ __launch_bounds__(256) void lda_gather_probe_row_kernel(
    const int32_t* __restrict__ w, const int64_t* __restrict__ doc_off,
    const int32_t* __restrict__ seg_base, int n_segs, const float* __restrict__ phi, int D, int ldk) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int seg = blockIdx.x * 4 + wave;
  if (seg >= n_segs) return;
  const Segment sg = segment_of(doc_off, seg_base, D, seg);
  const int row = lane >> 4, j = lane & 15;
  const uint32_t lane_off = 16u * (uint32_t)j;
  const uint32_t last_off = 4u * (uint32_t)min(64 * (NS - 1) + 4 * j, ldk - 4);
  const char* phi_bytes = reinterpret_cast<const char*>(phi);
  const uint32_t row_bytes = 4u * (uint32_t)ldk;
  const int64_t lo = sg.first > sg.a ? sg.first : sg.a, hi = sg.end;
  for (int64_t i0 = lo; i0 < hi; i0 += 4) {
    const int64_t i = i0 + row;
    const uint32_t v = (uint32_t)w[i < hi ? i : lo];
    const uint32_t row_off = v * row_bytes;
    const char* rowp = phi_bytes + (size_t)(row_off + lane_off);
    float4 qv[NS];
#pragma unroll
    for (int m = 0; m < NS - 1; ++m) qv[m] = *reinterpret_cast<const float4*>(rowp + 256 * m);
    qv[NS - 1] = *reinterpret_cast<const float4*>(phi_bytes + (size_t)(row_off + last_off));
#pragma unroll
    for (int m = 0; m < NS; ++m)
      asm volatile("" ::"v"(qv[m].x), "v"(qv[m].y), "v"(qv[m].z), "v"(qv[m].w));
  }
}

// ------------------------------------------------------- fp64 state: sample z
// The same draw with theta and phi stored as doubles (the precision the paper's experiments
// ran in): every product and sum in fp64, so the result differs from a sum in index order by
// fp64 rounding only.  Written for any K up to 1024 and for checking rather than for speed:
// a quad per token, theta_d as doubles in LDS; one walk over the row leaves the running sum at
// the end of every 16-topic stripe in LDS, the crossing stripe is found there, and that one
// stripe is read again for the topic inside it.
__device__ __forceinline__ double quad_sum_f64(double s) {
  s += __shfl_xor(s, 1, 64);
  s += __shfl_xor(s, 2, 64);
  return s;
}
// Dynamic LDS of a workgroup (four waves): per wave theta_d [ldk] doubles and the stripe ends
// [ldk / 16][16 tokens] doubles, then per wave the histogram [ldk] ints.
__host__ __device__ constexpr size_t z_f64_lds_bytes(int ldk) {
  return 4 * ((size_t)ldk * (2 * sizeof(double) + sizeof(int32_t)));
}
template <bool kCountDocs>
__global__ __launch_bounds__(256) void lda_sample_z_f64_kernel(
    const int32_t* __restrict__ w, const int64_t* __restrict__ doc_off,
    const int32_t* __restrict__ seg_base, int n_segs, const double* __restrict__ theta,
    const double* __restrict__ phi, int32_t* __restrict__ z, int32_t* __restrict__ n_dk, int D, int K,
    int ldk, uint64_t seed, SweepRef sweep_ref, unsigned long long* __restrict__ n_degenerate,
    uint8_t* __restrict__ zb) {
  extern __shared__ __align__(16) double lds_f64[];
  const uint32_t sweep = sweep_ref.get();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int seg = blockIdx.x * 4 + wave;
  if (seg >= n_segs) return;
  const Segment sg = segment_of(doc_off, seg_base, D, seg);
  const int d = sg.d;
  const int tq = lane >> 2, q = lane & 3;
  const int stripes = ldk >> 4;  // rows are padded to whole stripes
  double* th = lds_f64 + (size_t)wave * 2 * ldk;
  double* ends = th + ldk;  // [stripes][16]: running sum at the end of stripe c for token slot tq
  int32_t* hist = reinterpret_cast<int32_t*>(lds_f64 + (size_t)8 * ldk) + (size_t)wave * ldk;
  for (int k = lane; k < ldk; k += 64) {
    th[k] = k < K ? theta[(size_t)d * ldk + k] : 0.0;
    if (kCountDocs) hist[k] = 0;
  }
  wave_lds_fence();
  const double* th_q = th + 4 * q;
  // the lane's four entries of stripe c of row `row`; entries at or past column K count as zero
  auto chunk = [&](const double* row, int c, double (&y)[4]) {
    const int col = 16 * c + 4 * q;
    const double2 lo = *reinterpret_cast<const double2*>(row + col);
    const double2 hi = *reinterpret_cast<const double2*>(row + col + 2);
    y[0] = col + 0 < K ? lo.x : 0.0;
    y[1] = col + 1 < K ? lo.y : 0.0;
    y[2] = col + 2 < K ? hi.x : 0.0;
    y[3] = col + 3 < K ? hi.y : 0.0;
  };
  const int64_t a = sg.first > sg.a ? sg.first : sg.a, b = sg.end;
  for (int64_t i0 = a; i0 < b; i0 += 16) {
    const int64_t i = i0 + tq;
    const bool valid = i < b;
    const int64_t ii = valid ? i : a;
    const double* row = phi + (size_t)w[ii] * ldk;
    const uint32_t r = word_of(random_block(seed, (uint64_t)(ii >> 2), sweep, kStreamZ, 0), (uint32_t)(ii & 3));
    // the walk: the lane's own running sum, the quad's sum of them at every stripe end
    double acc = 0.0;
    wave_lds_fence();  // the previous tokens' stripe ends have been read
    for (int c = 0; c < stripes; ++c) {
      double y[4];
      chunk(row, c, y);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc = fma(th_q[16 * c + e], y[e], acc);
      const double cum = quad_sum_f64(acc);
      if (q == 0) ends[16 * c + tq] = cum;
    }
    const double S = quad_sum_f64(acc);
    const double t = (double)u24(r) * S;
    wave_lds_fence();
    // the crossing stripe among all but the last: the stripe ends do not decrease, so it is the
    // number of ends at or below t, and the running sum before it the last of those
    int cs = 0;
    for (int c = q; c < stripes - 1; c += 4) cs += ends[16 * c + tq] <= t ? 1 : 0;
    cs += __shfl_xor(cs, 1, 64);
    cs += __shfl_xor(cs, 2, 64);
    const double cprev = cs > 0 ? ends[16 * (cs - 1) + tq] : 0.0;
    // the topic inside stripe cs
    double y[4];
    chunk(row, cs, y);
    const double* t2 = th_q + 16 * cs;
    const double l0 = t2[0] * y[0];
    const double l1 = fma(t2[1], y[1], l0);
    const double l2 = fma(t2[2], y[2], l1);
    const double l3 = fma(t2[3], y[3], l2);
    const int qb = lane & ~3;
    const double v0 = __shfl(l3, qb + 0, 64), v1 = __shfl(l3, qb + 1, 64), v2 = __shfl(l3, qb + 2, 64);
    const double excl = q == 0 ? 0.0 : q == 1 ? v0 : q == 2 ? v0 + v1 : (v0 + v1) + v2;
    const double tt = fmax(t - (cprev + excl), 0.0);
    const int e = (l0 <= tt) + (l1 <= tt) + (l2 <= tt);
    int cand = l3 > tt ? 4 * q + e : kNoTopic;
    cand = min(cand, __shfl_xor(cand, 1, 64));
    cand = min(cand, __shfl_xor(cand, 2, 64));
    int k = 16 * cs + cand;
    const bool ok = S > 0.0 && S <= DBL_MAX;  // false for 0, inf and NaN
    const bool in_row = S > t;
    const bool found = in_row && cand != kNoTopic;
    if (__builtin_expect(__any(valid && !(ok && found)), 0)) {
      if (!ok) {
        k = u24_times(r, K);  // zero or non-finite mass: z = floor(u K)
        if (valid && q == 0) atomicAdd(n_degenerate, 1ULL);
      } else if (!found) {
        // rounding put t at or past the running sum that should exceed it: the last topic
        // of positive mass in the crossing stripe (or overall)
        const int limit = in_row ? 16 * (cs + 1) : 16 * stripes;
        int last = -1;
        for (int c = 0; c < stripes; ++c) {
          double yy[4];
          chunk(row, c, yy);
          const int kk = 16 * c + 4 * q;
          if (kk < limit) {
#pragma unroll
            for (int ee = 0; ee < 4; ++ee)
              if (th_q[16 * c + ee] * yy[ee] > 0.0) last = kk + ee;
          }
        }
        last = max(last, __shfl_xor(last, 1, 64));
        last = max(last, __shfl_xor(last, 2, 64));
        k = last;
      }
    }
    k = min(max(k, 0), K - 1);
    if (valid && q == 0) {
      z[i] = k;
      if (zb != nullptr) zb[i] = (uint8_t)k;
      if (kCountDocs) atomicAdd(&hist[k], 1);
    }
  }
  if (kCountDocs) {
    wave_lds_fence();
    flush_doc_histogram(hist, n_dk + (size_t)d * ldk, ldk, is_split(seg_base, d), lane);
  }
}

// --------------------------------------------------------------- count step
// Counting phase (Sect. 4.2): n_dk[d][k] = tokens of document d with z = k;
// n_wk[v][k] = tokens of word v with z = k.  No global atomics: both tables are
// built from LDS histograms whose owner is fixed by the static structure of the
// corpus.
//
// Documents: one wave per segment (a whole document unless it is split) builds
// the row in LDS and stores it, or adds it to the zeroed row of a split document.
__global__ __launch_bounds__(256) void lda_count_docs_kernel(
    const int32_t* __restrict__ z, const int64_t* __restrict__ doc_off,
    const int32_t* __restrict__ seg_base, int n_segs, int32_t* __restrict__ n_dk, int D, int ldk) {
  extern __shared__ int32_t hist_all[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int seg = blockIdx.x * 4 + wave;
  if (seg >= n_segs) return;
  const Segment sg = segment_of(doc_off, seg_base, D, seg);
  int32_t* hist = hist_all + (size_t)wave * ldk;
  for (int k = lane; k < ldk; k += 64) hist[k] = 0;
  wave_lds_fence();
  const int64_t a = sg.first > sg.a ? sg.first : sg.a;
  for (int64_t i = a + lane; i < sg.end; i += 64) atomicAdd(&hist[z[i]], 1);
  wave_lds_fence();
  flush_doc_histogram(hist, n_dk + (size_t)sg.d * ldk, ldk, is_split(seg_base, sg.d), lane);
}

// Words: tokens were sorted by word once (perm).  A word's run of tokens is cut
// into slices; a wave gathers a slice's z through perm into an LDS histogram.
// The gathers touch a cache line per token.  For K <= 256 they read the one-byte
// copy of z that the z kernel writes beside z: a quarter of the footprint, which
// (75 MB at 75M tokens) stays in the 256 MB last-level cache where z itself
// (300 MB) does not.
// A word with a single slice stores its row; a word with several has its row zeroed
// before the launch and every slice adds its non-zero bins with integer atomics (a
// few thousand per address at most: cheap, unlike one atomic per token).  Every word
// has at least one slice, so every row is written each sweep.
//
// The visit is planned once on the host (build_word_major).  The unit of work is an item: a
// list of slices, slice_desc[item_off[i] .. item_off[i + 1]), of about 1500 tokens in all; a
// slice is {first position in perm, end, word, 0 = store the row / 1 = add to it}.
//
// Frequent words are cut by position first.  The token positions 0..N are divided into `ranges`
// equal parts; a frequent word's run (sorted by position) is cut where it passes from one part
// to the next; the pieces of part r, in word order, are dealt into items of equal token counts,
// and the items are visited part by part.  The waves in flight then all gather from the same
// MiB or two of z, which an XCD's L2 holds, instead of from all of it: a line (128 tokens of
// the byte copy) is fetched once per part and XCD rather than once per token (75M tokens: 26M
// L2 misses instead of 50M).  The waves must stay in step for this, and they do not by
// themselves (a wave whose gathers hit runs several times faster than one whose gathers
// miss): a workgroup takes its next four items from a counter (one device-scope atomic per
// workgroup and round; one per wave and slice on that single address cost more than the whole
// kernel).  Rare words (fewer than 64 tokens a part) keep whole slices, bundled into items
// after the parts: their gathers touch a line per token whatever the order.
template <typename ZT>
__global__ __launch_bounds__(256) void lda_count_words_kernel(
    const ZT* __restrict__ z, const int32_t* __restrict__ perm, const int4* __restrict__ slice_desc,
    const int32_t* __restrict__ item_off, int32_t* __restrict__ n_wk, int ldk, int n_items,
    uint32_t* __restrict__ next) {
  extern __shared__ int32_t hist_all[];
  __shared__ uint32_t grabbed[2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int32_t* hist = hist_all + (size_t)wave * ldk;
  // next == NULL: one wave per item.  Otherwise the grid is smaller than the list and loops.
  for (uint32_t round = 0;; ++round) {
    uint32_t first = blockIdx.x * 4u;
    if (next != nullptr) {
      if (threadIdx.x == 0) grabbed[round & 1] = atomicAdd(next, 4u);
      __syncthreads();  // grabbed[] alternates, so one barrier a round is enough
      first = grabbed[round & 1];
    }
    if (first >= (uint32_t)n_items) break;  // the same for the four waves
    const uint32_t it = first + (uint32_t)wave;
    const int i0 = it < (uint32_t)n_items ? item_off[it] : 0;
    const int i1 = it < (uint32_t)n_items ? item_off[it + 1] : 0;
    for (int i = i0; i < i1; ++i) {
      const int4 d = slice_desc[i];
      wave_lds_fence();  // the previous row has been read out
      for (int k = lane; k < ldk; k += 64) hist[k] = 0;
      wave_lds_fence();
      const int end = d.y;
      int j = d.x + lane;
      for (; j + 192 < end; j += 256) {  // four gathers in flight per lane
        const int p0 = perm[j], p1 = perm[j + 64], p2 = perm[j + 128], p3 = perm[j + 192];
        const int z0 = (int)z[p0], z1 = (int)z[p1], z2 = (int)z[p2], z3 = (int)z[p3];
        atomicAdd(&hist[z0], 1);
        atomicAdd(&hist[z1], 1);
        atomicAdd(&hist[z2], 1);
        atomicAdd(&hist[z3], 1);
      }
      for (; j < end; j += 64) atomicAdd(&hist[(int)z[perm[j]]], 1);
      wave_lds_fence();
      int32_t* dst = n_wk + (size_t)d.z * ldk;
      if (d.w == 0) {
        for (int k = lane; k < ldk; k += 64) dst[k] = hist[k];
      } else {
        for (int k = lane; k < ldk; k += 64) {
          const int32_t c = hist[k];
          if (c != 0) atomicAdd(&dst[k], c);
        }
      }
    }
    if (next == nullptr) break;
  }
}

// Zeroes the counter of the looping word-table kernel and the rows of the words whose slices
// add to them (listed in multi_words).
__global__ __launch_bounds__(256) void lda_count_words_prepare_kernel(
    const int32_t* __restrict__ multi_words, int n_multi, int32_t* __restrict__ n_wk, int ldk,
    uint32_t* __restrict__ next) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *next = 0u;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)n_multi * ldk) return;
  const int m = (int)(t / ldk), k = (int)(t - (int64_t)m * ldk);
  n_wk[(size_t)multi_words[m] * ldk + k] = 0;
}

// ---- word table, staged form (large corpora, K <= 256) ----
// The gathers of the kernel above pull a 128-byte line for a byte of z whenever a word's
// tokens lie far apart, which is the rule for all but the most frequent words (75M tokens:
// 4.3 GB moved for 0.46 GB needed).  Here the bytes of z are instead *permuted* into
// word-major order in two passes that read and write whole lines, through LDS; the
// permutation is a property of the corpus and is planned once (build_staged_word_table):
//   pass 1: a workgroup takes a tile of 65536 consecutive positions of zb into LDS and writes
//           them out sorted by destination (the token's index in word-major order).  The
//           destinations 0..N are cut into buckets of 49152; the tile's tokens of bucket b
//           form one run, written to the bucket's part of the intermediate array, behind the
//           runs of the earlier tiles.  (src: the local position of every output slot;
//           ostart / istart: where a tile's run for bucket b starts among its slots / in the
//           intermediate array.)
//   pass 2: a workgroup takes a bucket of the intermediate array (whole lines again) and
//           scatters it inside LDS to word-major order (dst: the local destination of every
//           entry); each wave then owns a chunk of 3072 destinations, walks the words in it
//           and turns each piece into a row with an LDS histogram.  A word that lies inside
//           one chunk has its row stored; a word cut by a chunk border is listed in
//           multi_words (rows zeroed first) and its pieces add their non-zero bins.
constexpr int kWtTile = 65536;                   // positions per tile: a local index fits 16 bits
constexpr int kWtChunk = 3072;                   // destinations per wave of pass 2
constexpr int kWtWaves = 16;
constexpr int kWtBucket = kWtWaves * kWtChunk;   // destinations per workgroup of pass 2
constexpr int kWtMaxBuckets = 8000;              // pass 1 keeps two words per bucket in LDS
__global__ __launch_bounds__(1024) void lda_wt_pass1_kernel(
    const uint8_t* __restrict__ zb, const uint16_t* __restrict__ src, const uint32_t* __restrict__ ostart,
    const uint32_t* __restrict__ istart, uint8_t* __restrict__ inter, int64_t N, int nb) {
  extern __shared__ __align__(16) unsigned char wt_lds[];  // the tile, then ostart[nb + 1], then istart - ostart [nb]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Workgroups go to the 8 XCDs in turn.  An XCD takes a run of consecutive tiles: their runs
  // for a bucket lie one behind the other in the intermediate array, and meet in that XCD's L2
  // as whole lines before they are written back.  (The grid is a multiple of 8.)
  const int t = (int)(blockIdx.x % 8u) * (int)(gridDim.x / 8u) + (int)(blockIdx.x / 8u);
  const int64_t base = (int64_t)t * kWtTile;
  if (base >= N) return;
  const int n = (int)(N - base < kWtTile ? N - base : kWtTile);
  uint32_t* os = reinterpret_cast<uint32_t*>(wt_lds + kWtTile);
  uint32_t* adj = os + (nb + 1);
  for (int e = threadIdx.x * 16; e < n; e += 1024 * 16)  // (zb is padded: the last piece may pass N)
    *reinterpret_cast<uint4*>(wt_lds + e) = *reinterpret_cast<const uint4*>(zb + base + e);
  for (int b = threadIdx.x; b <= nb; b += 1024) os[b] = ostart[(size_t)t * (nb + 1) + b];
  for (int b = threadIdx.x; b < nb; b += 1024)
    adj[b] = istart[(size_t)t * nb + b] - ostart[(size_t)t * (nb + 1) + b];
  __syncthreads();
  // a wave takes a run of consecutive slots; a slot's bucket is found by walking on from the
  // bucket of the slot before (the slots are sorted by bucket)
  const int per = ((n + kWtWaves - 1) / kWtWaves + 63) & ~63;
  const int s0 = wave * per, s1 = min(n, s0 + per);
  if (s0 >= s1) return;
  int b_cur = 0;  // the bucket of slot s0: os[b_cur] <= s0 < os[b_cur + 1]
  {
    int lo = 0, hi = nb;  // largest b with os[b] <= s0
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (os[mid] <= (uint32_t)s0) lo = mid; else hi = mid;
    }
    b_cur = lo;
  }
  constexpr int kDeep = 16;  // slots per lane and round: the loads of all of them are in flight together
  for (int o0 = s0; o0 < s1; o0 += 64 * kDeep) {
    uint32_t p[kDeep];
#pragma unroll
    for (int e = 0; e < kDeep; ++e) {
      const int o = o0 + 64 * e + lane;
      p[e] = o < s1 ? (uint32_t)src[base + o] : 0u;
    }
    int b = b_cur;
#pragma unroll
    for (int e = 0; e < kDeep; ++e) {
      const int o = o0 + 64 * e + lane;
      if (o < s1) {
        while (os[b + 1] <= (uint32_t)o) ++b;  // ends: os[nb] = n > o
        inter[adj[b] + (uint32_t)o] = wt_lds[p[e]];
      }
    }
    // the bucket of the next round's first slot (the same for every lane)
    const int o_next = o0 + 64 * kDeep;
    if (o_next < s1)
      while (os[b_cur + 1] <= (uint32_t)o_next) ++b_cur;
  }
}

__global__ __launch_bounds__(1024) void lda_wt_pass2_kernel(
    const uint8_t* __restrict__ inter, const uint16_t* __restrict__ dst,
    const int32_t* __restrict__ word_off, const int32_t* __restrict__ chunk_word,
    int32_t* __restrict__ n_wk, int ldk, int V, int64_t N) {
  extern __shared__ __align__(16) unsigned char wt_lds[];  // the bucket in word-major order, then 16 histograms [ldk]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t base = (int64_t)blockIdx.x * kWtBucket;
  const int n = (int)(N - base < kWtBucket ? N - base : kWtBucket);
  for (int e = threadIdx.x * 16; e < n; e += 1024 * 16) {  // (both arrays are padded past N)
    const uint4 v = *reinterpret_cast<const uint4*>(inter + base + e);
    const uint4 d0 = *reinterpret_cast<const uint4*>(dst + base + e);
    const uint4 d1 = *reinterpret_cast<const uint4*>(dst + base + e + 8);
    const uint32_t vb[4] = {v.x, v.y, v.z, v.w};
    const uint32_t db[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (e + i < n)
        wt_lds[(db[i >> 1] >> (16 * (i & 1))) & 0xFFFFu] = (unsigned char)(vb[i >> 2] >> (8 * (i & 3)));
  }
  __syncthreads();
  const int c0 = wave * kWtChunk;
  if (c0 >= n) return;
  const int c1 = min(n, c0 + kWtChunk);
  const int64_t g0 = base + c0, g1 = base + c1;  // the chunk's destinations
  int32_t* hist = reinterpret_cast<int32_t*>(wt_lds + kWtBucket) + (size_t)wave * ldk;
  for (int k = lane; k < ldk; k += 64) hist[k] = 0;
  wave_lds_fence();
  int v = chunk_word[blockIdx.x * kWtWaves + wave];  // the word that destination g0 belongs to
  for (bool done = false; !done;) {
    // the offsets of the next 64 words, then up to 63 words from them
    const int64_t off_l = (int64_t)word_off[min(v + lane, V)];
    for (int idx = 0; idx < 63 && !done; ++idx) {
      const int64_t ws = __shfl(off_l, idx, 64), we = __shfl(off_l, idx + 1, 64);
      if (v + idx >= V || ws >= g1) { done = true; break; }
      const int64_t ps = ws > g0 ? ws : g0, pe = we < g1 ? we : g1;
      if (pe > ps) {
        const int a = (int)(ps - base), b = (int)(pe - base);
        for (int o = a + lane; o < b; o += 64) atomicAdd(&hist[wt_lds[o]], 1);
        wave_lds_fence();
        int32_t* row = n_wk + (size_t)(v + idx) * ldk;
        const bool whole = ws >= g0 && we <= g1;
        for (int k = lane; k < ldk; k += 64) {
          const int32_t c = hist[k];
          hist[k] = 0;
          if (whole) row[k] = c;
          else if (c != 0) atomicAdd(&row[k], c);
        }
        wave_lds_fence();
      }
      if (we >= g1) done = true;
    }
    v += 63;
  }
}

// ---- the plan of the staged word table (create) ----
// key = tile of the token with destination j, val = j.
__global__ __launch_bounds__(256) void wt_tile_keys_kernel(const int32_t* __restrict__ perm, int64_t N,
                                                            uint32_t* __restrict__ key,
                                                            uint32_t* __restrict__ val) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= N) return;
  key[j] = (uint32_t)perm[j] / (uint32_t)kWtTile;
  val[j] = (uint32_t)j;
}
// sorted_j: the destinations in (tile, destination) order, i.e. by output slot of pass 1.
// Writes every slot's local source position and counts the tokens of every (tile, bucket).
__global__ __launch_bounds__(256) void wt_slots_kernel(const int32_t* __restrict__ perm,
                                                        const uint32_t* __restrict__ sorted_j, int64_t N,
                                                        int nb, uint16_t* __restrict__ src,
                                                        uint32_t* __restrict__ cnt) {
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= N) return;
  const uint32_t j = sorted_j[s];
  src[s] = (uint16_t)((uint32_t)perm[j] % (uint32_t)kWtTile);
  atomicAdd(&cnt[(size_t)(s / kWtTile) * (nb + 1) + j / (uint32_t)kWtBucket], 1u);
}
// istart[t][b] = b kWtBucket + the tokens of bucket b in tiles before t  (a thread per bucket).
__global__ __launch_bounds__(256) void wt_prefix_buckets_kernel(const uint32_t* __restrict__ cnt, int nt,
                                                                 int nb, uint32_t* __restrict__ istart) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= nb) return;
  uint32_t run = (uint32_t)b * (uint32_t)kWtBucket;
  for (int t = 0; t < nt; ++t) {
    istart[(size_t)t * nb + b] = run;
    run += cnt[(size_t)t * (nb + 1) + b];
  }
}
// In place: cnt[t][0..nb] becomes ostart[t][0..nb], the exclusive sums over b  (a thread per tile).
__global__ __launch_bounds__(256) void wt_prefix_tiles_kernel(uint32_t* __restrict__ cnt, int nt, int nb) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= nt) return;
  uint32_t run = 0;
  for (int b = 0; b <= nb; ++b) {
    const uint32_t c = cnt[(size_t)t * (nb + 1) + b];
    cnt[(size_t)t * (nb + 1) + b] = run;
    run += c;
  }
}
// dst[i] = local destination of the entry that pass 1 writes to intermediate index i.
__global__ __launch_bounds__(256) void wt_dst_kernel(const uint32_t* __restrict__ sorted_j,
                                                      const uint32_t* __restrict__ ostart,
                                                      const uint32_t* __restrict__ istart, int64_t N, int nb,
                                                      uint16_t* __restrict__ dst) {
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= N) return;
  const uint32_t j = sorted_j[s];
  const uint32_t t = (uint32_t)(s / kWtTile), b = j / (uint32_t)kWtBucket;
  const uint32_t i = istart[(size_t)t * nb + b] + ((uint32_t)(s % kWtTile) - ostart[(size_t)t * (nb + 1) + b]);
  dst[i] = (uint16_t)(j - b * (uint32_t)kWtBucket);
}
// chunk_word[c] = the word that destination c kWtChunk belongs to.
__global__ __launch_bounds__(256) void wt_chunk_words_kernel(const int32_t* __restrict__ word_off, int V,
                                                              int n_chunks, int32_t* __restrict__ chunk_word) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= n_chunks) return;
  const int64_t g = (int64_t)c * kWtChunk;
  int lo = 0, hi = V;  // largest v < V with word_off[v] <= g (word_off[0] = 0)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)word_off[mid] <= g) lo = mid; else hi = mid;
  }
  chunk_word[c] = lo;
}

// ---- one-time structure of the corpus (create) ----
__global__ __launch_bounds__(256) void iota_kernel(int32_t* __restrict__ a, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) a[i] = (int32_t)i;
}
// word_off[v] = first position of a key >= v in the sorted keys (v = 0..V).
__global__ __launch_bounds__(256) void word_offsets_kernel(const int32_t* __restrict__ sorted_w,
                                                            int64_t N, int V,
                                                            int32_t* __restrict__ word_off) {
  const int v = blockIdx.x * blockDim.x + threadIdx.x;
  if (v > V) return;
  int64_t lo = 0, hi = N;  // first index with sorted_w[index] >= v
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (sorted_w[mid] < v) lo = mid + 1; else hi = mid;
  }
  word_off[v] = (int32_t)lo;
}
// A rare word's run is cut to about kSliceTokens tokens (at most kMaxSlicesPerWord pieces, at
// least one).
constexpr int kSliceTokens = 4096;
constexpr int kMaxSlicesPerWord = 512;
constexpr int kCountBlocks = 512;     // workgroups of the word-table kernel when it loops
constexpr int kItemsPerRange = 512;   // items a part's frequent-word tokens are dealt into
constexpr int kItemSlicesMax = 32;    // most rare-word slices bundled into one item
// border[h * (ranges + 1) + r] = first index in the run of frequent word heavy[h] (in perm,
// where a word's positions increase) whose position is at least r * range_len.
__global__ __launch_bounds__(256) void range_borders_kernel(
    const int32_t* __restrict__ word_off, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ heavy, int n_heavy, int ranges, int64_t range_len,
    int32_t* __restrict__ border) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_heavy * (ranges + 1)) return;
  const int hi_word = t / (ranges + 1), r = t - hi_word * (ranges + 1);
  const int v = heavy[hi_word];
  int lo = word_off[v], hi = word_off[v + 1];
  if (r == ranges) { border[t] = hi; return; }
  const int64_t pos = (int64_t)r * range_len;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)perm[mid] < pos) lo = mid + 1; else hi = mid;
  }
  border[t] = lo;
}

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

// ------------------------------------------- scratch of augur_lda_loglik_static
// Device memory of the entry point that allocates nothing: the document offsets it forms
// from the caller's lengths, the block partials of its reductions and the logarithm table.
// One copy per GPU, held until the process ends; its contents are whatever the last call
// left.  Host code never uses this name as an address: it asks the runtime for the array's
// device address once per device (static_scratch) and passes that.
constexpr int kStaticMaxDocs = 1 << 20;
constexpr size_t kScratchOffBytes = (sizeof(int64_t) * ((size_t)kStaticMaxDocs + 1) + 255) / 256 * 256;
constexpr size_t kScratchRedBytes = (sizeof(double) * (4 * (size_t)kRedBlocks + 2) + 255) / 256 * 256;
constexpr size_t kScratchTabBytes = (sizeof(double2) * (size_t)kLogTableSize + 255) / 256 * 256;
constexpr size_t kScratchBytes = kScratchOffBytes + kScratchRedBytes + kScratchTabBytes;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// ======================================================================= host
struct augur_lda {
  augur_lda_config cfg{};
  int64_t N = 0;
  int ldk = 0;
  int ns = 0;  // stripes of 64 topics per token row
  hipStream_t stream = nullptr;
  hipStream_t side = nullptr;  // second stream: word counts beside the theta step
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  bool overlap = true;
  bool phi_observed = false;  // phi is data: sweeps leave it (and the word table) alone
  double alpha = 0, beta = 0;
  int32_t *w = nullptr, *z = nullptr, *n_dk = nullptr, *n_wk = nullptr;
  int64_t* doc_off = nullptr;
  int32_t *perm = nullptr, *word_off = nullptr;
  int4* slice_desc = nullptr;     // the slices in visiting order
  int32_t* item_off = nullptr;    // [n_items + 1] into slice_desc
  int n_items = 0;
  bool count_loops = false;       // the word-table kernel takes items from cw_next
  uint32_t* cw_next = nullptr;
  int32_t* multi_words = nullptr;  // words with more than one slice (rows zeroed, slices add)
  int n_multi = 0;
  // the staged form of the word table (K <= 256, from the byte copy of z)
  bool wt_ready = false;
  int wt_mode = 0;                 // 0 automatic, 1 whenever available, 2 never
  int wt_tiles = 0, wt_buckets = 0;
  uint16_t *wt_src = nullptr, *wt_dst = nullptr;
  uint32_t *wt_ostart = nullptr, *wt_istart = nullptr;
  uint8_t* wt_inter = nullptr;
  int32_t* wt_chunk_word = nullptr;
  int32_t* wt_multi = nullptr;     // words cut by a chunk border, and words without tokens
  int wt_n_multi = 0;
  uint8_t* zb = nullptr;    // z in bytes, written by the z kernel when K <= 256
  bool zb_current = false;  // zb holds the z of the last z step
  int32_t* seg_base = nullptr;  // NULL: every document is one segment
  int n_segs = 0;
  // the resident form of the z kernel (K <= 256): rows of the most frequent words in LDS
  std::vector<int32_t> hot_host;  // words by falling frequency (the most frequent 255 that occur)
  int32_t* hot_words = nullptr;   // [n_hot] the cached words, slot order
  int n_hot = 0;                  // cached rows per workgroup (0: form not available)
  int32_t* wz = nullptr;          // [N] word | slot << 24 in processing order
  uint8_t* ord = nullptr;         // [N] position in the chunk, in processing order
  int z_cache_mode = 0;           // 0 automatic, 1 always (when available), 2 never
  int num_cus = 0;
  size_t hot_lds_bytes = 0;       // dynamic LDS of a resident workgroup
  float *theta = nullptr, *phi = nullptr;
  bool f64 = false;                          // fp64 state: theta64 and phi64 hold the state, theta and phi stay NULL
  double *theta64 = nullptr, *phi64 = nullptr;
  double* lg = nullptr;          // [V][ldk] ln Gamma draws of the phi step
  double2* col_partial = nullptr;  // [phi row blocks][K]
  double* col_logZ = nullptr;    // [K]
  GammaShape *shapes_alpha = nullptr, *shapes_beta = nullptr;  // [kShapeTable] each
  double2* log_table = nullptr;                                // [kLogTableSize], see log_tab
  double* exp_table = nullptr;                                 // [kExpTableSize], see exp_tab
  double* red = nullptr;         // [4][kRedBlocks] reduction partials, then the two results
  unsigned long long* counters = nullptr;  // [0] degenerate tokens [1] capped draws [2] bad input [3] sweep counter of the graph (low word)
  int phi_blocks = 0, phi_rows = 0;
  int64_t sweep = 0;
  unsigned long long degenerate_reported = 0;
  // sweep() as a recorded graph
  bool use_graph = true;
  hipGraph_t graph = nullptr;
  hipGraphExec_t graph_exec = nullptr;
  int graph_for = -1;          // the switches the graph was recorded with
  int64_t counter_value = -1;  // what the device's sweep counter (counters[3]) holds once the stream has drained
};

namespace {

bool device_ptrs(const augur_lda* h) { return (h->cfg.flags & AUGUR_PTRS_DEVICE) != 0; }

// Row stride of the [.][K] tables, in elements.  A token's lanes read a row in pieces of 64
// bytes (a quad, up to 256 topics) or 256 bytes (a 16-lane row, beyond); rows that start on
// a multiple of that never have a piece straddle two 128-byte cache lines, which the
// texture addresser pays for with a second pass (with K = 200 and a stride of 800 bytes a
// quarter of the pieces did).
int row_stride(int K) { return (int)round_up(K, K <= 256 ? 16 : 64); }

void free_all(augur_lda* h) {
  (void)hipFree(h->w); (void)hipFree(h->z); (void)hipFree(h->n_dk); (void)hipFree(h->n_wk);
  (void)hipFree(h->doc_off); (void)hipFree(h->theta); (void)hipFree(h->phi); (void)hipFree(h->lg);
  (void)hipFree(h->col_partial); (void)hipFree(h->col_logZ); (void)hipFree(h->red);
  (void)hipFree(h->counters); (void)hipFree(h->perm); (void)hipFree(h->word_off);
  (void)hipFree(h->zb);
  (void)hipFree(h->slice_desc); (void)hipFree(h->item_off); (void)hipFree(h->cw_next);
  (void)hipFree(h->multi_words);
  (void)hipFree(h->shapes_alpha); (void)hipFree(h->shapes_beta); (void)hipFree(h->seg_base);
  (void)hipFree(h->log_table); (void)hipFree(h->exp_table);
  (void)hipFree(h->hot_words); (void)hipFree(h->wz); (void)hipFree(h->ord);
  (void)hipFree(h->theta64); (void)hipFree(h->phi64);
  (void)hipFree(h->wt_src); (void)hipFree(h->wt_dst); (void)hipFree(h->wt_ostart);
  (void)hipFree(h->wt_istart); (void)hipFree(h->wt_inter); (void)hipFree(h->wt_chunk_word);
  (void)hipFree(h->wt_multi);
  if (h->graph_exec) (void)hipGraphExecDestroy(h->graph_exec);
  if (h->graph) (void)hipGraphDestroy(h->graph);
  if (h->side) (void)hipStreamDestroy(h->side);
  if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
  if (h->ev_join) (void)hipEventDestroy(h->ev_join);
}

// Rows of n_dk that several segments add to start from zero.
int zero_split_rows(augur_lda* h, hipStream_t stream) {
  if (h->seg_base == nullptr) return AUGUR_OK;
  hipLaunchKernelGGL(zero_split_rows_kernel, dim3((h->cfg.D + 3) / 4), dim3(256), 0, stream,
                     h->seg_base, h->n_dk, h->cfg.D, h->ldk);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

// Whether the kernels that walk the tokens (z step, log-likelihood) take their resident form.
// By itself the library does when every wave of the chip gets at least 16 documents (fewer leave
// the waves unevenly loaded and the copy of the cached rows unpaid for: 3M tokens in 20,000
// documents at K = 100 take 0.081 against 0.075 ms) and rows are at least five stripes long
// (shorter rows are too cheap to load for the detour to pay).
bool resident_form(const augur_lda* h) {
  return h->n_hot > 0 && h->z_cache_mode != 2 &&
         (h->z_cache_mode == 1 ||
          (h->n_segs >= 16 * kHotWaves * h->num_cus && h->ldk >= 16 * kHotMinStripes));
}

// fused: the kernel also writes the document table n_dk (K <= 256 only); returns
// whether it did through *did_count.
int launch_sample_z(augur_lda* h, SweepRef sweep, bool fuse_doc_counts = false,
                    bool* did_count = nullptr) {
  const int D = h->cfg.D;
  if (did_count) *did_count = false;
  if (D == 0 || h->N == 0) return AUGUR_OK;
  const dim3 grid((h->n_segs + 3) / 4), block(256);
  if (h->f64) {
    if (fuse_doc_counts) {
      const int rc = zero_split_rows(h, h->stream);
      if (rc != AUGUR_OK) return rc;
    }
    const size_t shm = z_f64_lds_bytes(h->ldk);
    uint8_t* zb = h->ldk <= 256 ? h->zb : nullptr;
#define AUGUR_ZD_ARGS                                                                             \
  grid, block, shm, h->stream, h->w, h->doc_off, h->seg_base, h->n_segs, h->theta64, h->phi64, h->z, \
      h->n_dk, D, h->cfg.K, h->ldk, h->cfg.seed, sweep, h->counters, zb
    if (fuse_doc_counts) hipLaunchKernelGGL(lda_sample_z_f64_kernel<true>, AUGUR_ZD_ARGS);
    else hipLaunchKernelGGL(lda_sample_z_f64_kernel<false>, AUGUR_ZD_ARGS);
#undef AUGUR_ZD_ARGS
    AUGUR_HIP_TRY(hipGetLastError());
    if (did_count) *did_count = fuse_doc_counts;
    h->zb_current = zb != nullptr;
    return AUGUR_OK;
  }
  if (fuse_doc_counts && h->ldk <= 256) {
    const int rc = zero_split_rows(h, h->stream);
    if (rc != AUGUR_OK) return rc;
  }
#define AUGUR_ZQ_ARGS                                                                          \
  grid, block, 0, h->stream, h->w, h->doc_off, h->seg_base, h->n_segs, h->theta, h->phi, h->z,  \
      h->n_dk, D, h->cfg.K, h->ldk, h->cfg.seed, sweep, h->counters, h->zb
#define AUGUR_Z_ARGS                                                                          \
  grid, block, 0, h->stream, h->w, h->doc_off, h->seg_base, h->n_segs, h->theta, h->phi, h->z, \
      D, h->cfg.K, h->ldk, h->cfg.seed, sweep, h->counters
#define AUGUR_ZQ_CASE(N16)                                                                   \
  case N16:                                                                                  \
    if (fuse_doc_counts) hipLaunchKernelGGL((lda_sample_z_quad_kernel<N16, true>), AUGUR_ZQ_ARGS);  \
    else hipLaunchKernelGGL((lda_sample_z_quad_kernel<N16, false>), AUGUR_ZQ_ARGS);          \
    break;
#define AUGUR_Z_CASE(NSV) \
  case NSV: hipLaunchKernelGGL(lda_sample_z_kernel<NSV>, AUGUR_Z_ARGS); break;
  if (resident_form(h)) {
    // one workgroup per CU (fewer if there is not a segment for every wave), resident until done
    const dim3 hgrid((unsigned)std::min(h->num_cus, (h->n_segs + kHotWaves - 1) / kHotWaves));
#define AUGUR_ZH_ARGS                                                                               \
  hgrid, dim3(64 * kHotWaves), h->hot_lds_bytes, h->stream, h->wz, h->ord, h->doc_off, h->seg_base, \
      h->n_segs, h->theta, h->phi, h->z, h->n_dk, D, h->cfg.K, h->ldk, h->cfg.seed, sweep,          \
      h->counters, h->zb, h->hot_words, h->n_hot
#define AUGUR_ZH_CASE(N16)                                                                      \
  case N16:                                                                                     \
    if (fuse_doc_counts) hipLaunchKernelGGL((lda_sample_z_hot_kernel<N16, true>), AUGUR_ZH_ARGS);  \
    else hipLaunchKernelGGL((lda_sample_z_hot_kernel<N16, false>), AUGUR_ZH_ARGS);              \
    break;
    switch (h->ldk / 16) {
      AUGUR_ZH_CASE(1) AUGUR_ZH_CASE(2) AUGUR_ZH_CASE(3) AUGUR_ZH_CASE(4) AUGUR_ZH_CASE(5)
      AUGUR_ZH_CASE(6) AUGUR_ZH_CASE(7) AUGUR_ZH_CASE(8) AUGUR_ZH_CASE(9) AUGUR_ZH_CASE(10)
      AUGUR_ZH_CASE(11) AUGUR_ZH_CASE(12) AUGUR_ZH_CASE(13) AUGUR_ZH_CASE(14) AUGUR_ZH_CASE(15)
      AUGUR_ZH_CASE(16)
    }
#undef AUGUR_ZH_CASE
#undef AUGUR_ZH_ARGS
    if (did_count) *did_count = fuse_doc_counts;
    h->zb_current = true;
  } else if (h->ldk <= 256) {
    switch ((h->ldk + 15) / 16) {
      AUGUR_ZQ_CASE(1) AUGUR_ZQ_CASE(2) AUGUR_ZQ_CASE(3) AUGUR_ZQ_CASE(4) AUGUR_ZQ_CASE(5)
      AUGUR_ZQ_CASE(6) AUGUR_ZQ_CASE(7) AUGUR_ZQ_CASE(8) AUGUR_ZQ_CASE(9) AUGUR_ZQ_CASE(10)
      AUGUR_ZQ_CASE(11) AUGUR_ZQ_CASE(12) AUGUR_ZQ_CASE(13) AUGUR_ZQ_CASE(14) AUGUR_ZQ_CASE(15)
      AUGUR_ZQ_CASE(16)
    }
    if (did_count) *did_count = fuse_doc_counts;
    h->zb_current = true;
  } else {
    h->zb_current = false;
    switch (h->ns) {
      AUGUR_Z_CASE(5) AUGUR_Z_CASE(6) AUGUR_Z_CASE(7) AUGUR_Z_CASE(8) AUGUR_Z_CASE(9)
      AUGUR_Z_CASE(10) AUGUR_Z_CASE(11) AUGUR_Z_CASE(12) AUGUR_Z_CASE(13) AUGUR_Z_CASE(14)
      AUGUR_Z_CASE(15) AUGUR_Z_CASE(16)
      default:
        set_error("K = %d is above the supported maximum of 1024 topics", h->cfg.K);
        return AUGUR_ERR_UNIMPLEMENTED;
    }
  }
#undef AUGUR_Z_CASE
#undef AUGUR_ZQ_CASE
#undef AUGUR_Z_ARGS
#undef AUGUR_ZQ_ARGS
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

int launch_count_docs(augur_lda* h, hipStream_t stream) {
  const int D = h->cfg.D;
  if (D == 0) return AUGUR_OK;
  {
    const int rc = zero_split_rows(h, stream);
    if (rc != AUGUR_OK) return rc;
  }
  hipLaunchKernelGGL(lda_count_docs_kernel, dim3((h->n_segs + 3) / 4), dim3(256),
                     sizeof(int32_t) * 4 * (size_t)h->ldk, stream, h->z, h->doc_off, h->seg_base,
                     h->n_segs, h->n_dk, D, h->ldk);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

// Whether the word table is built by the staged kernels.  They read the byte copy of z.  Alone
// on the chip they beat the gathering kernel where that one misses the caches (from about 16M
// tokens on; below, the byte copy lies in the L2s): 75M tokens, 0.38 against 0.70 ms.  Beside
// the theta step they lose: their workgroups need a CU's 16 wave slots and 64 to 76 KiB of
// its LDS at once, which the theta step's small workgroups leave free only rarely, while the
// gathering kernel's workgroups slip in anywhere and their time hides behind the theta step's
// arithmetic (sweep 3.81 against 3.57 ms).  So by itself the library takes the staged form
// only when the word table has the stream to itself.
constexpr int64_t kWtMinTokens = 16 << 20;
bool staged_word_table(const augur_lda* h, bool beside_theta) {
  return h->wt_ready && h->zb_current && h->wt_mode != 2 &&
         (h->wt_mode == 1 || (!beside_theta && h->N >= kWtMinTokens));
}

int launch_count_words(augur_lda* h, hipStream_t stream, bool beside_theta = false) {
  if (h->n_items == 0) return AUGUR_OK;
  if (staged_word_table(h, beside_theta)) {
    const int64_t cells = (int64_t)h->wt_n_multi * h->ldk;
    hipLaunchKernelGGL(lda_count_words_prepare_kernel, dim3((unsigned)std::max<int64_t>(1, (cells + 255) / 256)),
                       dim3(256), 0, stream, h->wt_multi, h->wt_n_multi, h->n_wk, h->ldk, h->cw_next);
    hipLaunchKernelGGL(lda_wt_pass1_kernel, dim3((unsigned)round_up(h->wt_tiles, 8)), dim3(1024),
                       (size_t)kWtTile + sizeof(uint32_t) * (2 * (size_t)h->wt_buckets + 1), stream, h->zb,
                       h->wt_src, h->wt_ostart, h->wt_istart, h->wt_inter, h->N, h->wt_buckets);
    hipLaunchKernelGGL(lda_wt_pass2_kernel, dim3(h->wt_buckets), dim3(1024),
                       (size_t)kWtBucket + sizeof(int32_t) * kWtWaves * (size_t)h->ldk, stream, h->wt_inter,
                       h->wt_dst, h->word_off, h->wt_chunk_word, h->n_wk, h->ldk, h->cfg.V, h->N);
    AUGUR_HIP_TRY(hipGetLastError());
    return AUGUR_OK;
  }
  const size_t shm = sizeof(int32_t) * 4 * (size_t)h->ldk;
  {
    const int64_t cells = (int64_t)h->n_multi * h->ldk;
    hipLaunchKernelGGL(lda_count_words_prepare_kernel, dim3((unsigned)std::max<int64_t>(1, (cells + 255) / 256)),
                       dim3(256), 0, stream, h->multi_words, h->n_multi, h->n_wk, h->ldk, h->cw_next);
  }
  const int cw_blocks = h->count_loops ? kCountBlocks : (h->n_items + 3) / 4;
  uint32_t* next = h->count_loops ? h->cw_next : nullptr;
  if (h->zb_current)
    hipLaunchKernelGGL(lda_count_words_kernel<uint8_t>, dim3(cw_blocks), dim3(256), shm, stream,
                       h->zb, h->perm, h->slice_desc, h->item_off, h->n_wk, h->ldk, h->n_items, next);
  else
    hipLaunchKernelGGL(lda_count_words_kernel<int32_t>, dim3(cw_blocks), dim3(256), shm, stream,
                       h->z, h->perm, h->slice_desc, h->item_off, h->n_wk, h->ldk, h->n_items, next);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

int launch_count(augur_lda* h) {
  const int rc = launch_count_docs(h, h->stream);
  return rc != AUGUR_OK ? rc : launch_count_words(h, h->stream);
}

// Sort the tokens by word once and cut each word's run into slices.
int build_word_major(augur_lda* h) {
  const int64_t N = h->N;
  const int V = h->cfg.V;
  const size_t n_alloc = (size_t)std::max<int64_t>(N, 1);
  int32_t *iota = nullptr, *sorted_w = nullptr, *d_heavy = nullptr, *d_border = nullptr;
  void* temp = nullptr;
  int rc = AUGUR_OK;
  auto check = [&](hipError_t e, const char* what) {
    if (e != hipSuccess && rc == AUGUR_OK) {
      set_error("%s failed: %s", what, hipGetErrorString(e));
      (void)hipGetLastError();  // or the runtime hands the error to the next caller
      rc = AUGUR_ERR_HIP;
    }
    return rc == AUGUR_OK;
  };
  try {
  do {
    if (!check(hipMalloc(&h->perm, sizeof(int32_t) * n_alloc), "hipMalloc(perm)")) break;
    if (!check(hipMalloc(&h->word_off, sizeof(int32_t) * ((size_t)V + 1)), "hipMalloc(word_off)")) break;
    if (!check(hipMalloc(&iota, sizeof(int32_t) * n_alloc), "hipMalloc(iota)")) break;
    if (!check(hipMalloc(&sorted_w, sizeof(int32_t) * n_alloc), "hipMalloc(sorted_w)")) break;
    if (N > 0) {
      hipLaunchKernelGGL(iota_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, h->stream,
                         iota, N);
      int end_bit = 1;
      while ((1LL << end_bit) < V) ++end_bit;
      size_t temp_bytes = 0;
      if (!check(hipcub::DeviceRadixSort::SortPairs(nullptr, temp_bytes, h->w, sorted_w, iota,
                                                    h->perm, (int)N, 0, end_bit, h->stream),
                 "radix sort (size query)")) break;
      if (!check(hipMalloc(&temp, std::max<size_t>(temp_bytes, 16)), "hipMalloc(sort temp)")) break;
      if (!check(hipcub::DeviceRadixSort::SortPairs(temp, temp_bytes, h->w, sorted_w, iota, h->perm,
                                                    (int)N, 0, end_bit, h->stream),
                 "radix sort")) break;
      (void)hipFree(temp);
      temp = nullptr;
    }
    hipLaunchKernelGGL(word_offsets_kernel, dim3((V + 256) / 256), dim3(256), 0, h->stream, sorted_w,
                       N, V, h->word_off);
    // ---- the plan of the word-table kernel, made on the host from the word offsets ----
    std::vector<int32_t> off((size_t)V + 1);
    if (!check(hipMemcpyAsync(off.data(), h->word_off, sizeof(int32_t) * off.size(),
                              hipMemcpyDeviceToHost, h->stream), "hipMemcpyAsync")) break;
    if (!check(hipStreamSynchronize(h->stream), "hipStreamSynchronize")) break;
    {
      // the words whose phi rows the resident z kernel may keep in LDS: the most frequent ones
      std::vector<int32_t> by_freq;
      for (int v = 0; v < V; ++v)
        if (off[v + 1] > off[v]) by_freq.push_back(v);
      const size_t keep = std::min<size_t>(255, by_freq.size());
      std::partial_sort(by_freq.begin(), by_freq.begin() + keep, by_freq.end(), [&](int32_t x, int32_t y) {
        const int fx = off[x + 1] - off[x], fy = off[y + 1] - off[y];
        return fx != fy ? fx > fy : x < y;
      });
      by_freq.resize(keep);
      h->hot_host = std::move(by_freq);
    }
    auto rare_pieces = [](int f) {
      return std::max(1, std::min(kMaxSlicesPerWord, (f + kSliceTokens - 1) / kSliceTokens));
    };
    int64_t n_basic = 0;
    for (int v = 0; v < V; ++v) n_basic += rare_pieces(off[v + 1] - off[v]);
    // One wave per slice when the slices are short (small corpora: the per-slice set-up
    // dominates and parallelism hides it); kCountBlocks looping workgroups when they are long.
    // The kernel then runs beside the theta step (other stream), and the two slow each other
    // down: a bounded grid keeps enough gathers in flight, keeps the waves within two parts of
    // the positions, and lets the theta step finish sooner (large workload, sweep: 4.73 ms at
    // 256 workgroups, 4.52 at 512, 4.64 at 768; one wave per item is slower still).
    const bool looping = n_basic > 4 * kCountBlocks && N / n_basic >= 256;
    // parts of the positions for the frequent words: about 1 MiB of the gathered array each (a
    // quarter of an XCD's L2); none if the whole array is a few MiB anyway
    const int64_t gathered_bytes = N * (h->ldk <= 256 ? 1 : 4);
    int ranges = looping ? (int)std::min<int64_t>(128, (gathered_bytes + (1 << 20) - 1) >> 20) : 1;
    if (ranges <= 4) ranges = 1;
    const int64_t range_len = std::max<int64_t>(1, (N + ranges - 1) / ranges);
    const int heavy_min = 64 * ranges;
    std::vector<int32_t> heavy, border;
    if (ranges > 1)
      for (int v = 0; v < V; ++v)
        if (off[v + 1] - off[v] >= heavy_min) heavy.push_back(v);
    const int n_heavy = (int)heavy.size();
    if (n_heavy > 0) {
      border.resize((size_t)n_heavy * (ranges + 1));
      if (!check(hipMalloc(&d_heavy, sizeof(int32_t) * heavy.size()), "hipMalloc(heavy)")) break;
      if (!check(hipMalloc(&d_border, sizeof(int32_t) * border.size()), "hipMalloc(border)")) break;
      if (!check(hipMemcpyAsync(d_heavy, heavy.data(), sizeof(int32_t) * heavy.size(),
                                hipMemcpyHostToDevice, h->stream), "hipMemcpyAsync")) break;
      const int n_t = n_heavy * (ranges + 1);
      hipLaunchKernelGGL(range_borders_kernel, dim3((n_t + 255) / 256), dim3(256), 0, h->stream,
                         h->word_off, h->perm, d_heavy, n_heavy, ranges, range_len, d_border);
      if (!check(hipMemcpyAsync(border.data(), d_border, sizeof(int32_t) * border.size(),
                                hipMemcpyDeviceToHost, h->stream), "hipMemcpyAsync")) break;
      if (!check(hipStreamSynchronize(h->stream), "hipStreamSynchronize")) break;
    }
    std::vector<int4> desc;            // x first, y end, z word, w: slice index of its word for now
    std::vector<int32_t> item_off(1, 0);
    std::vector<int32_t> pieces_of((size_t)V, 0);
    auto add_slice = [&](int32_t start, int32_t end, int32_t v) {
      desc.push_back(make_int4(start, end, v, 0));
      ++pieces_of[(size_t)v];
    };
    auto close_item = [&]() {
      if ((size_t)item_off.back() != desc.size()) item_off.push_back((int32_t)desc.size());
    };
    // frequent words: part by part, the pieces dealt into items of equal token counts
    int64_t heavy_tokens = 0;
    for (int r = 0; r < ranges && n_heavy > 0; ++r) {
      int64_t total = 0;
      for (int hw = 0; hw < n_heavy; ++hw)
        total += border[(size_t)hw * (ranges + 1) + r + 1] - border[(size_t)hw * (ranges + 1) + r];
      if (total == 0) continue;
      heavy_tokens += total;
      const int64_t share = (total + kItemsPerRange - 1) / kItemsPerRange;
      int64_t pos = 0;
      for (int hw = 0; hw < n_heavy; ++hw) {
        int32_t a = border[(size_t)hw * (ranges + 1) + r];
        const int32_t e = border[(size_t)hw * (ranges + 1) + r + 1];
        while (a < e) {
          const int64_t room = (pos / share + 1) * share - pos;
          const int32_t take = (int32_t)std::min<int64_t>(room, e - a);
          add_slice(a, a + take, heavy[(size_t)hw]);
          a += take;
          pos += take;
          if (pos % share == 0) close_item();
        }
      }
      close_item();
    }
    // rare words: whole slices; when the kernel loops, bundled into items of about the same size
    {
      const int64_t item_tokens =
          heavy_tokens > 0 ? std::max<int64_t>(256, heavy_tokens / ((int64_t)ranges * kItemsPerRange))
                           : 1536;
      size_t next_heavy = 0;
      int64_t in_item = 0;
      for (int v = 0; v < V; ++v) {
        if (next_heavy < heavy.size() && heavy[next_heavy] == v) { ++next_heavy; continue; }
        const int f = off[v + 1] - off[v];
        const int n = rare_pieces(f);
        const int len = (f + n - 1) / n;
        for (int q = 0; q < n; ++q) {
          const int32_t start = std::min(off[v + 1], off[v] + q * len);
          const int32_t end = std::min(off[v + 1], start + len);
          add_slice(start, end, v);
          in_item += end - start;
          const bool full = !looping || in_item >= item_tokens ||
                            (int64_t)desc.size() - item_off.back() >= kItemSlicesMax;
          if (full) { close_item(); in_item = 0; }
        }
      }
      close_item();
    }
    std::vector<int32_t> multi;
    for (int v = 0; v < V; ++v)
      if (pieces_of[(size_t)v] > 1) multi.push_back(v);
    for (auto& d : desc) d.w = pieces_of[(size_t)d.z] > 1 ? 1 : 0;
    h->n_items = (int)item_off.size() - 1;
    h->count_loops = looping;
    h->n_multi = (int)multi.size();
    if (!check(hipMalloc(&h->slice_desc, sizeof(int4) * std::max<size_t>(desc.size(), 1)),
               "hipMalloc(slice_desc)")) break;
    if (!check(hipMalloc(&h->item_off, sizeof(int32_t) * item_off.size()), "hipMalloc(item_off)")) break;
    if (!check(hipMalloc(&h->cw_next, sizeof(uint32_t)), "hipMalloc(cw_next)")) break;
    if (!check(hipMalloc(&h->multi_words, sizeof(int32_t) * std::max<size_t>(multi.size(), 1)),
               "hipMalloc(multi_words)")) break;
    if (!desc.empty() &&
        !check(hipMemcpy(h->slice_desc, desc.data(), sizeof(int4) * desc.size(), hipMemcpyHostToDevice),
               "hipMemcpy")) break;
    if (!check(hipMemcpy(h->item_off, item_off.data(), sizeof(int32_t) * item_off.size(),
                         hipMemcpyHostToDevice), "hipMemcpy")) break;
    if (h->n_multi > 0 &&
        !check(hipMemcpy(h->multi_words, multi.data(), sizeof(int32_t) * multi.size(),
                         hipMemcpyHostToDevice), "hipMemcpy")) break;
  } while (false);
  } catch (const std::exception& e) {  // the host-side plan allocates; nothing may throw out of the C ABI
    set_error("planning the word table failed: %s", e.what());
    rc = AUGUR_ERR_INVALID_ARG;
  }
  (void)hipFree(temp); (void)hipFree(iota); (void)hipFree(sorted_w); (void)hipFree(d_heavy);
  (void)hipFree(d_border);
  return rc;
}

// The plan of the staged word table (see lda_wt_pass1_kernel): made once on the device from
// perm (destination -> position) and the word offsets.  Leaves wt_ready false where the form
// does not apply (more than 256 topics, no tokens, more buckets than pass 1 has LDS for).
int build_staged_word_table(augur_lda* h) {
  h->wt_ready = false;
  const int64_t N = h->N;
  const int V = h->cfg.V;
  if (h->ldk > 256 || N == 0) return AUGUR_OK;
  const int nt = (int)((N + kWtTile - 1) / kWtTile), nb = (int)((N + kWtBucket - 1) / kWtBucket);
  if (nb > kWtMaxBuckets) return AUGUR_OK;
  const int n_chunks = nb * kWtWaves;
  uint32_t *key = nullptr, *key2 = nullptr, *val = nullptr, *sorted_j = nullptr;
  void* temp = nullptr;
  int rc = AUGUR_OK;
  auto check = [&](hipError_t e, const char* what) {
    if (e != hipSuccess && rc == AUGUR_OK) {
      set_error("%s failed: %s", what, hipGetErrorString(e));
      (void)hipGetLastError();  // or the runtime hands the error to the next caller
      rc = AUGUR_ERR_HIP;
    }
    return rc == AUGUR_OK;
  };
  try {
  do {
    // the words whose rows are zeroed first: cut by a chunk border, or without tokens
    std::vector<int32_t> off((size_t)V + 1), multi;
    if (!check(hipMemcpyAsync(off.data(), h->word_off, sizeof(int32_t) * off.size(), hipMemcpyDeviceToHost,
                              h->stream), "hipMemcpyAsync")) break;
    if (!check(hipStreamSynchronize(h->stream), "hipStreamSynchronize")) break;
    for (int v = 0; v < V; ++v)
      if (off[v + 1] == off[v] || off[v] / kWtChunk != (off[v + 1] - 1) / kWtChunk) multi.push_back(v);
    h->wt_n_multi = (int)multi.size();
    const size_t n_pad = (size_t)N + 64;  // the kernels read 16 entries at a time
    if (!check(hipMalloc(&h->wt_multi, sizeof(int32_t) * std::max<size_t>(multi.size(), 1)), "hipMalloc(wt_multi)")) break;
    if (!multi.empty() &&
        !check(hipMemcpy(h->wt_multi, multi.data(), sizeof(int32_t) * multi.size(), hipMemcpyHostToDevice),
               "hipMemcpy")) break;
    if (!check(hipMalloc(&h->wt_src, sizeof(uint16_t) * n_pad), "hipMalloc(wt_src)")) break;
    if (!check(hipMalloc(&h->wt_dst, sizeof(uint16_t) * n_pad), "hipMalloc(wt_dst)")) break;
    if (!check(hipMalloc(&h->wt_inter, n_pad), "hipMalloc(wt_inter)")) break;
    if (!check(hipMalloc(&h->wt_ostart, sizeof(uint32_t) * (size_t)nt * (nb + 1)), "hipMalloc(wt_ostart)")) break;
    if (!check(hipMalloc(&h->wt_istart, sizeof(uint32_t) * (size_t)nt * nb), "hipMalloc(wt_istart)")) break;
    if (!check(hipMalloc(&h->wt_chunk_word, sizeof(int32_t) * (size_t)n_chunks), "hipMalloc(wt_chunk_word)")) break;
    if (!check(hipMalloc(&key, sizeof(uint32_t) * (size_t)N), "hipMalloc(keys)")) break;
    if (!check(hipMalloc(&key2, sizeof(uint32_t) * (size_t)N), "hipMalloc(keys)")) break;
    if (!check(hipMalloc(&val, sizeof(uint32_t) * (size_t)N), "hipMalloc(values)")) break;
    if (!check(hipMalloc(&sorted_j, sizeof(uint32_t) * (size_t)N), "hipMalloc(values)")) break;
    if (!check(hipMemsetAsync(h->wt_ostart, 0, sizeof(uint32_t) * (size_t)nt * (nb + 1), h->stream), "hipMemsetAsync")) break;
    if (!check(hipMemsetAsync(h->wt_dst, 0, sizeof(uint16_t) * n_pad, h->stream), "hipMemsetAsync")) break;
    if (!check(hipMemsetAsync(h->wt_src, 0, sizeof(uint16_t) * n_pad, h->stream), "hipMemsetAsync")) break;
    if (!check(hipMemsetAsync(h->wt_inter, 0, n_pad, h->stream), "hipMemsetAsync")) break;
    const dim3 grid_n((unsigned)((N + 255) / 256)), block(256);
    hipLaunchKernelGGL(wt_tile_keys_kernel, grid_n, block, 0, h->stream, h->perm, N, key, val);
    int end_bit = 1;
    while ((1LL << end_bit) < nt) ++end_bit;
    size_t temp_bytes = 0;
    if (!check(hipcub::DeviceRadixSort::SortPairs(nullptr, temp_bytes, key, key2, val, sorted_j, (int)N, 0,
                                                  end_bit, h->stream), "radix sort (size query)")) break;
    if (!check(hipMalloc(&temp, std::max<size_t>(temp_bytes, 16)), "hipMalloc(sort temp)")) break;
    if (!check(hipcub::DeviceRadixSort::SortPairs(temp, temp_bytes, key, key2, val, sorted_j, (int)N, 0,
                                                  end_bit, h->stream), "radix sort")) break;
    hipLaunchKernelGGL(wt_slots_kernel, grid_n, block, 0, h->stream, h->perm, sorted_j, N, nb, h->wt_src,
                       h->wt_ostart);
    hipLaunchKernelGGL(wt_prefix_buckets_kernel, dim3((nb + 255) / 256), block, 0, h->stream, h->wt_ostart, nt,
                       nb, h->wt_istart);
    hipLaunchKernelGGL(wt_prefix_tiles_kernel, dim3((nt + 255) / 256), block, 0, h->stream, h->wt_ostart, nt, nb);
    hipLaunchKernelGGL(wt_dst_kernel, grid_n, block, 0, h->stream, sorted_j, h->wt_ostart, h->wt_istart, N, nb,
                       h->wt_dst);
    hipLaunchKernelGGL(wt_chunk_words_kernel, dim3((n_chunks + 255) / 256), block, 0, h->stream, h->word_off, V,
                       n_chunks, h->wt_chunk_word);
    if (!check(hipGetLastError(), "launch")) break;
    if (!check(hipStreamSynchronize(h->stream), "hipStreamSynchronize")) break;
    // pass 1 needs more LDS than a kernel gets unasked (the limit belongs to the kernel: always the most)
    if (!check(hipFuncSetAttribute(reinterpret_cast<const void*>(&lda_wt_pass1_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kWtTile + (int)sizeof(uint32_t) * (2 * kWtMaxBuckets + 1)), "hipFuncSetAttribute")) break;
    if (!check(hipFuncSetAttribute(reinterpret_cast<const void*>(&lda_wt_pass2_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kWtBucket + (int)sizeof(int32_t) * kWtWaves * 256), "hipFuncSetAttribute")) break;
    h->wt_tiles = nt;
    h->wt_buckets = nb;
    h->wt_ready = true;
  } while (false);
  } catch (const std::exception& e) {  // the host-side list allocates; nothing may throw out of the C ABI
    set_error("planning the staged word table failed: %s", e.what());
    rc = AUGUR_ERR_INVALID_ARG;
  }
  (void)hipFree(temp); (void)hipFree(key); (void)hipFree(key2); (void)hipFree(val); (void)hipFree(sorted_j);
  return rc;
}

// The resident form of the z kernel (K <= 256): how many phi rows fit in LDS beside the
// strips of 16 waves, which words they are, and the tokens of every chunk in processing
// order.  Leaves n_hot = 0 (form not available) when fewer than 8 rows would fit.
constexpr int kHotLdsBudget = 152 * 1024;  // of the 160 KiB of a CU
const void* hot_kernel_ptr(int ns16, bool count_docs) {
#define AUGUR_HP_CASE(N16)                                                                     \
  case N16:                                                                                    \
    return count_docs ? reinterpret_cast<const void*>(&lda_sample_z_hot_kernel<N16, true>)      \
                      : reinterpret_cast<const void*>(&lda_sample_z_hot_kernel<N16, false>);
  switch (ns16) {
    AUGUR_HP_CASE(1) AUGUR_HP_CASE(2) AUGUR_HP_CASE(3) AUGUR_HP_CASE(4) AUGUR_HP_CASE(5)
    AUGUR_HP_CASE(6) AUGUR_HP_CASE(7) AUGUR_HP_CASE(8) AUGUR_HP_CASE(9) AUGUR_HP_CASE(10)
    AUGUR_HP_CASE(11) AUGUR_HP_CASE(12) AUGUR_HP_CASE(13) AUGUR_HP_CASE(14) AUGUR_HP_CASE(15)
    AUGUR_HP_CASE(16)
  }
#undef AUGUR_HP_CASE
  return nullptr;
}
const void* hot_loglik_kernel_ptr(int ns16) {
#define AUGUR_HL_CASE(N16) \
  case N16: return reinterpret_cast<const void*>(&lda_loglik_hot_kernel<N16>);
  switch (ns16) {
    AUGUR_HL_CASE(1) AUGUR_HL_CASE(2) AUGUR_HL_CASE(3) AUGUR_HL_CASE(4) AUGUR_HL_CASE(5)
    AUGUR_HL_CASE(6) AUGUR_HL_CASE(7) AUGUR_HL_CASE(8) AUGUR_HL_CASE(9) AUGUR_HL_CASE(10)
    AUGUR_HL_CASE(11) AUGUR_HL_CASE(12) AUGUR_HL_CASE(13) AUGUR_HL_CASE(14) AUGUR_HL_CASE(15)
    AUGUR_HL_CASE(16)
  }
#undef AUGUR_HL_CASE
  return nullptr;
}
int setup_resident_form(augur_lda* h) {
  h->n_hot = 0;
  if (h->f64 || h->ldk > 256 || h->N == 0 || h->hot_host.empty()) return AUGUR_OK;
  int cus = 0;
  AUGUR_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->cfg.device));
  h->num_cus = std::max(1, cus);
  const int ns16 = h->ldk / 16;  // rows of tables with up to 256 topics are whole stripes
  const int row_lds = 64 * ns16 + hot_row_pad_bytes(ns16);
  const int waves_bytes = kHotWaves * hot_wave_bytes(ns16, true);
  const int rows = std::min<int>((int)h->hot_host.size(), std::min(255, (kHotLdsBudget - waves_bytes) / row_lds));
  if (rows < 8) return AUGUR_OK;
  h->hot_lds_bytes = (size_t)rows * row_lds + (size_t)waves_bytes;
  for (int cd = 0; cd < 2; ++cd)
    // the limit belongs to the kernel, not to the handle: always the whole budget, so that a
    // handle with fewer cached rows does not lower it under another handle's launches
    AUGUR_HIP_TRY(hipFuncSetAttribute(hot_kernel_ptr(ns16, cd != 0), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      kHotLdsBudget));
  AUGUR_HIP_TRY(hipFuncSetAttribute(hot_loglik_kernel_ptr(ns16), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kHotLdsBudget));
  const int V = h->cfg.V;
  std::vector<uint8_t> slot_of;
  try {
    slot_of.assign((size_t)V, 0);
  } catch (const std::exception&) {
    set_error("out of host memory for the cache slots of %d words", V);
    return AUGUR_ERR_INVALID_ARG;
  }
  for (int s = 0; s < rows; ++s) slot_of[(size_t)h->hot_host[(size_t)s]] = (uint8_t)(s + 1);
  uint8_t* d_slot = nullptr;  // only needed here; the handle's own arrays are freed with the handle
  AUGUR_HIP_TRY(hipMalloc(&h->hot_words, sizeof(int32_t) * (size_t)rows));
  AUGUR_HIP_TRY(hipMalloc(&h->wz, sizeof(int32_t) * (size_t)h->N));
  AUGUR_HIP_TRY(hipMalloc(&h->ord, (size_t)h->N));
  hipError_t e = hipMalloc(&d_slot, (size_t)V);
  if (e == hipSuccess)
    e = hipMemcpy(h->hot_words, h->hot_host.data(), sizeof(int32_t) * (size_t)rows, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(d_slot, slot_of.data(), (size_t)V, hipMemcpyHostToDevice);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(lda_build_order_kernel, dim3((h->n_segs + 3) / 4), dim3(256), 0, h->stream, h->w,
                       h->doc_off, h->seg_base, h->n_segs, h->cfg.D, d_slot, h->wz, h->ord);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
  (void)hipFree(d_slot);
  AUGUR_HIP_TRY(e);
  h->n_hot = rows;
  return AUGUR_OK;
}

// Documents per wave in the theta step: about 600 variables per wave, ten per lane (fewer
// leave the lanes' retry loops unbalanced, more leave a corpus of 20,000 documents with too few
// waves to fill the chip: 3M tokens at K = 100, 0.049 ms at 1000 variables per wave, 0.041 at
// 300 to 600; 300,000 documents at K = 200: 0.71 ms at 1000, 0.66 at 600, 0.84 at 200), and
// the four waves' LDS strips (rows * K doubles each) small enough for several workgroups per CU.
int theta_rows_per_wave(int K) { return std::max(1, std::min(16, 640 / K)); }

int launch_theta(augur_lda* h, SweepRef sweep) {
  const int D = h->cfg.D, K = h->cfg.K;
  const int rows = theta_rows_per_wave(K);
  const int waves = (D + rows - 1) / rows;
  if (h->f64)
    hipLaunchKernelGGL(lda_resample_theta_kernel<double>, dim3((waves + 3) / 4), dim3(256),
                       sizeof(double) * 4 * (size_t)rows * K, h->stream, h->n_dk, h->theta64, D, K,
                       h->ldk, rows, h->alpha, h->shapes_alpha, h->log_table, h->exp_table,
                       h->cfg.seed, sweep, h->counters + 1);
  else
    hipLaunchKernelGGL(lda_resample_theta_kernel<float>, dim3((waves + 3) / 4), dim3(256),
                       sizeof(double) * 4 * (size_t)rows * K, h->stream, h->n_dk, h->theta, D, K,
                       h->ldk, rows, h->alpha, h->shapes_alpha, h->log_table, h->exp_table,
                       h->cfg.seed, sweep, h->counters + 1);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

int launch_phi(augur_lda* h, SweepRef sweep, hipStream_t stream) {
  const int V = h->cfg.V, K = h->cfg.K;
  // Columns per workgroup: all K up to 512, else K cut into equal parts of at most 512 (a
  // workgroup of 1024 threads fills a CU alone and holds it until its slowest wave ends: at
  // K = 1000 two workgroups of 512 threads draw 100M variables in 1.52 instead of 1.65 ms).  Row blocks per workgroup: the
  // count that leaves the fewest idle lanes, in workgroups of at most 512 threads.
  const int col_parts = (K + 511) / 512;
  const int col_w = (K + col_parts - 1) / col_parts;
  int groups = 1;
  double best = 0.0;
  for (int g = 1; g == 1 || g * col_w <= 512; ++g) {
    const double fill = (double)(g * col_w) / (double)round_up(g * col_w, 64);
    if (fill > best + 1e-9) {
      best = fill;
      groups = g;
    }
  }
  const int threads = (int)round_up(groups * col_w, 64);
  hipLaunchKernelGGL(lda_phi_draw_kernel, dim3((h->phi_blocks + groups - 1) / groups, col_parts),
                     dim3(threads), 0, stream, h->n_wk, h->lg, h->col_partial, V, K, h->ldk,
                     h->phi_rows, groups, h->phi_blocks, col_w, h->beta, h->shapes_beta, h->log_table,
                     h->exp_table, h->cfg.seed, sweep, h->counters + 1);
  hipLaunchKernelGGL(lda_phi_norm_kernel, dim3(K), dim3(1024), 0, stream, h->col_partial,
                     h->col_logZ, h->phi_blocks, K);
  const int64_t total = (int64_t)V * h->ldk;
  if (h->f64)
    hipLaunchKernelGGL(lda_phi_write_kernel<double>, dim3((unsigned)((total + 255) / 256)), dim3(256),
                       0, stream, h->lg, h->col_logZ, h->phi64, V, K, h->ldk);
  else
    hipLaunchKernelGGL(lda_phi_write_kernel<float>, dim3((unsigned)((total + 255) / 256)), dim3(256),
                       0, stream, h->lg, h->col_logZ, h->phi, V, K, h->ldk);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

// The log joint and the log marginal of a state: three reduction kernels write block partials
// into red ([4][kRedBlocks] doubles), a last one adds them and writes out[0], out[1] (device).
// seg_base == NULL: one wave per document (n_segs = D).
const void* hot_loglik_kernel_ptr(int ns16);
int launch_loglik(hipStream_t stream, const int32_t* w, const int32_t* z, const int64_t* doc_off,
                  const int32_t* seg_base, int n_segs, const float* theta, const float* phi, int D,
                  int V, int K, int ldk, double alpha, double beta, const double2* log_table,
                  double* red, double* out, const augur_lda* resident = nullptr) {
  double* p_lik = red;
  double* p_marg = red + kRedBlocks;
  double* p_th = red + 2 * kRedBlocks;
  double* p_ph = red + 3 * kRedBlocks;
  const int stripes = (ldk + 15) / 16;
  const size_t shm = sizeof(double) * 4 * 16 * (size_t)stripes;
  if (resident != nullptr) {
    // the token terms by the kernel that keeps the rows of the most frequent words in LDS
    const augur_lda* h = resident;
    const dim3 hgrid((unsigned)std::min(h->num_cus, (n_segs + kHotWaves - 1) / kHotWaves));
    void* args[] = {(void*)&h->wz, (void*)&h->ord, (void*)&z, (void*)&doc_off, (void*)&seg_base, (void*)&n_segs,
                    (void*)&theta, (void*)&phi, (void*)&D, (void*)&K, (void*)&ldk, (void*)&log_table,
                    (void*)&p_lik, (void*)&p_marg, (void*)&h->hot_words, (void*)&h->n_hot};
    AUGUR_HIP_TRY(hipLaunchKernel(hot_loglik_kernel_ptr(ldk / 16), hgrid, dim3(64 * kHotWaves), args,
                                  h->hot_lds_bytes, stream));
  } else {
#define AUGUR_LL_ARGS                                                                            \
  dim3(kRedBlocks), dim3(256), shm, stream, w, z, doc_off, seg_base, n_segs, theta, phi, D, V, K, \
      ldk, log_table, p_lik, p_marg
#define AUGUR_LL_CASE(N16) \
  case N16: hipLaunchKernelGGL(lda_loglik_tokens_kernel<N16>, AUGUR_LL_ARGS); break;
  switch (stripes <= 16 ? stripes : 0) {
    AUGUR_LL_CASE(1) AUGUR_LL_CASE(2) AUGUR_LL_CASE(3) AUGUR_LL_CASE(4) AUGUR_LL_CASE(5)
    AUGUR_LL_CASE(6) AUGUR_LL_CASE(7) AUGUR_LL_CASE(8) AUGUR_LL_CASE(9) AUGUR_LL_CASE(10)
    AUGUR_LL_CASE(11) AUGUR_LL_CASE(12) AUGUR_LL_CASE(13) AUGUR_LL_CASE(14) AUGUR_LL_CASE(15)
    AUGUR_LL_CASE(16)
    default: hipLaunchKernelGGL(lda_loglik_tokens_kernel<0>, AUGUR_LL_ARGS); break;
  }
#undef AUGUR_LL_CASE
#undef AUGUR_LL_ARGS
  }
  hipLaunchKernelGGL(sum_log_kernel<float>, dim3(kRedBlocks), dim3(256), 0, stream, theta, (int64_t)D,
                     K, ldk, log_table, p_th);
  hipLaunchKernelGGL(sum_log_kernel<float>, dim3(kRedBlocks), dim3(256), 0, stream, phi, (int64_t)V, K,
                     ldk, log_table, p_ph);
  const double c_theta = (double)D * (std::lgamma(K * alpha) - K * std::lgamma(alpha));
  const double c_phi = (double)K * (std::lgamma(V * beta) - V * std::lgamma(beta));
  hipLaunchKernelGGL(lda_loglik_finish_kernel, dim3(1), dim3(256), 0, stream, red, c_theta,
                     alpha - 1.0, c_phi, beta - 1.0, out);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}
// The same for the fp64 state.
int launch_loglik_f64(hipStream_t stream, const int32_t* w, const int32_t* z, const int64_t* doc_off,
                      const int32_t* seg_base, int n_segs, const double* theta, const double* phi,
                      int D, int V, int K, int ldk, double alpha, double beta,
                      const double2* log_table, double* red, double* out) {
  double* p_lik = red;
  double* p_marg = red + kRedBlocks;
  double* p_th = red + 2 * kRedBlocks;
  double* p_ph = red + 3 * kRedBlocks;
  hipLaunchKernelGGL(lda_loglik_tokens_f64_kernel, dim3(kRedBlocks), dim3(256),
                     sizeof(double) * 4 * (size_t)ldk, stream, w, z, doc_off, seg_base, n_segs, theta,
                     phi, D, V, K, ldk, log_table, p_lik, p_marg);
  hipLaunchKernelGGL(sum_log_kernel<double>, dim3(kRedBlocks), dim3(256), 0, stream, theta, (int64_t)D,
                     K, ldk, log_table, p_th);
  hipLaunchKernelGGL(sum_log_kernel<double>, dim3(kRedBlocks), dim3(256), 0, stream, phi, (int64_t)V,
                     K, ldk, log_table, p_ph);
  const double c_theta = (double)D * (std::lgamma(K * alpha) - K * std::lgamma(alpha));
  const double c_phi = (double)K * (std::lgamma(V * beta) - V * std::lgamma(beta));
  hipLaunchKernelGGL(lda_loglik_finish_kernel, dim3(1), dim3(256), 0, stream, red, c_theta,
                     alpha - 1.0, c_phi, beta - 1.0, out);
  AUGUR_HIP_TRY(hipGetLastError());
  return AUGUR_OK;
}

// Strided copies between the caller's dense [rows][K] arrays and the padded
// device arrays.
int copy_in(augur_lda* h, void* dst, const void* src, size_t elem, int64_t rows) {
  AUGUR_HIP_TRY(hipMemcpy2DAsync(dst, elem * h->ldk, src, elem * h->cfg.K, elem * h->cfg.K,
                                 (size_t)rows,
                                 device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice,
                                 h->stream));
  return AUGUR_OK;
}
int copy_out(augur_lda* h, void* dst, const void* src, size_t elem, int64_t rows) {
  AUGUR_HIP_TRY(hipMemcpy2DAsync(dst, elem * h->cfg.K, src, elem * h->ldk, elem * h->cfg.K,
                                 (size_t)rows,
                                 device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost,
                                 h->stream));
  return AUGUR_OK;
}

int read_counter(augur_lda* h, int which, unsigned long long* out) {
  AUGUR_HIP_TRY(hipMemcpyAsync(out, h->counters + which, sizeof(unsigned long long),
                               hipMemcpyDeviceToHost, h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  return AUGUR_OK;
}

#define AUGUR_CHECK_HANDLE(h)                              \
  AUGUR_REQUIRE((h) != nullptr, "handle is NULL");         \
  DeviceGuard guard_((h)->cfg.device);                     \
  AUGUR_REQUIRE(guard_.ok, "cannot select device %d", (h)->cfg.device)

#define AUGUR_TRY(expr)              \
  do {                               \
    const int rc_ = (expr);          \
    if (rc_ != AUGUR_OK) return rc_; \
  } while (0)

}  // namespace

extern "C" {

int augur_lda_create(const augur_lda_config* cfg, const int32_t* doc_len, const int32_t* w,
                     augur_lda** out) {
  AUGUR_REQUIRE(out != nullptr, "out is NULL");
  *out = nullptr;
  AUGUR_REQUIRE(cfg != nullptr, "config is NULL");
  AUGUR_REQUIRE(cfg->D > 0 && cfg->V > 0 && cfg->K > 0, "D, V, K must be positive (got %d, %d, %d)",
                cfg->D, cfg->V, cfg->K);
  AUGUR_REQUIRE(cfg->K <= 1024, "K = %d is above the supported maximum of 1024 topics", cfg->K);
  AUGUR_REQUIRE(cfg->V <= (1 << 24), "V = %d is above the supported maximum of 2^24 words", cfg->V);
  AUGUR_REQUIRE((int64_t)cfg->V * row_stride(cfg->K) <= (1LL << 30),
                "V * K = %lld exceeds 2^30 table entries (phi rows are addressed with 32-bit "
                "byte offsets)", (long long)cfg->V * cfg->K);
  AUGUR_REQUIRE(std::isfinite(cfg->alpha) && cfg->alpha > 0.f && std::isfinite(cfg->beta) &&
                    cfg->beta > 0.f,
                "alpha and beta must be positive and finite");
  AUGUR_REQUIRE((cfg->flags & ~(AUGUR_PTRS_DEVICE | AUGUR_STATE_F64)) == 0, "unknown flag bits 0x%x",
                cfg->flags);
  AUGUR_REQUIRE(doc_len != nullptr, "doc_len is NULL");
  int ndev = 0;
  AUGUR_HIP_TRY(hipGetDeviceCount(&ndev));
  AUGUR_REQUIRE(cfg->device >= 0 && cfg->device < ndev, "device %d out of range (%d present)",
                cfg->device, ndev);
  DeviceGuard guard(cfg->device);
  AUGUR_REQUIRE(guard.ok, "cannot select device %d", cfg->device);
  const bool dev = (cfg->flags & AUGUR_PTRS_DEVICE) != 0;
  const int D = cfg->D, V = cfg->V, K = cfg->K;

  augur_lda* h = new (std::nothrow) augur_lda();
  AUGUR_REQUIRE(h != nullptr, "out of host memory");
  h->cfg = *cfg;
  h->stream = (hipStream_t)cfg->stream;
  h->use_graph = h->stream != nullptr;  // the default stream cannot be recorded
  h->f64 = (cfg->flags & AUGUR_STATE_F64) != 0;
  h->alpha = (double)cfg->alpha;
  h->beta = (double)cfg->beta;
  h->ldk = row_stride(K);
  h->ns = (h->ldk + 63) / 64;
  {
    // enough column-waves to fill the chip several times over, at most kPhiRowsMax rows each
    const int waves_per_block = (int)std::min<int64_t>(4, round_up(K, 64) / 64);
    const int want_blocks = (16384 + waves_per_block - 1) / waves_per_block;
    h->phi_rows = std::max(4, std::min(kPhiRowsMax, V / want_blocks));
    h->phi_blocks = (V + h->phi_rows - 1) / h->phi_rows;
  }

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
#define AUGUR_CREATE_FAIL(...)  \
  do {                          \
    set_error(__VA_ARGS__);     \
    free_all(h);                \
    delete h;                   \
    return AUGUR_ERR_INVALID_ARG; \
  } while (0)

  AUGUR_CREATE_TRY(hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking));  // default priority
  AUGUR_CREATE_TRY(hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming));
  AUGUR_CREATE_TRY(hipEventCreateWithFlags(&h->ev_join, hipEventDisableTiming));
  AUGUR_CREATE_TRY(hipMalloc(&h->counters, 4 * sizeof(unsigned long long)));
  AUGUR_CREATE_TRY(hipMemsetAsync(h->counters, 0, 4 * sizeof(unsigned long long), h->stream));
  AUGUR_CREATE_TRY(hipMalloc(&h->doc_off, sizeof(int64_t) * ((size_t)D + 1)));

  // document offsets and N
  if (dev) {
    hipLaunchKernelGGL(doc_offsets_kernel, dim3(1), dim3(1024), 0, h->stream, doc_len, h->doc_off, D,
                       h->counters + 2);
    AUGUR_CREATE_TRY(hipGetLastError());
    int64_t n = 0;
    unsigned long long bad = 0;
    AUGUR_CREATE_TRY(hipMemcpyAsync(&n, h->doc_off + D, sizeof(int64_t), hipMemcpyDeviceToHost,
                                    h->stream));
    AUGUR_CREATE_TRY(hipMemcpyAsync(&bad, h->counters + 2, sizeof(bad), hipMemcpyDeviceToHost,
                                    h->stream));
    AUGUR_CREATE_TRY(hipStreamSynchronize(h->stream));
    if (bad) AUGUR_CREATE_FAIL("doc_len has %llu negative entries", bad);
    h->N = n;
  } else {
    std::vector<int64_t> off;
    try {
      off.assign((size_t)D + 1, 0);
    } catch (const std::exception&) {
      AUGUR_CREATE_FAIL("out of host memory for the offsets of %d documents", D);
    }
    for (int d = 0; d < D; ++d) {
      if (doc_len[d] < 0) AUGUR_CREATE_FAIL("doc_len[%d] = %d is negative", d, doc_len[d]);
      off[d + 1] = off[d] + doc_len[d];
    }
    h->N = off[D];
    AUGUR_CREATE_TRY(hipMemcpy(h->doc_off, off.data(), sizeof(int64_t) * off.size(),
                               hipMemcpyHostToDevice));
  }
  if (h->N > 2147483647LL) AUGUR_CREATE_FAIL("N = %lld tokens exceeds 2^31-1", (long long)h->N);
  if (h->N > 0 && w == nullptr) AUGUR_CREATE_FAIL("w is NULL");
  const size_t n_alloc = (size_t)std::max<int64_t>(h->N, 1);

  if (!dev)
    for (int64_t i = 0; i < h->N; ++i)
      if (w[i] < 0 || w[i] >= V)
        AUGUR_CREATE_FAIL("w[%lld] = %d is outside [0, %d)", (long long)i, w[i], V);

  // 256 spare entries after the last token: the sampler reads word ids four at a time
  AUGUR_CREATE_TRY(hipMalloc(&h->w, sizeof(int32_t) * (n_alloc + 256)));
  AUGUR_CREATE_TRY(hipMemsetAsync(h->w, 0, sizeof(int32_t) * (n_alloc + 256), h->stream));
  AUGUR_CREATE_TRY(hipMalloc(&h->z, sizeof(int32_t) * n_alloc));
  AUGUR_CREATE_TRY(hipMalloc(&h->zb, n_alloc + 64));  // the staged word table reads 16 bytes at a time
  if (h->N > 0)
    AUGUR_CREATE_TRY(hipMemcpyAsync(h->w, w, sizeof(int32_t) * (size_t)h->N,
                                    dev ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice,
                                    h->stream));
  if (dev && h->N > 0) {
    hipLaunchKernelGGL(check_range_kernel, dim3(1024), dim3(256), 0, h->stream, h->w, h->N, 0, V,
                       h->counters + 2);
    unsigned long long bad = 0;
    AUGUR_CREATE_TRY(hipMemcpyAsync(&bad, h->counters + 2, sizeof(bad), hipMemcpyDeviceToHost,
                                    h->stream));
    AUGUR_CREATE_TRY(hipStreamSynchronize(h->stream));
    if (bad) AUGUR_CREATE_FAIL("%llu entries of w are outside [0, %d)", bad, V);
  }

  const size_t dk = (size_t)D * h->ldk, vk = (size_t)V * h->ldk;
  if (h->f64) {
    AUGUR_CREATE_TRY(hipMalloc(&h->theta64, sizeof(double) * dk));
    AUGUR_CREATE_TRY(hipMalloc(&h->phi64, sizeof(double) * vk));
  } else {
    AUGUR_CREATE_TRY(hipMalloc(&h->theta, sizeof(float) * dk));
    AUGUR_CREATE_TRY(hipMalloc(&h->phi, sizeof(float) * vk));
  }
  AUGUR_CREATE_TRY(hipMalloc(&h->n_dk, sizeof(int32_t) * dk));
  AUGUR_CREATE_TRY(hipMalloc(&h->n_wk, sizeof(int32_t) * vk));
  AUGUR_CREATE_TRY(hipMalloc(&h->lg, sizeof(double) * vk));
  AUGUR_CREATE_TRY(hipMalloc(&h->col_partial, sizeof(double2) * (size_t)h->phi_blocks * K));
  AUGUR_CREATE_TRY(hipMalloc(&h->col_logZ, sizeof(double) * (size_t)K));
  AUGUR_CREATE_TRY(hipMalloc(&h->red, sizeof(double) * (4 * kRedBlocks + 2)));
  {
    double2 table[kLogTableSize];
    fill_log_table(table);
    AUGUR_CREATE_TRY(hipMalloc(&h->log_table, sizeof(table)));
    AUGUR_CREATE_TRY(hipMemcpy(h->log_table, table, sizeof(table), hipMemcpyHostToDevice));
    double et[kExpTableSize];
    fill_exp_table(et);
    AUGUR_CREATE_TRY(hipMalloc(&h->exp_table, sizeof(et)));
    AUGUR_CREATE_TRY(hipMemcpy(h->exp_table, et, sizeof(et), hipMemcpyHostToDevice));
  }
  AUGUR_CREATE_TRY(hipMalloc(&h->shapes_alpha, sizeof(GammaShape) * kShapeTable));
  AUGUR_CREATE_TRY(hipMalloc(&h->shapes_beta, sizeof(GammaShape) * kShapeTable));
  hipLaunchKernelGGL(shape_table_kernel, dim3(kShapeTable / 256), dim3(256), 0, h->stream,
                     h->shapes_alpha, h->alpha);
  hipLaunchKernelGGL(shape_table_kernel, dim3(kShapeTable / 256), dim3(256), 0, h->stream,
                     h->shapes_beta, h->beta);
  AUGUR_CREATE_TRY(hipGetLastError());
  if (h->f64) {
    AUGUR_CREATE_TRY(hipMemsetAsync(h->theta64, 0, sizeof(double) * dk, h->stream));
    AUGUR_CREATE_TRY(hipMemsetAsync(h->phi64, 0, sizeof(double) * vk, h->stream));
  } else {
    AUGUR_CREATE_TRY(hipMemsetAsync(h->theta, 0, sizeof(float) * dk, h->stream));
    AUGUR_CREATE_TRY(hipMemsetAsync(h->phi, 0, sizeof(float) * vk, h->stream));
  }
  AUGUR_CREATE_TRY(hipMemsetAsync(h->n_dk, 0, sizeof(int32_t) * dk, h->stream));

  {
    const int rc_w = build_word_major(h);
    if (rc_w != AUGUR_OK) {
      free_all(h);
      delete h;
      return rc_w;
    }
  }

  {
    const int rc_s = build_staged_word_table(h);
    if (rc_s != AUGUR_OK) {
      free_all(h);
      delete h;
      return rc_s;
    }
  }

  {
    // segments of long documents
    int32_t* ns = nullptr;
    void* temp = nullptr;
    size_t temp_bytes = 0;
    AUGUR_CREATE_TRY(hipMalloc(&ns, sizeof(int32_t) * ((size_t)D + 1)));
    hipError_t e = hipMalloc(&h->seg_base, sizeof(int32_t) * ((size_t)D + 1));
    hipLaunchKernelGGL(segment_counts_kernel, dim3((D + 256) / 256), dim3(256), 0, h->stream,
                       h->doc_off, D, ns);
    if (e == hipSuccess)
      e = hipcub::DeviceScan::ExclusiveSum(nullptr, temp_bytes, ns, h->seg_base, D + 1, h->stream);
    if (e == hipSuccess) e = hipMalloc(&temp, std::max<size_t>(temp_bytes, 16));
    if (e == hipSuccess)
      e = hipcub::DeviceScan::ExclusiveSum(temp, temp_bytes, ns, h->seg_base, D + 1, h->stream);
    int32_t total = 0;
    if (e == hipSuccess)
      e = hipMemcpyAsync(&total, h->seg_base + D, sizeof(int32_t), hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    (void)hipFree(ns);
    (void)hipFree(temp);
    AUGUR_CREATE_TRY(e);
    h->n_segs = total;
    if (total == D) {  // the common case: no table needed
      (void)hipFree(h->seg_base);
      h->seg_base = nullptr;
    }
  }

  {
    const int rc_hot = setup_resident_form(h);
    if (rc_hot != AUGUR_OK) {
      free_all(h);
      delete h;
      return rc_hot;
    }
  }

  if (h->f64) {
    // up to 80 KiB of LDS per workgroup at 1024 topics: above the 64 KiB a kernel gets unasked
    // (the limit belongs to the kernel, not to the handle: always the most any handle needs)
    const int lds = (int)z_f64_lds_bytes(1024);
    AUGUR_CREATE_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&lda_sample_z_f64_kernel<true>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    AUGUR_CREATE_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&lda_sample_z_f64_kernel<false>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  }

  // initial state (sweep index 0)
  if (h->N > 0) {
    const int64_t blocks4 = (h->N + 3) / 4;
    hipLaunchKernelGGL(lda_init_z_kernel, dim3((unsigned)((blocks4 + 255) / 256)), dim3(256), 0,
                       h->stream, h->z, h->N, K, cfg->seed);
    AUGUR_CREATE_TRY(hipGetLastError());
  }
  int rc = launch_count(h);
  if (rc == AUGUR_OK) rc = launch_theta(h, SweepRef{0u, nullptr});
  if (rc == AUGUR_OK) rc = launch_phi(h, SweepRef{0u, nullptr}, h->stream);
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
  h->sweep = 0;
  *out = h;
  return AUGUR_OK;
#undef AUGUR_CREATE_TRY
#undef AUGUR_CREATE_FAIL
}

void augur_lda_destroy(augur_lda* h) {
  if (!h) return;
  DeviceGuard guard(h->cfg.device);
  (void)hipStreamSynchronize(h->stream);
  free_all(h);
  delete h;
}

int augur_lda_step_sample_z(augur_lda* h) {
  AUGUR_CHECK_HANDLE(h);
  return launch_sample_z(h, SweepRef{(uint32_t)(h->sweep + 1), nullptr});
}
int augur_lda_step_count(augur_lda* h) {
  AUGUR_CHECK_HANDLE(h);
  return launch_count(h);
}
int augur_lda_step_resample_theta(augur_lda* h) {
  AUGUR_CHECK_HANDLE(h);
  return launch_theta(h, SweepRef{(uint32_t)(h->sweep + 1), nullptr});
}
int augur_lda_step_resample_phi(augur_lda* h) {
  AUGUR_CHECK_HANDLE(h);
  return launch_phi(h, SweepRef{(uint32_t)(h->sweep + 1), nullptr}, h->stream);
}
int augur_lda_step_finish(augur_lda* h) {
  AUGUR_REQUIRE(h != nullptr, "handle is NULL");
  h->sweep += 1;
  return AUGUR_OK;
}

// One sweep with index t.  After the z step the two halves are independent: the
// document table feeds the theta step, the word table the phi step (Sect. 4.2:
// theta and phi are conditionally independent given z).  With overlap on, the
// word table (bound by 4-byte gathers) and the phi step run on a second stream
// beside the document table and the theta step (bound by fp64 arithmetic); the
// main stream then waits for the second.  ev, if given, receives five events on
// the main stream: before z, after z, after the document counts, after theta,
// after everything.
static int run_sweep(augur_lda* h, SweepRef t, hipEvent_t* ev) {
#define AUGUR_MARK(i)                                            \
  if (ev) AUGUR_HIP_TRY(hipEventRecord(ev[i], h->stream))
  AUGUR_MARK(0);
  bool have_doc_counts = false;
  AUGUR_TRY(launch_sample_z(h, t, true, &have_doc_counts));
  AUGUR_MARK(1);
  if (h->phi_observed) {
    // phi held fixed (the paper's map(Set("phi"), ...) use on held-out documents):
    // only z and theta are inferred, so neither the word table nor phi is touched
    if (!have_doc_counts) AUGUR_TRY(launch_count_docs(h, h->stream));
    AUGUR_MARK(2);
    AUGUR_TRY(launch_theta(h, t));
    AUGUR_MARK(3);
    AUGUR_MARK(4);
    h->sweep += 1;
    return AUGUR_OK;
  }
  if (h->overlap) {
    // the short document-table kernel (if the z kernel did not build the table
    // itself) first, so that the theta step and the word-table kernel reach the
    // dispatcher together
    if (!have_doc_counts) AUGUR_TRY(launch_count_docs(h, h->stream));
    AUGUR_HIP_TRY(hipEventRecord(h->ev_fork, h->stream));
    AUGUR_HIP_TRY(hipStreamWaitEvent(h->side, h->ev_fork, 0));
  } else {
    if (!have_doc_counts) AUGUR_TRY(launch_count_docs(h, h->stream));
    AUGUR_TRY(launch_count_words(h, h->stream));
  }
  AUGUR_MARK(2);
  if (h->overlap) {
    AUGUR_TRY(launch_count_words(h, h->side, true));
    AUGUR_TRY(launch_phi(h, t, h->side));
    AUGUR_HIP_TRY(hipEventRecord(h->ev_join, h->side));
  }
  AUGUR_TRY(launch_theta(h, t));
  AUGUR_MARK(3);
  if (h->overlap) AUGUR_HIP_TRY(hipStreamWaitEvent(h->stream, h->ev_join, 0));
  else AUGUR_TRY(launch_phi(h, t, h->stream));
  AUGUR_MARK(4);
#undef AUGUR_MARK
  h->sweep += 1;
  return AUGUR_OK;
}

// One sweep recorded as a HIP graph: the launches of run_sweep (both streams, joined) with the
// sweep index read from the handle's device counter, then a kernel that advances the counter.
// Recorded again when a switch that changes the sequence of launches has been flipped.
static void drop_graph(augur_lda* h) {
  if (h->graph_exec) (void)hipGraphExecDestroy(h->graph_exec);
  if (h->graph) (void)hipGraphDestroy(h->graph);
  h->graph_exec = nullptr;
  h->graph = nullptr;
}
static int graph_key(const augur_lda* h) {
  return (h->overlap ? 1 : 0) | (h->phi_observed ? 2 : 0) | (h->z_cache_mode << 2) | (h->wt_mode << 4);
}
static int record_graph(augur_lda* h) {
  drop_graph(h);
  uint32_t* counter = reinterpret_cast<uint32_t*>(h->counters + 3);
  AUGUR_HIP_TRY(hipStreamBeginCapture(h->stream, hipStreamCaptureModeThreadLocal));
  const int64_t sweep_before = h->sweep;
  int rc = run_sweep(h, SweepRef{0u, counter}, nullptr);
  h->sweep = sweep_before;  // nothing has run yet
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
  h->graph = g;
  const hipError_t ei = hipGraphInstantiate(&h->graph_exec, g, nullptr, nullptr, 0);
  if (ei != hipSuccess) {
    set_error("hipGraphInstantiate failed: %s", hipGetErrorString(ei));
    (void)hipGetLastError();
    drop_graph(h);
    return AUGUR_ERR_HIP;
  }
  h->graph_for = graph_key(h);
  return AUGUR_OK;
}

int augur_lda_sweep(augur_lda* h, int32_t n_sweeps) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(n_sweeps >= 0, "n_sweeps = %d is negative", n_sweeps);
  if (!h->use_graph || n_sweeps == 0) {
    for (int32_t s = 0; s < n_sweeps; ++s)
      AUGUR_TRY(run_sweep(h, SweepRef{(uint32_t)(h->sweep + 1), nullptr}, nullptr));
    return AUGUR_OK;
  }
  if (h->graph_exec == nullptr || h->graph_for != graph_key(h)) AUGUR_TRY(record_graph(h));
  // the device counter holds the index of the next sweep; steps, profiled sweeps and set_state
  // move the host's count without it
  uint32_t* counter = reinterpret_cast<uint32_t*>(h->counters + 3);
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
  h->zb_current = h->ldk <= 256;  // as the recorded z step leaves it
  return AUGUR_OK;
}

int augur_lda_set_graph(augur_lda* h, int32_t on) {
  AUGUR_REQUIRE(h != nullptr, "handle is NULL");
  AUGUR_REQUIRE(on == 0 || h->stream != nullptr,
                "sweeps can only be recorded on a stream of the caller's (config.stream), not on the default stream");
  h->use_graph = on != 0;
  return AUGUR_OK;
}

int augur_lda_set_observed(augur_lda* h, uint32_t mask) {
  AUGUR_REQUIRE(h != nullptr, "handle is NULL");
  AUGUR_REQUIRE((mask & ~AUGUR_OBSERVE_PHI) == 0, "unknown observed-variable bits 0x%x", mask);
  h->phi_observed = (mask & AUGUR_OBSERVE_PHI) != 0;
  return AUGUR_OK;
}

int augur_lda_set_z_cache(augur_lda* h, int32_t mode) {
  AUGUR_REQUIRE(h != nullptr, "handle is NULL");
  AUGUR_REQUIRE(mode >= 0 && mode <= 2, "mode must be 0 (automatic), 1 (always) or 2 (never), got %d", mode);
  h->z_cache_mode = mode;
  return AUGUR_OK;
}

int augur_lda_set_word_table(augur_lda* h, int32_t mode) {
  AUGUR_REQUIRE(h != nullptr, "handle is NULL");
  AUGUR_REQUIRE(mode >= 0 && mode <= 2, "mode must be 0 (automatic), 1 (always) or 2 (never), got %d", mode);
  h->wt_mode = mode;
  return AUGUR_OK;
}

int augur_lda_set_overlap(augur_lda* h, int32_t on) {
  AUGUR_REQUIRE(h != nullptr, "handle is NULL");
  h->overlap = on != 0;
  return AUGUR_OK;
}

int augur_lda_sweep_profile(augur_lda* h, int32_t n_sweeps, double* ms) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(n_sweeps >= 0 && n_sweeps <= 4096 && ms != nullptr,
                "n_sweeps must lie in [0, 4096] and ms must not be NULL");
  for (int i = 0; i < AUGUR_LDA_NSTEPS; ++i) ms[i] = 0.0;
  // five events per sweep, all recorded without a host wait; read back at the end
  std::vector<hipEvent_t> ev((size_t)n_sweeps * 5, nullptr);
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
    rc = run_sweep(h, SweepRef{(uint32_t)(h->sweep + 1), nullptr}, &ev[(size_t)s * 5]);
    if (rc == AUGUR_OK) ++done;
  }
  fail_hip(hipStreamSynchronize(h->stream), "hipStreamSynchronize");
  for (int s = 0; s < done && rc == AUGUR_OK; ++s) {
    hipEvent_t* e = &ev[(size_t)s * 5];
    for (int i = 0; i < 4; ++i) {
      float x = 0.f;
      if (fail_hip(hipEventElapsedTime(&x, e[i], e[i + 1]), "hipEventElapsedTime")) break;
      ms[i] += (double)x;
    }
    float x = 0.f;
    if (fail_hip(hipEventElapsedTime(&x, e[0], e[4]), "hipEventElapsedTime")) break;
    ms[4] += (double)x;
  }
  for (auto& e : ev)
    if (e) (void)hipEventDestroy(e);
  return rc;
}

int augur_lda_probe_gather(augur_lda* h, int32_t reps, double* ms_per_pass) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(reps > 0 && reps <= 4096 && ms_per_pass != nullptr,
                "reps must lie in [1, 4096] and ms_per_pass must not be NULL");
  *ms_per_pass = 0.0;
  if (h->f64) {
    set_error("the gather probe covers the fp32 state only");
    return AUGUR_ERR_UNIMPLEMENTED;
  }
  if (h->N == 0) return AUGUR_OK;
  const dim3 grid((h->n_segs + 3) / 4), block(256);
  auto launch = [&]() -> int {
#define AUGUR_GP_ARGS \
  grid, block, 0, h->stream, h->w, h->doc_off, h->seg_base, h->n_segs, h->phi, h->cfg.D, h->ldk
#define AUGUR_GQ_CASE(N16) \
  case N16: hipLaunchKernelGGL(lda_gather_probe_quad_kernel<N16>, AUGUR_GP_ARGS); break;
#define AUGUR_GR_CASE(NSV) \
  case NSV: hipLaunchKernelGGL(lda_gather_probe_row_kernel<NSV>, AUGUR_GP_ARGS); break;
    if (h->ldk <= 256) {
      switch ((h->ldk + 15) / 16) {
        AUGUR_GQ_CASE(1) AUGUR_GQ_CASE(2) AUGUR_GQ_CASE(3) AUGUR_GQ_CASE(4) AUGUR_GQ_CASE(5)
        AUGUR_GQ_CASE(6) AUGUR_GQ_CASE(7) AUGUR_GQ_CASE(8) AUGUR_GQ_CASE(9) AUGUR_GQ_CASE(10)
        AUGUR_GQ_CASE(11) AUGUR_GQ_CASE(12) AUGUR_GQ_CASE(13) AUGUR_GQ_CASE(14) AUGUR_GQ_CASE(15)
        AUGUR_GQ_CASE(16)
      }
    } else {
      switch (h->ns) {
        AUGUR_GR_CASE(5) AUGUR_GR_CASE(6) AUGUR_GR_CASE(7) AUGUR_GR_CASE(8) AUGUR_GR_CASE(9)
        AUGUR_GR_CASE(10) AUGUR_GR_CASE(11) AUGUR_GR_CASE(12) AUGUR_GR_CASE(13) AUGUR_GR_CASE(14)
        AUGUR_GR_CASE(15) AUGUR_GR_CASE(16)
      }
    }
#undef AUGUR_GR_CASE
#undef AUGUR_GQ_CASE
#undef AUGUR_GP_ARGS
    AUGUR_HIP_TRY(hipGetLastError());
    return AUGUR_OK;
  };
  hipEvent_t e0 = nullptr, e1 = nullptr;
  AUGUR_HIP_TRY(hipEventCreate(&e0));
  hipError_t err = hipEventCreate(&e1);
  int rc = err == hipSuccess ? launch() : AUGUR_OK;  // warm-up pass
  if (err == hipSuccess && rc == AUGUR_OK) err = hipEventRecord(e0, h->stream);
  for (int r = 0; r < reps && err == hipSuccess && rc == AUGUR_OK; ++r) rc = launch();
  if (err == hipSuccess && rc == AUGUR_OK) err = hipEventRecord(e1, h->stream);
  if (err == hipSuccess) err = hipStreamSynchronize(h->stream);
  float ms = 0.f;
  if (err == hipSuccess && rc == AUGUR_OK) err = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (rc != AUGUR_OK) return rc;
  AUGUR_HIP_TRY(err);
  *ms_per_pass = (double)ms / reps;
  return AUGUR_OK;
}

int augur_lda_loglik(augur_lda* h, double* log_joint, double* log_marginal_w) {
  AUGUR_CHECK_HANDLE(h);
  double* out = h->red + 4 * kRedBlocks;
  if (h->f64)
    AUGUR_TRY(launch_loglik_f64(h->stream, h->w, h->z, h->doc_off, h->seg_base, h->n_segs, h->theta64,
                                h->phi64, h->cfg.D, h->cfg.V, h->cfg.K, h->ldk, h->alpha, h->beta,
                                h->log_table, h->red, out));
  else
    AUGUR_TRY(launch_loglik(h->stream, h->w, h->z, h->doc_off, h->seg_base, h->n_segs, h->theta,
                            h->phi, h->cfg.D, h->cfg.V, h->cfg.K, h->ldk, h->alpha, h->beta,
                            h->log_table, h->red, out, resident_form(h) ? h : nullptr));
  double host[2] = {0.0, 0.0};
  AUGUR_HIP_TRY(hipMemcpyAsync(host, out, sizeof(host), hipMemcpyDeviceToHost, h->stream));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  if (log_joint) *log_joint = host[0];
  if (log_marginal_w) *log_marginal_w = host[1];
  unsigned long long deg = 0;
  AUGUR_TRY(read_counter(h, 0, &deg));
  if (deg > h->degenerate_reported) {
    set_error("%llu tokens met a conditional of zero or non-finite mass since the last report",
              deg - h->degenerate_reported);
    h->degenerate_reported = deg;
    return AUGUR_ERR_DEGENERATE;
  }
  return AUGUR_OK;
}

// theta and phi in the handle's own type (elem = its size in bytes).
static int get_state_impl(augur_lda* h, int32_t* z, void* theta, void* phi, int64_t* sweep,
                          size_t elem) {
  if (z && h->N > 0)
    AUGUR_HIP_TRY(hipMemcpyAsync(z, h->z, sizeof(int32_t) * (size_t)h->N,
                                 device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost,
                                 h->stream));
  const void* th = h->f64 ? (const void*)h->theta64 : (const void*)h->theta;
  const void* ph = h->f64 ? (const void*)h->phi64 : (const void*)h->phi;
  if (theta) AUGUR_TRY(copy_out(h, theta, th, elem, h->cfg.D));
  if (phi) AUGUR_TRY(copy_out(h, phi, ph, elem, h->cfg.V));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  if (sweep) *sweep = h->sweep;
  return AUGUR_OK;
}

static int set_state_impl(augur_lda* h, const int32_t* z, const void* theta, const void* phi,
                          int64_t sweep, size_t elem) {
  if (z && h->N > 0) {
    if (!device_ptrs(h)) {
      for (int64_t i = 0; i < h->N; ++i)
        AUGUR_REQUIRE(z[i] >= 0 && z[i] < h->cfg.K, "z[%lld] = %d is outside [0, %d)",
                      (long long)i, z[i], h->cfg.K);
    } else {
      AUGUR_HIP_TRY(hipMemsetAsync(h->counters + 2, 0, sizeof(unsigned long long), h->stream));
      hipLaunchKernelGGL(check_range_kernel, dim3(1024), dim3(256), 0, h->stream, z, h->N, 0,
                         h->cfg.K, h->counters + 2);
      unsigned long long bad = 0;
      AUGUR_TRY(read_counter(h, 2, &bad));
      AUGUR_REQUIRE(bad == 0, "%llu entries of z are outside [0, %d)", bad, h->cfg.K);
    }
    AUGUR_HIP_TRY(hipMemcpyAsync(h->z, z, sizeof(int32_t) * (size_t)h->N,
                                 device_ptrs(h) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice,
                                 h->stream));
    h->zb_current = false;  // the word table reads z itself until the next z step
    AUGUR_TRY(launch_count(h));
  }
  void* th = h->f64 ? (void*)h->theta64 : (void*)h->theta;
  void* ph = h->f64 ? (void*)h->phi64 : (void*)h->phi;
  if (theta) AUGUR_TRY(copy_in(h, th, theta, elem, h->cfg.D));
  if (phi) AUGUR_TRY(copy_in(h, ph, phi, elem, h->cfg.V));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  if (sweep >= 0) h->sweep = sweep;
  return AUGUR_OK;
}

int augur_lda_get_state(augur_lda* h, int32_t* z, float* theta, float* phi, int64_t* sweep) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(!h->f64 || (theta == nullptr && phi == nullptr),
                "this handle keeps theta and phi as fp64: use augur_lda_get_state_f64");
  return get_state_impl(h, z, theta, phi, sweep, sizeof(float));
}
int augur_lda_get_state_f64(augur_lda* h, int32_t* z, double* theta, double* phi, int64_t* sweep) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(h->f64 || (theta == nullptr && phi == nullptr),
                "this handle keeps theta and phi as fp32: use augur_lda_get_state");
  return get_state_impl(h, z, theta, phi, sweep, sizeof(double));
}

int augur_lda_set_state(augur_lda* h, const int32_t* z, const float* theta, const float* phi,
                        int64_t sweep) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(!h->f64 || (theta == nullptr && phi == nullptr),
                "this handle keeps theta and phi as fp64: use augur_lda_set_state_f64");
  return set_state_impl(h, z, theta, phi, sweep, sizeof(float));
}
int augur_lda_set_state_f64(augur_lda* h, const int32_t* z, const double* theta, const double* phi,
                            int64_t sweep) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(h->f64 || (theta == nullptr && phi == nullptr),
                "this handle keeps theta and phi as fp32: use augur_lda_set_state");
  return set_state_impl(h, z, theta, phi, sweep, sizeof(double));
}

int augur_lda_get_counts(augur_lda* h, int32_t* n_dk, int32_t* n_wk) {
  AUGUR_CHECK_HANDLE(h);
  if (n_dk) AUGUR_TRY(copy_out(h, n_dk, h->n_dk, sizeof(int32_t), h->cfg.D));
  if (n_wk) AUGUR_TRY(copy_out(h, n_wk, h->n_wk, sizeof(int32_t), h->cfg.V));
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  return AUGUR_OK;
}

int augur_lda_get_degenerate(augur_lda* h, int64_t* count) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_REQUIRE(count != nullptr, "count is NULL");
  unsigned long long c = 0;
  AUGUR_TRY(read_counter(h, 0, &c));
  *count = (int64_t)c;
  return AUGUR_OK;
}

int augur_lda_sync(augur_lda* h) {
  AUGUR_CHECK_HANDLE(h);
  AUGUR_HIP_TRY(hipStreamSynchronize(h->stream));
  return AUGUR_OK;
}

// ---------------------------------------------------- the call that allocates nothing
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};
// Device address of `scratch` on the current device (asked for once per device).
int static_scratch(int device, unsigned char** out) {
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device] == nullptr) {
    void* p = nullptr;
    AUGUR_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    AUGUR_REQUIRE(p != nullptr, "the runtime returned no address for the scratch array");
    g_scratch_ptr[device] = static_cast<unsigned char*>(p);
  }
  *out = g_scratch_ptr[device];
  return AUGUR_OK;
}
}  // namespace

int augur_lda_loglik_static(const augur_lda_static_args* a, double* out) {
  AUGUR_REQUIRE(a != nullptr && out != nullptr, "args or out is NULL");
  AUGUR_REQUIRE(a->D > 0 && a->V > 0 && a->K > 0, "D, V, K must be positive (got %d, %d, %d)", a->D,
                a->V, a->K);
  AUGUR_REQUIRE(a->D <= kStaticMaxDocs,
                "D = %d exceeds the %d documents whose offsets fit the library's static scratch "
                "memory; use a handle (augur_lda_create, augur_lda_loglik) for larger corpora",
                a->D, kStaticMaxDocs);
  AUGUR_REQUIRE(a->K <= 1024, "K = %d is above the supported maximum of 1024 topics", a->K);
  AUGUR_REQUIRE(a->ld >= a->K && a->ld % 4 == 0,
                "ld = %d must be a multiple of 4 and at least K = %d", a->ld, a->K);
  AUGUR_REQUIRE((int64_t)a->V * a->ld <= (1LL << 30), "V * ld = %lld exceeds 2^30 table entries",
                (long long)a->V * a->ld);
  AUGUR_REQUIRE(std::isfinite(a->alpha) && a->alpha > 0.f && std::isfinite(a->beta) && a->beta > 0.f,
                "alpha and beta must be positive and finite");
  AUGUR_REQUIRE(a->doc_len != nullptr && a->w != nullptr && a->z != nullptr && a->theta != nullptr &&
                    a->phi != nullptr,
                "doc_len, w, z, theta and phi must not be NULL");
  AUGUR_REQUIRE(((uintptr_t)a->theta & 15) == 0 && ((uintptr_t)a->phi & 15) == 0 &&
                    ((uintptr_t)out & 7) == 0,
                "theta and phi must be 16-byte aligned and out 8-byte aligned");
  AUGUR_REQUIRE(a->device >= 0 && a->device < kMaxDevices, "device %d out of range", a->device);
  int ndev = 0;
  AUGUR_HIP_TRY(hipGetDeviceCount(&ndev));
  AUGUR_REQUIRE(a->device < ndev, "device %d out of range (%d present)", a->device, ndev);
  DeviceGuard guard(a->device);
  AUGUR_REQUIRE(guard.ok, "cannot select device %d", a->device);
  unsigned char* base = nullptr;
  AUGUR_TRY(static_scratch(a->device, &base));
  int64_t* doc_off = reinterpret_cast<int64_t*>(base);
  double* red = reinterpret_cast<double*>(base + kScratchOffBytes);
  double2* table = reinterpret_cast<double2*>(base + kScratchOffBytes + kScratchRedBytes);
  hipStream_t stream = (hipStream_t)a->stream;
  // every part of the scratch memory that the kernels below read is written first, on this
  // stream: the offsets [0, D], all block partials, the table; nothing needs clearing
  hipLaunchKernelGGL(doc_offsets_kernel, dim3(1), dim3(1024), 0, stream, a->doc_len, doc_off, a->D,
                     (unsigned long long*)nullptr);
  hipLaunchKernelGGL(log_table_kernel, dim3(1), dim3(256), 0, stream, table);
  AUGUR_HIP_TRY(hipGetLastError());
  return launch_loglik(stream, a->w, a->z, doc_off, nullptr, a->D, a->theta, a->phi, a->D, a->V, a->K,
                       a->ld, (double)a->alpha, (double)a->beta, table, red, out);
}

}  // extern "C"

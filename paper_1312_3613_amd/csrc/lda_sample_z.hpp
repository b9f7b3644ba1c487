// sample_z (Sect. 4.2): the row kernel (up to 1024 topics), the quad kernel and its resident form (up to 256),
// the gather probe that measures their memory side, and the kernel of the fp64 state.
// Part of the LDA translation unit (lda.hip includes these files in order; they share one
// anonymous namespace's worth of helpers and are not meant to be included anywhere else).
#pragma once

namespace {

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
  // A workgroup owns a run of consecutive segments; its waves take them one at a time from a
  // counter in LDS, so that none idles while another still has documents waiting (with fixed
  // shares of a few documents a wave, as in a corpus of 20,000 documents, the slowest wave
  // sets the time).  Which wave draws a document does not matter to the result.
  __shared__ int next_seg;
  if (threadIdx.x == 0) next_seg = 0;
  __syncthreads();  // the only barrier: every wave passes it before it looks for work
  const int segs_per_group = (n_segs + (int)gridDim.x - 1) / (int)gridDim.x;
  const int seg_first = (int)blockIdx.x * segs_per_group;
  const int seg_end = min(n_segs, seg_first + segs_per_group);
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

  for (;;) {
    int taken = 0;
    if (lane == 0) taken = atomicAdd(&next_seg, 1);
    const int seg = seg_first + __builtin_amdgcn_readfirstlane(taken);
    if (seg >= seg_end) break;
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

}  // namespace

// Constants, wave-level helpers, document segments and the initial z of the LDA kernels.
// Part of the LDA translation unit (lda.hip includes these files in order; they share one
// anonymous namespace's worth of helpers and are not meant to be included anywhere else).
#pragma once

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

}  // namespace

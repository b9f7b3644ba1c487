// count_accumulate (Sect. 4.2): the document table, the word table by gathers and in its staged form, and the
// kernels that plan both once per corpus.
// Part of the LDA translation unit (lda.hip includes these files in order; they share one
// anonymous namespace's worth of helpers and are not meant to be included anywhere else).
#pragma once

namespace {

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

// The same for small corpora, where most slices have a few dozen tokens (3M tokens over 50,000 words:
// 60 on average, most words far fewer) and a wave per slice spends its time waiting on chains of
// dependent loads (perm, then z, then the LDS histogram, then the row).  Used when the kernel does
// not loop; every item is then a single slice, and the plan lists the slices of at least 64 tokens
// first.  Those keep a wave each (workgroups [0, big_blocks)).  The shorter ones are taken four
// at a time by a wave, 16 lanes a slice: four times the loads in flight and a quarter of the
// instructions per slice for clearing and writing out rows (16 bytes a lane).
template <typename ZT>
__global__ __launch_bounds__(256) void lda_count_words_mixed_kernel(
    const ZT* __restrict__ z, const int32_t* __restrict__ perm, const int4* __restrict__ slice_desc,
    int32_t* __restrict__ n_wk, int ldk, int n_big, int n_slices, int big_blocks) {
  extern __shared__ __align__(16) int32_t hist_all[];  // [4 waves][4 quarters][ldk]; a whole wave uses its first
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if ((int)blockIdx.x < big_blocks) {
    const int i = blockIdx.x * 4 + wave;
    if (i >= n_big) return;
    int32_t* hist = hist_all + (size_t)(wave * 4) * ldk;
    const int4 d = slice_desc[i];
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
    return;
  }
  const int l16 = lane & 15, quarter = lane >> 4;
  const int i = n_big + (((int)blockIdx.x - big_blocks) * 4 + wave) * 4 + quarter;
  if (i >= n_slices) return;
  int4* hist4 = reinterpret_cast<int4*>(hist_all + (size_t)(wave * 4 + quarter) * ldk);
  int32_t* hist = reinterpret_cast<int32_t*>(hist4);
  const int n4 = ldk >> 2;  // rows are multiples of 16 entries
  const int4 d = slice_desc[i];
  for (int k4 = l16; k4 < n4; k4 += 16) hist4[k4] = make_int4(0, 0, 0, 0);
  wave_lds_fence();
  for (int j = d.x + l16; j < d.y; j += 16) atomicAdd(&hist[(int)z[perm[j]]], 1);  // fewer than 64 tokens
  wave_lds_fence();
  int32_t* dst = n_wk + (size_t)d.z * ldk;
  if (d.w == 0) {
    for (int k4 = l16; k4 < n4; k4 += 16) reinterpret_cast<int4*>(dst)[k4] = hist4[k4];
  } else {
    for (int k = l16; k < ldk; k += 16) {
      const int32_t c = hist[k];
      if (c != 0) atomicAdd(&dst[k], c);
    }
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

}  // namespace

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
//
// This file holds the host side (handle, launches, schedule, graph, C ABI); the kernels are in
// lda_device.hpp (helpers, segments), lda_sample_z.hpp, lda_count.hpp, lda_gamma.hpp and
// lda_loglik.hpp, included below into this one translation unit.
#include "common.hpp"

#include <hipcub/hipcub.hpp>

#include <algorithm>
#include <exception>
#include <mutex>
#include <new>
#include <vector>

using namespace augur;

// The kernels, in the order of the sweep:
#include "lda_device.hpp"
#include "lda_sample_z.hpp"
#include "lda_count.hpp"
#include "lda_gamma.hpp"
#include "lda_loglik.hpp"

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
  int n_big = 0;                  // not looping: the slices of at least 64 tokens, listed first
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
  if (!h->count_loops) {
    // a wave per slice of at least 64 tokens, four shorter slices per wave
    const int big_blocks = (h->n_big + 3) / 4;
    const dim3 qgrid((unsigned)(big_blocks + (h->n_items - h->n_big + 15) / 16));
    if (h->zb_current)
      hipLaunchKernelGGL(lda_count_words_mixed_kernel<uint8_t>, qgrid, dim3(256), 4 * shm, stream, h->zb,
                         h->perm, h->slice_desc, h->n_wk, h->ldk, h->n_big, h->n_items, big_blocks);
    else
      hipLaunchKernelGGL(lda_count_words_mixed_kernel<int32_t>, qgrid, dim3(256), 4 * shm, stream, h->z,
                         h->perm, h->slice_desc, h->n_wk, h->ldk, h->n_big, h->n_items, big_blocks);
    AUGUR_HIP_TRY(hipGetLastError());
    return AUGUR_OK;
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
    int slice_tokens = kSliceTokens;
    auto rare_pieces = [&slice_tokens](int f) {
      return std::max(1, std::min(kMaxSlicesPerWord, (f + slice_tokens - 1) / slice_tokens));
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
    // a wave per slice: shorter slices, so that the most frequent words do not end the kernel alone
    // (3M tokens: word table 0.034 ms with slices of 4096 tokens, 0.030 with 1024 to 2048, 0.036 with 256)
    if (!looping) slice_tokens = kSliceTokens / 2;
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
    if (!looping) {
      // every item is one slice: the long ones first (a wave each), then the short ones (four a wave)
      std::stable_partition(desc.begin(), desc.end(), [](const int4& d) { return d.y - d.x >= 64; });
      h->n_big = (int)std::count_if(desc.begin(), desc.end(), [](const int4& d) { return d.y - d.x >= 64; });
    }
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

/*
 * augur.h - C ABI of the MI355X (gfx950) uncollapsed Gibbs sweep for the two
 * latent-variable models of Augur (arXiv 1312.3613): latent Dirichlet allocation
 * (Fig. 1) and a Gaussian mixture (supplementary material, known-covariance
 * variant).  One process, one GPU.  Every step of the sweep runs in HIP kernels;
 * there is no CPU fallback.
 *
 * Conventions (all entry points)
 *   - Return value: AUGUR_OK (0) or a negative AUGUR_ERR_* code.  Nothing throws
 *     or aborts.  augur_last_error() gives the message of the last failing call
 *     on the calling thread.  A failing HIP call is reported through the return
 *     value only: its error is cleared from the runtime's own per-thread state,
 *     so that the caller's next HIP call does not find it there.
 *   - Data pointers are HOST pointers unless the handle was created with
 *     AUGUR_PTRS_DEVICE in config.flags, in which case every data pointer passed
 *     to create/get_x/set_x of that handle is a DEVICE pointer on config.device.
 *     Scalar outputs (double*, int64_t*) are always host pointers.
 *   - create copies its inputs; the caller keeps ownership of every buffer it
 *     passes and may free it on return.  get_x copies into caller-allocated
 *     buffers; a NULL data pointer means "skip this array".
 *   - Work is enqueued on config.stream (a hipStream_t; NULL = the default
 *     stream).  sweep and step_x do not synchronise; loglik, get_x, set_x and
 *     sync do.  A handle must not be used from two threads at once; distinct
 *     handles are independent.
 *   - Random numbers: Philox4x32-10 with key = seed and counter =
 *     (variable index lo, hi, sweep index, stream<<24 | attempt), so a state and
 *     a sweep index determine every draw.  Sweep index 0 initialises; sweep()
 *     advances the index by one per sweep, starting at 1.
 */
#ifndef AUGUR_H
#define AUGUR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AUGUR_OK 0
#define AUGUR_ERR_INVALID_ARG (-1)   /* NULL, non-positive size, out-of-range word, ... */
#define AUGUR_ERR_HIP (-2)           /* HIP runtime failure; message has hipGetErrorString */
#define AUGUR_ERR_DEGENERATE (-3)    /* non-fatal: some conditional had zero/non-finite mass */
#define AUGUR_ERR_UNIMPLEMENTED (-4)

#define AUGUR_PTRS_DEVICE 1u
/* LDA only: theta and phi are stored, read and multiplied as fp64 (the precision the paper's
 * own experiments ran in, Sect. 5) instead of fp32.  The draws (Philox stream, Gamma variates,
 * normalisation in fp64) are the same; what changes is the rounding of the stored
 * probabilities (floored at DBL_MIN instead of FLT_MIN) and of the z step's products and
 * running sums.  The z step of such a handle is a plain kernel written for checking, about
 * three times slower than the fp32 one (it moves twice the bytes); theta, phi, the counts and
 * the log densities cost the same.  augur_lda_probe_gather is not available on such a handle. */
#define AUGUR_STATE_F64 2u

const char* augur_last_error(void); /* thread-local; valid until the next call on this thread */
const char* augur_version(void);

/* ------------------------------------------------------------------ LDA (Fig. 1)
 * phi_k ~ Dirichlet(beta 1_V), theta_d ~ Dirichlet(alpha 1_K),
 * z_i ~ Categorical(theta_d), w_i ~ Categorical(phi_{z_i}); w observed.
 * Layout: w, z flat doc-major int32[N]; theta float[D][K]; phi float[V][K]
 * (row = word, i.e. the transpose of the paper's K x V array); counts
 * n_dk int32[D][K] (the paper's c_m), n_wk int32[V][K] (the paper's c_k). */
typedef struct augur_lda augur_lda;

typedef struct {
  int32_t D, V, K;      /* documents (paper: M), vocabulary size, topics */
  float alpha, beta;    /* symmetric Dirichlet hyper-parameters, > 0, finite */
  uint64_t seed;
  int32_t device;       /* HIP device ordinal */
  void* stream;         /* hipStream_t or NULL */
  uint32_t flags;       /* 0 or any of AUGUR_PTRS_DEVICE, AUGUR_STATE_F64 */
} augur_lda_config;

/* Builds the sampler state for a corpus.  doc_len[D] >= 0 (empty documents
 * allowed), w[N] with N = sum(doc_len) <= 2^31-1 and 0 <= w[i] < V.  The
 * initial state is z_i = floor(K r_i / 2^32) from the init stream, the counts of
 * that z, then theta and phi drawn from their conditionals with sweep index 0.
 * Errors: INVALID_ARG for bad sizes/values (nothing is allocated), HIP. */
int augur_lda_create(const augur_lda_config* cfg, const int32_t* doc_len, const int32_t* w,
                     augur_lda** out);
void augur_lda_destroy(augur_lda* h); /* NULL is a no-op */

/* n_sweeps Gibbs sweeps (Sect. 4.2), each in the order: draw every z_i from
 * p(k) ~ theta_d[k] phi[w_i][k]; count n_dk, n_wk; theta_d ~ Dirichlet(alpha +
 * n_dk[d]); phi_k ~ Dirichlet(beta + n_wk[.][k]).  Asynchronous. */
int augur_lda_sweep(augur_lda* h, int32_t n_sweeps);

/* Extra observed variables, as in the paper's second call of Fig. 3,
 * map(Set("phi"), ...): with AUGUR_OBSERVE_PHI the handle's phi (put there with
 * set_state, e.g. the phi learnt on a training corpus) is data; sweep then draws
 * z, counts n_dk and redraws theta only, and leaves phi and n_wk untouched.
 * loglik's log_marginal_w of such a handle over held-out documents is the log
 * predictive probability sum_i ln sum_k theta_d[k] phi[w_i][k].  mask = 0 turns
 * it off.  The step_x calls are not affected. */
#define AUGUR_OBSERVE_PHI 1u
int augur_lda_set_observed(augur_lda* h, uint32_t mask);

/* After the z step the pair (word table n_wk, phi step) and the pair (document
 * table n_dk, theta step) do not depend on each other (Sect. 4.2: theta and phi
 * are conditionally independent given z).  With overlap on (the default) the
 * first pair runs on a second stream of the library's own (default priority)
 * beside the second; the handle's stream waits for it before the sweep ends.
 * Results are identical either way.  Not to be changed while a sweep is in
 * flight. */
int augur_lda_set_overlap(augur_lda* h, int32_t on);

/* sweep() enqueues about ten kernels per sweep on two streams.  With a stream of the
 * caller's in config.stream the library records that sequence once as a HIP graph
 * (the sweep index comes from a counter in device memory that the graph itself
 * advances) and replays it: the same kernels, the same results, shorter gaps
 * between launches.  On by default when config.stream is not NULL (the default
 * stream cannot be recorded); on = 0 turns it off, on = 1 on again.  The step
 * calls and sweep_profile always launch directly.  Like every call on a handle,
 * sweep must not run while another thread uses the same stream. */
int augur_lda_set_graph(augur_lda* h, int32_t on);

/* The z step (Sect. 4.2) has two forms up to 256 topics, which draw the same bits.  One
 * gives every wave a document and reads every phi row from memory.  The other keeps
 * workgroups resident, one per CU, with the phi rows of the corpus's most frequent
 * words in LDS (as many as fit: about 100 at K = 200), and reads the rows of those
 * words from there; it pays when there are several documents for every wave of
 * the chip.  mode 0 (default): the library chooses by the number of documents;
 * 1: the resident form whenever it is available (K <= 256, at least 8 rows fit);
 * 2: never.  The same switch picks the form of loglik's token kernel, which has
 * the same two.  Not to be changed while a sweep is in flight. */
int augur_lda_set_z_cache(augur_lda* h, int32_t mode);

/* Which kernels build the word table n_wk during sweeps and count steps (count_accumulate,
 * Sect. 4.2; both give the same table).  The gathering kernel reads z through the word-major
 * permutation; the staged form (up to 256 topics, after a z step) moves the one-byte copy of z
 * into word-major order in two passes through LDS that read and write whole cache lines, which
 * pays when the copy is larger than the caches and the word table has the chip to itself (beside
 * the theta step of an overlapped sweep the gathering kernel hides better).  mode 0 (default):
 * the library chooses (staged from 16M tokens on, when nothing runs beside it); 1: the staged
 * form whenever it is available; 2: never.  Not to be changed
 * while a sweep is in flight. */
int augur_lda_set_word_table(augur_lda* h, int32_t mode);

/* Same as sweep, but records events on the handle's stream around the steps and
 * returns the summed device time over the n_sweeps, in ms: ms[0] sample_z;
 * ms[1] count_accumulate (with overlap on: the document table only; the word
 * table and the phi step run beside ms[1] and ms[2]); ms[2] resample theta;
 * ms[3] resample phi (with overlap on: the wait for the second stream after the
 * theta step); ms[4] whole sweep
 * (first event to last).  Events are recorded without host waits; the call
 * synchronises once at the end.  n_sweeps <= 4096. */
#define AUGUR_LDA_NSTEPS 5
int augur_lda_sweep_profile(augur_lda* h, int32_t n_sweeps, double* ms);

/* Steps of one sweep, for lock-step checking.  Each uses sweep index
 * (completed sweeps + 1); step_finish adds one to the completed count. */
int augur_lda_step_sample_z(augur_lda* h);
int augur_lda_step_count(augur_lda* h);
int augur_lda_step_resample_theta(augur_lda* h);
int augur_lda_step_resample_phi(augur_lda* h);
int augur_lda_step_finish(augur_lda* h);

/* log_joint = ln p(phi, theta, z, w) of Fig. 1's program; log_marginal_w =
 * sum_i ln sum_k theta_d[k] phi[w_i][k].  Log-space sums (Sect. 4.1), fp64.
 * Either output may be NULL.  Returns AUGUR_ERR_DEGENERATE once (with the
 * outputs still written) if a sweep since the last report met a token whose
 * conditional had zero or non-finite mass. */
int augur_lda_loglik(augur_lda* h, double* log_joint, double* log_marginal_w);

/* The state is the paper's `sig` bundle (Sect. 2.2, Fig. 3): the caller passes
 * initial values of the latent variables in it and reads the results back from
 * it.  get_state copies z int32[N], theta float[D][K], phi float[V][K] and the
 * number of completed sweeps out; set_state copies them in. */
int augur_lda_get_state(augur_lda* h, int32_t* z, float* theta, float* phi, int64_t* sweep);
/* The same for a handle created with AUGUR_STATE_F64: theta double[D][K], phi double[V][K].
 * Each pair serves its own kind of handle; asked for theta or phi of the other kind it
 * returns AUGUR_ERR_INVALID_ARG (z and sweep alone are served by either). */
int augur_lda_get_state_f64(augur_lda* h, int32_t* z, double* theta, double* phi, int64_t* sweep);
int augur_lda_set_state_f64(augur_lda* h, const int32_t* z, const double* theta, const double* phi,
                            int64_t sweep);
/* Any of z/theta/phi may be NULL (left as is); sweep < 0 leaves the index.
 * Setting z recomputes the counts.  z[i] must lie in [0,K). */
int augur_lda_set_state(augur_lda* h, const int32_t* z, const float* theta, const float* phi,
                        int64_t sweep);
int augur_lda_get_counts(augur_lda* h, int32_t* n_dk, int32_t* n_wk);
/* Number of tokens, over all sweeps so far, whose conditional was degenerate. */
int augur_lda_get_degenerate(augur_lda* h, int64_t* count);
int augur_lda_sync(augur_lda* h);

/* augur_lda_loglik for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  It needs
 * no handle: the caller passes the corpus and the state as DEVICE arrays and gets
 * the same two numbers back in DEVICE memory, out[0] = log joint, out[1] = log
 * marginal of w (see augur_lda_loglik).  The call allocates and frees nothing,
 * on the device or through any library, and does not synchronise: its kernels
 * are enqueued on args->stream and `out` is valid once they have run.
 *
 * Its working memory (the document offsets it forms from doc_len, the block
 * partials of its sums, a logarithm table: about 8.1 MiB) is a static device
 * array of the library, one per GPU, held until the process ends.  That fixes
 * the largest input: D <= 1048576 documents (AUGUR_ERR_INVALID_ARG beyond, as
 * for K > 1024, V * ld > 2^30, ld < K or ld not a multiple of 4, NULL or
 * misaligned pointers); the handle-based call has no such limit.  All calls on one
 * GPU share the array: calls that may overlap on a GPU (different streams,
 * different threads) race and must be ordered by the caller.  No call depends on
 * what an earlier one left in the array.
 *
 * Layout: doc_len int32[D]; w, z int32[N], N = sum of doc_len <= 2^31-1,
 * doc-major; theta float[D][ld], phi float[V][ld] with row stride ld >= K, a
 * multiple of 4 (rows 16-byte aligned); columns K..ld-1 may hold anything.
 * Not validated (validation would need a host wait): a negative doc_len counts
 * as 0, word ids and topics outside their tables are clamped into them; w and z
 * must hold at least N entries.  Every document is walked by one wave, so a
 * corpus of very few, very long documents is served faster by a handle. */
typedef struct {
  int32_t D, V, K;
  int32_t ld;             /* row stride of theta and phi, in elements */
  float alpha, beta;      /* > 0, finite */
  const int32_t* doc_len; /* device */
  const int32_t* w;       /* device */
  const int32_t* z;       /* device */
  const float* theta;     /* device, 16-byte aligned */
  const float* phi;       /* device, 16-byte aligned */
  int32_t device;         /* HIP device ordinal */
  void* stream;           /* hipStream_t or NULL */
} augur_lda_static_args;
int augur_lda_loglik_static(const augur_lda_static_args* args, double* out /* device double[2] */);

/* ------------------------------------------------------------- measurement
 * Not part of the sampler: the ceilings its kernels are held against, measured on
 * the same device in the same run (the measurement protocol asks for the
 * achievable bandwidths beside the achieved ones).  Both calls time with events on
 * the stream they are given and synchronise it.
 *
 * probe_gather: the memory side of the z step of Sect. 4.2 alone: the handle's own
 * word-id stream and phi table, walked and loaded exactly as the z kernel does
 * it, with no random numbers, arithmetic or stores; one warm-up pass, then reps
 * timed passes; *ms_per_pass is their mean duration.  State is not changed.
 *
 * probe_stream_copy: reps plain device copies of `bytes` bytes (a multiple of 16;
 * src and dst are 16-byte aligned DEVICE buffers of that size, owned by the
 * caller); *ms_per_copy is the mean duration of one copy, which reads and writes
 * `bytes` each.  Also the launch of known size that scales a profiler's byte
 * counters. */
int augur_lda_probe_gather(augur_lda* h, int32_t reps, double* ms_per_pass);
int augur_probe_stream_copy(const void* src, void* dst, int64_t bytes, int32_t reps, void* stream,
                            double* ms_per_copy);

/* ------------------------------------------------ Gaussian mixture (supplement)
 * pi ~ Dirichlet(alpha 1_K), mu_k ~ N(0, prior_sd^2 I), z_i ~ Categorical(pi),
 * x_i ~ N(mu_{z_i}, v_{z_i} I); x observed.  Known variance (var_shape = 0):
 * v_k = sigma^2 for every k.  Unknown variances (var_shape > 0, the model of
 * the supplement's Gaussian-mixture listing, whose per-component scale is read
 * as a variance): var_k ~ InverseGamma(var_shape, var_scale), v_k = var_k, and
 * sigma is ignored.  Layout: x float[N][dim], z int32[N], pi float[K],
 * mu float[K][dim], var float[K], n_k int32[K], s_k double[K][dim]. */
typedef struct augur_gmm augur_gmm;

typedef struct {
  int64_t N;
  int32_t dim, K;
  float alpha, prior_sd; /* > 0, finite */
  float sigma;           /* known variance: > 0, finite */
  float var_shape;       /* 0: known variance; > 0: inverse-Gamma shape a0 */
  float var_scale;       /* inverse-Gamma scale b0 (> 0 when var_shape > 0) */
  uint64_t seed;
  int32_t device;
  void* stream;
  uint32_t flags;
} augur_gmm_config;

int augur_gmm_create(const augur_gmm_config* cfg, const float* x, augur_gmm** out);
void augur_gmm_destroy(augur_gmm* h);
/* One sweep: z_i from p(k) ~ pi_k v_k^(-dim/2) exp(-|x_i - mu_k|^2 / (2 v_k));
 * n_k and s_k = sum of x_i with z_i = k; pi ~ Dirichlet(alpha + n); mu_kj ~
 * Normal with precision 1/prior_sd^2 + n_k/v_k and mean (s_kj/v_k)/precision;
 * with unknown variances then var_k ~ InverseGamma(var_shape + n_k dim / 2,
 * var_scale + SS_k / 2), SS_k = sum over z_i = k of |x_i - mu_k|^2 at the new
 * mean.  The initial state (sweep index 0) has var_k = var_scale / var_shape
 * before its first draw. */
int augur_gmm_sweep(augur_gmm* h, int32_t n_sweeps);
/* As augur_lda_set_graph: sweep() replays a recorded HIP graph when the handle has a
 * stream of the caller's (the default), or launches directly (on = 0). */
int augur_gmm_set_graph(augur_gmm* h, int32_t on);
/* Same as sweep, with events on the handle's stream around the steps; summed device time over
 * the n_sweeps in ms: ms[0] z step, ms[1] statistics, ms[2] resampling, ms[3] whole sweep.
 * Synchronises once at the end.  n_sweeps <= 4096. */
#define AUGUR_GMM_NSTEPS 4
int augur_gmm_sweep_profile(augur_gmm* h, int32_t n_sweeps, double* ms);
int augur_gmm_step_sample_z(augur_gmm* h);
int augur_gmm_step_stats(augur_gmm* h);
int augur_gmm_step_resample(augur_gmm* h);
int augur_gmm_step_finish(augur_gmm* h);
int augur_gmm_loglik(augur_gmm* h, double* log_joint);
/* The mixture's `sig` bundle (Sect. 2.2, Fig. 3), as for LDA. */
int augur_gmm_get_state(augur_gmm* h, int32_t* z, float* pi, float* mu, int64_t* sweep);
int augur_gmm_set_state(augur_gmm* h, const int32_t* z, const float* pi, const float* mu,
                        int64_t sweep);
/* Unknown variances only (AUGUR_ERR_INVALID_ARG otherwise): var float[K], host or
 * device as the handle's flags say; set_var requires positive finite values. */
int augur_gmm_get_var(augur_gmm* h, float* var);
int augur_gmm_set_var(augur_gmm* h, const float* var);
int augur_gmm_get_stats(augur_gmm* h, int32_t* n_k, double* s_k);
int augur_gmm_get_degenerate(augur_gmm* h, int64_t* count);
int augur_gmm_sync(augur_gmm* h);

/* ----------------------- Metropolis-Hastings on the multivariate regression model
 * Sect. 4.1 and Fig. "regression": w_k ~ N(0, prior_sd^2) (k < K),
 * b ~ N(0, prior_sd^2), tau ~ InverseGamma(tau_shape, tau_scale),
 * x_nk ~ Uniform(x_lo, x_hi), y_n ~ N(x_n . w + b, tau), tau a variance; x and y
 * observed.  ln f = ln of the product of these densities: the per-datum terms
 * are evaluated in parallel and summed (fp64).  The sampler is the random walk
 * of the supplement's "Multivariate Regression" experiment: step t proposes
 * theta' = theta + step * n_t (n_t standard normal, all parameters at once) and
 * accepts iff ln u_t < ln f(theta') - ln f(theta); a proposal with tau' <= 0 has
 * density zero and is refused.  theta = (w_0 .. w_{K-1}, b, tau): K + 2 doubles.
 * Layout: x float[N][K], y float[N]; array pointers are host or device as
 * flags say, scalars always host. */
typedef struct augur_mhreg augur_mhreg;

typedef struct {
  int64_t N;          /* 1 .. 2^31-1 */
  int32_t K;          /* 1 .. 64 predictors */
  float prior_sd;     /* > 0 */
  float tau_shape;    /* > 0 */
  float tau_scale;    /* > 0 */
  float x_lo, x_hi;   /* x_lo < x_hi; every x must lie in [x_lo, x_hi] */
  float step;         /* > 0: standard deviation of the random walk */
  uint64_t seed;
  int32_t device;
  void* stream;
  uint32_t flags;     /* AUGUR_PTRS_DEVICE */
} augur_mhreg_config;

/* Copies x and y.  theta0 may be NULL (w = 0, b = 0, tau = 1); otherwise finite
 * with tau > 0.  AUGUR_ERR_INVALID_ARG if a value of x is outside its support or
 * x or y holds a non-finite value. */
int augur_mhreg_create(const augur_mhreg_config* cfg, const float* x, const float* y,
                       const double* theta0, augur_mhreg** out);
void augur_mhreg_destroy(augur_mhreg* h);
/* n_steps steps, asynchronous on the handle's stream unless a host trace is
 * asked for.  trace: NULL, or n_steps rows of K + 3 doubles (theta, then ln f)
 * after each step. */
int augur_mhreg_run(augur_mhreg* h, int64_t n_steps, double* trace);
/* Any output may be NULL.  accepted counts accepted proposals since create. */
int augur_mhreg_get_state(augur_mhreg* h, double* theta, double* logf, int64_t* step_index,
                          int64_t* accepted);
/* theta NULL: left as is (else ln f is re-evaluated); step_index < 0: left as is. */
int augur_mhreg_set_state(augur_mhreg* h, const double* theta, int64_t step_index);
/* 0: automatic; 1: all steps of a run in one launch of one workgroup (N <= 65536);
 * 2: one launch per step over many workgroups.  Same results either way. */
int augur_mhreg_set_schedule(augur_mhreg* h, int32_t schedule);
int augur_mhreg_sync(augur_mhreg* h);

#ifdef __cplusplus
}
#endif
#endif /* AUGUR_H */

/*
 * regtopk.h -- C ABI of the RegTop-k per-round hot path for AMD MI355X (gfx950).
 *
 * One context simulates N workers of a parameter-server round on one GPU.
 * A call of regtopk_step() runs, for every worker n (rows of a [N,d] batch):
 *
 *   1. error-feedback accumulation  a_n = eps_n + g_n
 *        (paper: Algorithm 1 line 3 / Algorithm 2, "accumulated gradient");
 *   2. the posterior-regularised selection score
 *        score_j = |a_j| * tanh(|1 + Delta_j| / mu)   for j sent in the previous round,
 *        score_j = |a_j|                              otherwise (constant C = 1),
 *        Delta_j = (gprev_j - w a^{t-1}_j) / (w a^t_j),  w = omega_n (1/N unless set)
 *        (paper: definition of the posterior distortion Delta in the subsection
 *        "Characterizing the Likelihood"; likelihood
 *        with tanh in the section "RegTop-k Algorithm"; Algorithm 2 mask line);
 *   3. exact Top_k of the score, exactly k entries, the lower index winning
 *        among equal scores (paper: Top_k selector of the subsection "Top-k:
 *        Classical Sparsification Scheme");
 *   4. compaction of the k (index, value) pairs, value = a_j, and the error
 *        update eps_n <- a_n - s_n (.) a_n (paper: last three lines of
 *        Algorithm 2);
 *   5. the server's aggregation g = sum_n omega_n * ghat_n into a dense vector
 *        (paper: aggregation equation after Algorithm 1; omega_n = 1/N, computed
 *        as 1.0f/(float)N, unless regtopk_set_weights gave other weights).
 *
 * Round 0 has no previous mask and is plain Top-k (first block of Algorithm 2).
 * mu == 0 switches the regulariser off in every round (Algorithm 1).
 *
 * Arithmetic is IEEE binary32 without fused multiply-add, in this order:
 *   a = eps + g;  num = gprev - w*aprev;  den = w*a;  if den == 0: f = 1, else
 *   D = num/den;  r = |1 + D|;  x = r/mu;  f = tanh(x) correctly rounded to
 *   binary32 (f = 1 when x is NaN);  score = |a| * f;
 *   agg_j = (((+0 + w*v_n1) + w*v_n2) + ...) over the workers n1 < n2 < ...
 *   that selected j.
 *
 * All pointers named *_dev are device memory of the GPU that was current when
 * the context was created; the library never dereferences them on the host.
 * Every call returns 0 on success or a negative REGTOPK_* code; nothing throws
 * or aborts across this boundary.  regtopk_last_error() describes the last
 * failure of the calling thread.
 *
 * A context may be driven from one thread / one stream at a time.
 */
#ifndef REGTOPK_H
#define REGTOPK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define REGTOPK_OK            0
#define REGTOPK_INVALID_ARG  -1   /* bad size, null pointer, misaligned pointer, mu < 0 or NaN */
#define REGTOPK_BAD_STATE    -2   /* e.g. set_state with indices that are not ascending; a round that was given up */
#define REGTOPK_HIP_ERROR    -3   /* a HIP call or kernel launch failed */
#define REGTOPK_NO_MEMORY    -4   /* arena too small / allocation failed */

typedef struct regtopk_ctx regtopk_ctx;

/* Result of one round.  Device pointers into the context's arena; they stay
 * valid (and unchanged) until the next regtopk_step/reset/set_state/destroy on
 * the same context.  Contents are defined once the stream has been
 * synchronised. */
typedef struct {
  const int32_t* idx;  /* [N,k] selected indices of each worker, ascending          */
  const float*   val;  /* [N,k] val[n,i] = a_n[idx[n,i]] (un-weighted, as sent)     */
  const float*   agg;  /* [d]   aggregate g^t; +0 where no worker selected an entry */
} regtopk_result;

/* Per-worker diagnostics of the last round (host memory). */
typedef struct {
  uint32_t tau_lo_bits;   /* speculative lower bound on the k-th score used in pass 1 (bit pattern; 0xFFFFFFFF = none) */
  uint32_t n_candidates;  /* entries handed to the exact selection                   */
  uint32_t used_dense;    /* 1 if the dense (non-speculative) selection had to run   */
  uint32_t tau_bits;      /* bit pattern of the k-th largest score                   */
  uint32_t n_greater;     /* entries with score > tau                                */
  uint32_t n_ties_taken;  /* entries with score == tau that were selected            */
  uint32_t n_ties_total;  /* candidates with score == tau                            */
  uint32_t overflow;      /* 1 if the speculative candidate buffer overflowed        */
  uint32_t used_window;   /* 1 if the k-th score was found from the short boundary list */
  uint32_t n_boundary;    /* candidates whose score fell into the window around the expected k-th score */
  uint32_t n_valid;       /* candidates with score >= the speculative bound           */
  uint32_t window_half;   /* half width of that window in binary32 bit patterns (0 = none) */
} regtopk_worker_stats;

/* Bytes of device memory a context needs for (N, d, k): the state of Algorithm 2
 * for N workers (eps, previous lists), the outputs and the kernels' work areas.
 * 0 on invalid sizes. */
size_t regtopk_workspace_bytes(int32_t N, int64_t d, int64_t k);

/* Creates a context: eps = 0, round counter 0, empty previous mask
 * (initialisation line of Algorithm 2).
 *   1 <= N <= 65535 workers, 1 <= d < 2^31 entries per worker, 1 <= k <= d,
 *   mu >= 0 and finite (REGTOPK_INVALID_ARG otherwise).
 * regtopk_create allocates its arena with hipMalloc on the current device and
 * frees it in regtopk_destroy.  regtopk_create_in uses caller-owned device
 * memory instead: arena_dev must be 256-byte aligned, at least
 * regtopk_workspace_bytes(N,d,k) long, and must outlive the context; its
 * contents are overwritten.  Both zero the state (create_in on `stream`, a
 * hipStream_t, NULL = default stream) and wait for that to finish.
 * The context belongs to the device that is current at creation: every later
 * call that enqueues work for it must be made with that device current
 * (REGTOPK_INVALID_ARG otherwise; nothing is enqueued). */
int regtopk_create(regtopk_ctx** out, int32_t N, int64_t d, int64_t k, float mu);
int regtopk_create_in(regtopk_ctx** out, int32_t N, int64_t d, int64_t k, float mu,
                      void* arena_dev, size_t arena_bytes, void* stream);

/* One round (steps 1-5 above) enqueued on `stream`; no host synchronisation.
 *   grads_dev          [N,d] row-major binary32 local gradients g_n^t; read only;
 *                      finite values (otherwise the selection is undefined).
 *   prev_aggregate_dev [d] aggregate of the previous round, g^{t-1} (normally
 *                      the `agg` pointer of the previous result); read only;
 *                      ignored (may be NULL) in round 0 and when mu == 0.
 * Rows are read with 128-bit loads when d is a multiple of 4 and grads_dev is
 * 16-byte aligned, otherwise with scalar loads.
 * When a worker's speculative bound fails, its exact selection runs in a kernel
 * whose blocks synchronise with each other and must all be resident on the GPU
 * together.  The library never lets two such kernels of one process run at the
 * same time on a device (launches of different contexts are chained by an
 * event).  If the blocks still do not become resident together within a bounded
 * wait (another process saturating the same GPU), the kernel gives the round
 * up rather than compute from half-finished phases: the workers concerned are
 * flagged, regtopk_get_stats returns REGTOPK_BAD_STATE, and so does every
 * regtopk_step called after the kernel has run, until regtopk_reset or
 * regtopk_set_state; the lists of that round are undefined. */
int regtopk_step(regtopk_ctx* ctx, const float* grads_dev, const float* prev_aggregate_dev,
                 void* stream, regtopk_result* out);

/* The same round with the local gradients stored as bfloat16 (the upper 16
 * bits of a binary32 pattern; reduced-precision gradient inputs with binary32
 * state).  Each gradient is widened exactly to binary32 and everything else is
 * as in regtopk_step (paper: Algorithm 2; the paper fixes no input precision),
 * so the result equals regtopk_step on the widened values bit for bit, while
 * the sweep reads 10 instead of 12 bytes per entry.  grads_bf16_dev [N,d]
 * row-major, 2-byte aligned; read with 64-bit loads when d is a multiple of 4
 * and the pointer is 8-byte aligned.  Calls with either gradient type may be
 * mixed freely on one context. */
int regtopk_step_bf16(regtopk_ctx* ctx, const uint16_t* grads_bf16_dev, const float* prev_aggregate_dev,
                      void* stream, regtopk_result* out);

/* One round of the idealised "global Top-k" baseline (paper: subsection
 * "Statistical Global Top-k"): a genie reveals abar = sum_n omega_n a_n, the
 * aggregate of the accumulated gradients a_n = eps_n + g_n without
 * sparsification, and every worker keeps the k entries of largest |abar_j|
 * (lower index first among equals), so all N index rows are equal;
 * val[n,i] = a_n[idx[i]], eps_n <- a_n off that mask, agg = sum_n omega_n ghat_n.
 * abar is summed like the aggregate: from +0, + omega_n * a_n in ascending
 * worker order.  Shares the state with regtopk_step (rounds of both kinds may
 * alternate; a following regtopk_step regularises with this round's mask).
 * The round needs a selector over one row of d entries, which lives in
 * regtopk_global_workspace_bytes(d, k) bytes of device memory.  A context made
 * by regtopk_create allocates them with hipMalloc on the first call (freed by
 * regtopk_destroy).  A context made by regtopk_create_in never allocates: the
 * caller hands the memory over once with regtopk_bind_global (256-byte aligned,
 * must outlive the context; its contents are overwritten), otherwise
 * regtopk_step_global returns REGTOPK_BAD_STATE.  out->agg lives in that memory
 * and stays valid until the next regtopk_step_global. */
size_t regtopk_global_workspace_bytes(int64_t d, int64_t k);
int regtopk_bind_global(regtopk_ctx* ctx, void* mem_dev, size_t bytes, void* stream);
int regtopk_step_global(regtopk_ctx* ctx, const float* grads_dev, void* stream, regtopk_result* out);

int regtopk_destroy(regtopk_ctx* ctx);

/* Back to the state after create: eps = 0, round 0, no previous mask (paper:
 * initialisation line of Algorithm 2).  Enqueued on `stream`. */
int regtopk_reset(regtopk_ctx* ctx, void* stream);

/* Copies the persistent state out / in (device buffers of the caller).  The
 * state is what Algorithm 2 carries from round to round at worker n: the
 * sparsification error eps_n, the previous mask s_n^{t-1} and the accumulated
 * gradient a_n^{t-1} on that mask (as index and value lists), and the round
 * counter:
 *   e_dev [N,d] error eps, pidx_dev [N,k] / pval_dev [N,k] previous round's
 *   selected indices (ascending) and values, *t_host the round counter.
 * Before round 1 the previous lists are empty and pidx/pval are not written /
 * read.  Any of the output pointers of get_state may be NULL to skip it.
 * set_state enqueues a check that every row of pidx is strictly ascending and
 * within [0,d); a violation is reported by the next regtopk_get_stats
 * (REGTOPK_BAD_STATE) and the following rounds are undefined. */
int regtopk_get_state(regtopk_ctx* ctx, float* e_dev, int32_t* pidx_dev, float* pval_dev,
                      int64_t* t_host, void* stream);
int regtopk_set_state(regtopk_ctx* ctx, const float* e_dev, const int32_t* pidx_dev,
                      const float* pval_dev, int64_t t, void* stream);

/* Synchronises `stream` and copies the per-worker diagnostics of the last
 * round into stats_host[0..N).  Returns REGTOPK_BAD_STATE if a device-side
 * consistency check failed (selected count != k, bad set_state input). */
int regtopk_get_stats(regtopk_ctx* ctx, regtopk_worker_stats* stats_host, void* stream);

/* Aggregation weights omega_n of the N workers (paper: weighted average
 * g = sum_n omega_n g_n of the introduction; omega_n in the distortion line of
 * Algorithm 2).  weights_host[0..N) is HOST memory, finite values; worker n
 * uses omega_n both in its posterior distortion and in its term of the
 * aggregate, from the next regtopk_step on.  Copies synchronously (waits for
 * `stream`).  Weights survive regtopk_reset and set_state. */
int regtopk_set_weights(regtopk_ctx* ctx, const float* weights_host, void* stream);

/* Entries kept per worker (paper: Algorithm 2 is stated at worker n, and its
 * selector Top_k takes k as a parameter of that worker's sparsifier; the
 * paper's experiments give every worker the same k).  k_host[0..N) is HOST
 * memory, 1 <= k_host[n] <= k of regtopk_create (REGTOPK_INVALID_ARG
 * otherwise).  From the next round on worker n selects exactly k_host[n]
 * entries.  Layout: the lists stay [N,k] row-major; row n holds its k_host[n]
 * pairs first (indices ascending) and (-1, 0.0f) in the remaining positions;
 * the same holds for pidx/pval of get_state / set_state.  Copies synchronously
 * (waits for `stream`); survives regtopk_reset and set_state; the bounds
 * carried over from earlier rounds are dropped.  regtopk_step_global shares
 * one mask of k entries among all workers and returns REGTOPK_BAD_STATE while
 * some worker's k differs from k. */
int regtopk_set_worker_k(regtopk_ctx* ctx, const int64_t* k_host, void* stream);

/* Agreement of the workers' masks in the last completed round (paper: appendix
 * subsection "Comparing Sparsification Masks"): counts_dev[c], c = 0..N, device
 * memory of N+1 int64 (8-byte aligned), receives the number of entries j in
 * [0,d) that exactly c workers selected; all d entries fall into c = 0 before
 * the first round.  Enqueued on `stream`. */
int regtopk_mask_overlap(regtopk_ctx* ctx, int64_t* counts_dev, void* stream);

/* regtopk_mask_overlap for callers that must not allocate or touch the context's
 * scratch areas while they run: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same inputs, same result in
 * counts_dev, but the per-block partial counts go to a 4 MiB array that is
 * part of the library image on every GPU (no hipMalloc, hipFree or other
 * allocating call is made, and the context's arena is only read).  Limits:
 * N <= 1023 workers (REGTOPK_INVALID_ARG otherwise, with a message that says
 * so), and the context's device must be current.  All calls on one GPU share
 * that array: calls that overlap in time on one GPU (two streams) race and
 * give undefined counts; calls on one stream, or ordered by events, are fine. */
int regtopk_mask_overlap_static(regtopk_ctx* ctx, int64_t* counts_dev, void* stream);

/* Model update of distributed SGD (paper: introduction, theta^{t+1} = theta^t -
 * eta^t g^t): theta_dev[j] <- theta_dev[j] - eta * g_dev[j] for j in [0,d),
 * binary32, the product rounded before the subtraction (no fused multiply-add).
 * Device buffers of d floats that must not overlap; g_dev is read only.
 * Enqueued on `stream`.  No context is needed. */
int regtopk_sgd_update(float* theta_dev, const float* g_dev, float eta, int64_t d, void* stream);

/* Options (tuning and test hooks). */
#define REGTOPK_OPT_FORCE_DENSE   1  /* value != 0: never speculate, always run the dense selection */
#define REGTOPK_OPT_CAND_TARGET   2  /* speculative pass aims at value*k candidates (1 < value <= 3; default 1.25) */
#define REGTOPK_OPT_PROFILE       3  /* 1: HIP events on the step's stream around the stages of every step (an
                                        event recorded between two kernels keeps the second from starting back
                                        to back, about 4 us; the two events of the dense sweep kernel travel
                                        with its own dispatch instead, the other three are recorded: a profiled
                                        round is some 10 us longer);  2: only the two events of the dense sweep
                                        kernel (about 3 us);  0 switches it off.  Every setting resets the
                                        recorded rounds. */
/* Score variants (paper: remark on sub-linear scaling in the appendix, score
 * |a|^y * u(|1 + Delta|) with y <= 1; sentence after the tanh likelihood that
 * other cumulative functions u_mu are admissible).  Defaults are Algorithm 2.
 * They take effect from the next round; the bounds carried over from earlier
 * rounds are dropped. */
#define REGTOPK_OPT_PRIOR_ROOTS   4  /* value m in {0,1,2,3}: prior |a|^y with y = 2^-m, evaluated as m correctly
                                        rounded binary32 square roots of |a| */
#define REGTOPK_OPT_PRIOR_EXPONENT 6 /* value y in (0, 1]: prior |a|^y with a general binary32 exponent, defined as
                                        the correctly rounded binary32 value of the real power (y = 1: Algorithm
                                        2).  Replaces a setting of REGTOPK_OPT_PRIOR_ROOTS and is replaced by one. */
#define REGTOPK_OPT_LIKELIHOOD    5  /* 0: tanh(|1+Delta|/mu);  1: min(|1+Delta|/mu, 1), the cumulative function
                                        of an innovation uniform on [0, mu];  2: erf(|1+Delta|/mu) correctly
                                        rounded to binary32, the cumulative function of a Gaussian innovation of
                                        standard deviation mu/sqrt(2) with the constants dropped as the paper
                                        drops them for tanh (1/2 (1 + erf) -> erf) */
int regtopk_set_option(regtopk_ctx* ctx, int option, double value);

/* Stage times of the last n <= min(max_rounds, 64) profiled rounds, oldest
 * first, in milliseconds: out_host[4*i + 0] the dense sweep kernel (accumulate + emit),
 * + 1 scoring and selection, + 2 compaction, error update and aggregation,
 * + 3 the whole round (the last three are 0 for rounds recorded at profile
 * level 2).  Waits for the recorded events. */
int regtopk_get_timings(regtopk_ctx* ctx, float* out_host, int32_t max_rounds, int32_t* n_rounds);

/* Text of the last error on the calling thread ("" if none). */
const char* regtopk_last_error(void);

/* ------------------------------------------------------------------------
 * Test and profiling hooks.  Not part of the method's interface: the tests use
 * the first three to compare the tanh, erf and power steps with the oracle's,
 * the benchmark launches the last once as the dispatch of known size against which hardware traffic
 * counters are scaled.
 * ------------------------------------------------------------------------ */

/* The tanh step alone: y[i] = tanh(x[i]) correctly rounded to binary32 for
 * x[i] >= 0 (device buffers of n floats).  Test hook for the exhaustive
 * comparison of that step.  regtopk_erf_f32: the same for the erf step of
 * REGTOPK_OPT_LIKELIHOOD 2. */
int regtopk_tanh_f32(const float* x_dev, float* y_dev, int64_t n, void* stream);
int regtopk_erf_f32(const float* x_dev, float* y_dev, int64_t n, void* stream);
/* out[i] = x[i]^y correctly rounded to binary32 for x[i] >= 0 and 0 < y < 1: the prior of
 * REGTOPK_OPT_PRIOR_EXPONENT alone. */
int regtopk_pow_f32(const float* x_dev, float y, float* out_dev, int64_t n, void* stream);

/* Plain copy dst[i] = src[i] of n floats by one kernel (n*4 bytes read, n*4
 * written): the known-size reference dispatch against which hardware traffic
 * counters are scaled when profiling. */
int regtopk_copy_f32(float* dst_dev, const float* src_dev, int64_t n, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* REGTOPK_H */

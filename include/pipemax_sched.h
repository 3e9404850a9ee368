/*
 * pipemax_sched.h -- C ABI of the prefetch-aware decode scheduler (host code, no GPU work of its own).
 *
 * The scheduler is the control plane of PipeMax Sec. 3.3: it predicts the time of the decode step
 * that is about to run (Sec. 3.3.1, Eq. 2), turns it into the amount of KV that can be prefetched
 * behind that step (Sec. 3.3.2, Eq. 6) and chooses which host-resident requests of the next batch
 * to prefetch (App. A.4, Alg. 1 and Alg. 2).  It keeps its own mirror of the stage's bookkeeping
 * (lengths, residency, free GPU pages) and drives a `pipemax_stage_t` through the public calls of
 * pipemax.h only.
 *
 * Conventions: as in pipemax.h.  All pointers are host pointers owned by the caller, read or written
 * before the call returns, except hidden_in / hidden_out of pipemax_sched_iterate (device).
 * Lengths are in cached tokens; times in seconds; every order is total (by length, ties by index),
 * so every decision is reproducible.  One caller thread per scheduler.
 *
 * What the paper leaves open and this library fixes (documented, not derived):
 *  - an exchange of Alg. 2 trades ONE selected request against TWO unselected shorter ones (the pair
 *    with the largest total length that fits the budget) or TWO selected ones against ONE unselected
 *    longer one (the longest that fits), and is applied only if the modelled time of the selection
 *    moves closer to the target gap;
 *  - the steady flag latches once the budgets of the last `window` iterations satisfy
 *    (max - min) / mean < steady_rel_range;
 *  - candidates of an iteration are the host-resident requests of the batch being updated (D_j);
 *    requests of the overwritten batch (D_k) are released oldest-resident first and only as many
 *    as the prefetch and the next step's new pages need.
 */
#ifndef PIPEMAX_SCHED_H
#define PIPEMAX_SCHED_H

#include "pipemax.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pipemax_sched pipemax_sched_t;   /* opaque */

typedef struct {
  double  alpha_s;              /* Eq. 2: seconds per request of the batch                         */
  double  beta_s;               /* Eq. 2: seconds per cached token of the batch                    */
  double  delta_s;              /* Eq. 2: constant seconds per step                                */
  double  link_tokens_per_s;    /* B of Eq. 6 in tokens/s: bytes/s over the stage's KV bytes/token */
  double  steady_rel_range;     /* steady when (max-min)/mean of the window is below this          */
  double  refine_tol_s;         /* Alg. 2 stops when |modelled time - gap| <= this                 */
  int64_t static_budget_tokens; /* > 0: replaces Eq. 6 by this constant (static prefetching)       */
  int32_t window;               /* w: iterations in the sliding window (>= 1)                      */
  int32_t max_refine_steps;     /* cap on the exchanges of Alg. 2 (>= 0)                           */
  int32_t n_batches;            /* n: pipeline depth = number of decode batches (>= 1)             */
  int32_t page_tokens;          /* tokens per KV page (16)                                         */
} pipemax_sched_config_t;

/* What one iteration of Alg. 1 decided.                                                           */
typedef struct {
  int32_t exec_batch, n_exec;           /* i_t and the size of the executed batch                  */
  int32_t prefetch_batch, n_prefetch;   /* j_t and |P_t|                                           */
  int32_t evict_batch, n_evict;         /* k_t and the number of its requests released             */
  int32_t steady;                       /* phase flag after this iteration's budget                */
  int32_t n_exchanges;                  /* exchanges Alg. 2 applied                                */
  int64_t budget_tokens;                /* prefetch budget of this iteration                       */
  int64_t prefetch_tokens;              /* total prefix length of P_t                              */
  int64_t gpu_pages_free;               /* free GPU pages after the iteration (mirror)             */
  double  t_hat_s;                      /* predicted time of the executed batch                    */
  double  gap_s;                        /* T_hat - T_hat_res of the batch being updated            */
} pipemax_sched_iter_t;

/* Errors: ERR_ARG for a NULL pointer or a field out of the ranges stated above.                   */
int pipemax_sched_create(const pipemax_sched_config_t* cfg, pipemax_sched_t** out);
int pipemax_sched_destroy(pipemax_sched_t* s);

/* Eq. 2: alpha * b + beta * L + delta, evaluated left to right in double precision.               */
double pipemax_sched_predict(const pipemax_sched_t* s, int32_t b, int64_t total_len);
/* Eq. 6 in tokens: floor(link_tokens_per_s * t_hat), or static_budget_tokens if that is > 0.      */
int64_t pipemax_sched_budget(const pipemax_sched_t* s, double t_hat_s);
/* Feeds one budget to the sliding window; returns the (latched) steady flag, 0 or 1.              */
int pipemax_sched_observe(pipemax_sched_t* s, int64_t budget_tokens);

/* Warm-up selection of Alg. 1: shortest first while the cumulative length stays within the
 * budget.  len: n prefix lengths (>= 0).  sel (capacity n) receives the chosen indices in the order
 * they were taken, *n_sel their number.                                                           */
int pipemax_sched_short_first_fill(const int32_t* len, int32_t n, int64_t budget, int32_t* sel,
                                   int32_t* n_sel);
/* Greedy initialisation of Alg. 2: longest first, every request that still fits is taken.         */
int pipemax_sched_greedy_fill(const int32_t* len, int32_t n, int64_t budget, int32_t* sel,
                              int32_t* n_sel);
/* Local refinement of Alg. 2 starting from sel[0..*n_sel) (distinct indices, total length within
 * the budget; ERR_ARG otherwise).  sel has capacity n and is updated in place: an exchange removes
 * its request(s) and appends the replacement(s).  *n_exchanges (may be NULL) receives the number of
 * exchanges applied.  gap_s is the target of the modelled time alpha*|P| + beta*sum(len).         */
int pipemax_sched_refine(const pipemax_sched_t* s, const int32_t* len, int32_t n, int64_t budget,
                         double gap_s, int32_t* sel, int32_t* n_sel, int32_t* n_exchanges);

/* Initial partition (Sec. 3.3.2): n requests into n_batches batches whose sizes differ by at most
 * one, total lengths balanced by dealing the requests longest first in serpentine order.
 * batch_of (capacity n) receives the batch of every request.                                      */
int pipemax_sched_partition(const int32_t* len, int32_t n, int32_t n_batches, int32_t* batch_of);

/* The mirror.  set_batch declares the requests of batch `mb` (prefix lengths and 0/1 residency;
 * replaces an earlier declaration); set_gpu_pages_free the free pages of the GPU pool.  attach
 * fills both from a stage whose micro-batches are defined (cfg.n_batches must equal the stage's
 * number of micro-batches; sequences with a prefetch in flight count as resident).                */
int pipemax_sched_set_batch(pipemax_sched_t* s, int32_t mb, int32_t n, const int32_t* len,
                            const int32_t* resident);
int pipemax_sched_set_gpu_pages_free(pipemax_sched_t* s, int64_t pages);
int pipemax_sched_attach(pipemax_sched_t* s, pipemax_stage_t* stage);

/* One iteration of Alg. 1 on the mirror only: the executed batch is every resident request of
 * D_i (each grows by one token and takes a new page when its length is a multiple of the page
 * size); P_t is chosen among the host-resident requests of D_j by the warm-up or the steady
 * policy; requests of D_k are released until P_t and the new pages of the next step fit; if they
 * still do not, requests are dropped from the end of P_t.  exec_ids / prefetch_ids / evict_ids
 * (each NULL or with room for the batch's request count) receive the index lists.
 * Errors: ERR_ARG; ERR_STATE if a batch is undeclared or the executed batch's new pages do not
 * fit (the mirror is unchanged).                                                                  */
int pipemax_sched_plan(pipemax_sched_t* s, int64_t t, pipemax_sched_iter_t* out, int32_t* exec_ids,
                       int32_t* prefetch_ids, int32_t* evict_ids);

/* The same iteration applied to the attached stage: pipemax_evict_kv on the released requests of
 * D_k, pipemax_prefetch_kv of P_t into D_j, then pipemax_decode_step_seqs on D_i (rows in ascending
 * request index; hidden_in / hidden_out are device pointers with room for max_seqs_per_mb rows, of
 * which the first n_exec are used).  None of the three blocks; the transfers are arranged first so
 * that their copies start when the previous step ends, not after this one has been enqueued.
 * Afterwards the mirror's free
 * page count is checked against the stage's (ERR_STATE if they differ).  Other errors: those of
 * the stage calls, passed through; the mirror is then put back to its state before the call, and if the
 * failing call was not the first of the three the stage has moved on without it: attach again.     */
int pipemax_sched_iterate(pipemax_sched_t* s, pipemax_stage_t* stage, int64_t t, const void* hidden_in,
                          void* hidden_out, void* hip_stream, pipemax_sched_iter_t* out,
                          int32_t* exec_ids, int32_t* prefetch_ids, int32_t* evict_ids);

#ifdef __cplusplus
}
#endif
#endif

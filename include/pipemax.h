/*
 * pipemax.h -- C ABI of the MI355X (gfx950) stage-decode library.
 *
 * One `pipemax_stage_t` is one pipeline stage: a contiguous slice of Llama-style
 * decoder layers that runs the decode step of ONE active micro-batch at a time
 * (PipeMax Sec. 2.3.2: under pipeline parallelism each GPU executes one decode
 * batch at a time and the KV cache of the other batches sits idle), while the KV
 * caches of the inactive micro-batches live in pinned host memory and are
 * prefetched / written back on side HIP streams (Sec. 3, Sec. 3.3.2 Eq. 3,
 * Sec. 3.4.2).
 *
 * Conventions
 *  - Every call returns a pipemax_status_t (0 = OK, negative = error) and never
 *    throws.  `pipemax_last_error()` gives a thread-local text for the last
 *    failing call.  Argument and state errors are detected on the host before
 *    anything is enqueued and leave the stage unchanged.
 *  - "host" pointers are ordinary host memory owned by the caller and are read or
 *    written before the call returns.  "device" pointers are HIP device memory
 *    owned by the caller (e.g. PyTorch tensors) on the stage's device; the work on
 *    them is enqueued on the stream given to the call and they must stay allocated, and
 *    inputs unmodified, until that work has completed (a NULL stream means the stage's
 *    own compute stream, which is non-blocking: it does not synchronise with the legacy
 *    default stream).
 *  - The stage owns its weights, the GPU page pool, the pinned host page pool, the
 *    staging buffers, two side streams (host->device and device->host) and all
 *    events.  prefetch / decode_step / evict enqueue work and return; ordering
 *    between them is the library's job (events), not the caller's.
 *  - One caller thread per stage.
 *  - Canonical tensor layouts are row-major, in the stage's element type
 *    (float for PIPEMAX_F32, bfloat16 bit patterns for PIPEMAX_BF16).  The
 *    physical layout inside a KV page is internal (it is chosen so that the
 *    attention kernel's loads land directly in matrix-core operand order).
 */
#ifndef PIPEMAX_H
#define PIPEMAX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pipemax_stage pipemax_stage_t;   /* opaque */
typedef struct pipemax_pool  pipemax_pool_t;    /* opaque, host-only page allocator (tests) */

typedef enum {
  PIPEMAX_OK                 =  0,
  PIPEMAX_ERR_ARG            = -1,  /* bad argument / shape / index                       */
  PIPEMAX_ERR_OOM_DEVICE     = -2,  /* hipMalloc failed                                   */
  PIPEMAX_ERR_OOM_HOST       = -3,  /* pinned host allocation failed                      */
  PIPEMAX_ERR_NOT_RESIDENT   = -4,  /* decode_step on a sequence that is host-resident    */
  PIPEMAX_ERR_POOL_EXHAUSTED = -5,  /* not enough free pages (GPU or host pool)           */
  PIPEMAX_ERR_HIP            = -6,  /* a HIP runtime call failed                          */
  PIPEMAX_ERR_STATE          = -7   /* call not valid in this state (e.g. max_ctx reached) */
} pipemax_status_t;

enum { PIPEMAX_F32 = 0, PIPEMAX_BF16 = 1 };

/* which = argument of pipemax_set_weight; canonical shapes ("y = x @ W"):        */
enum {
  PIPEMAX_W_QKV  = 0,  /* [hidden][(Hq + 2 Hkv) * d]  columns: q heads, k heads, v heads */
  PIPEMAX_W_O    = 1,  /* [Hq * d][hidden]                                               */
  PIPEMAX_W_GU   = 2,  /* [hidden][2 * ffn]           columns: gate, then up             */
  PIPEMAX_W_D    = 3,  /* [ffn][hidden]                                                  */
  PIPEMAX_G_ATTN = 4,  /* [hidden]  RMSNorm gain before attention                        */
  PIPEMAX_G_FFN  = 5   /* [hidden]  RMSNorm gain before the FFN                          */
};

/* flags of pipemax_config_t */
enum {
  PIPEMAX_FLAG_FORCE_GENERIC  = 1,  /* use the shape-generic kernels even where the matrix-core
                                       kernels apply (diagnostics)                               */
  PIPEMAX_FLAG_CAPTURE_LAYERS = 2,  /* keep the residual stream after every layer of the last
                                       decode_step (see pipemax_get_layer_outputs)               */
  PIPEMAX_FLAG_TIME_KERNELS   = 4,  /* bracket every kernel class and every transfer with HIP
                                       events and accumulate their durations in the stats        */
  PIPEMAX_FLAG_NO_WRITEBACK   = 8,  /* do not write new K,V through to the host replica
                                       (compute-only timing runs; evict then loses new tokens)   */
  PIPEMAX_FLAG_TIME_ATTN_ONLY = 16, /* with TIME_KERNELS: bracket only the attention kernel, so that
                                       the other launches' event records do not perturb it       */
  PIPEMAX_FLAG_DEVICE_LAYER_MAJOR = 64,  /* GPU page pool laid out [layer][page] instead of block-first: the pages of
                                       the host replica (and a page's bytes on the link) stay block-first, a
                                       prefetch scatters each page run with one strided copy per layer.  An
                                       attention launch then reads one contiguous n_layers-th of the pool
                                       instead of one layer's 64 KiB out of every page.  Not with a transfer
                                       orchestrator attached (ERR_STATE).                                    */
  PIPEMAX_FLAG_STREAM_ORDERED_EVICT = 32  /* order a prefetch after the last reader of the pages it
                                       re-uses with a stream-side event wait instead of the default
                                       host-side wait of the prefetch worker (see pipemax_prefetch_kv) */
};

typedef struct {
  int32_t  n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn;
  float    rope_base, rms_eps;
  int32_t  dtype;            /* PIPEMAX_F32 | PIPEMAX_BF16                                   */
  int32_t  page_tokens;      /* tokens per KV page; must be 16 (Sec. 4.4 uses the same size) */
  int32_t  n_microbatches;   /* n of Eq. 3                                                   */
  int32_t  max_seqs_per_mb;  /* upper bound on b                                             */
  int32_t  max_ctx;          /* upper bound on a sequence's tokens, prompt + generated       */
  uint64_t gpu_kv_bytes;     /* size of the GPU page pool (rounded down to whole pages)      */
  uint64_t host_kv_bytes;    /* size of the pinned host page pool                            */
  int32_t  device;           /* HIP device ordinal                                           */
  uint32_t flags;            /* PIPEMAX_FLAG_*                                               */
  int32_t  host_reserve_tokens;  /* mb_define reserves host pages for min(max_ctx, len + this) tokens
                                    per sequence, consecutively, so that a sequence that grows stays
                                    one contiguous run of host pages (one copy per prefetch); 0 = none */
  int32_t  wb_layers_per_copy;   /* layers per write-back copy: 1 = one device->host copy per layer
                                    right after its QKV projection (the timeline of the paper's
                                    Sec. 3.4.2); 0 = all layers of a step in one copy             */
} pipemax_config_t;

/* kernel classes of the per-class timers (PIPEMAX_FLAG_TIME_KERNELS) */
enum {
  PIPEMAX_K_NORM = 0,     /* residual add + RMSNorm                        (steps a1, a7)  */
  PIPEMAX_K_GEMM_QKV,     /* QKV projection                                (a2)            */
  PIPEMAX_K_ROPE_APPEND,  /* RoPE + KV append + write-back staging         (a3, a4)        */
  PIPEMAX_K_ATTN,         /* GQA paged decode attention, split-K pass      (a5)            */
  PIPEMAX_K_ATTN_MERGE,   /* merge of the split-K partials                 (a5)            */
  PIPEMAX_K_GEMM_O,       /* output projection                             (a6)            */
  PIPEMAX_K_GEMM_GU,      /* gate/up projection                            (a8)            */
  PIPEMAX_K_SWIGLU,       /* SiLU(gate) * up                               (a8)            */
  PIPEMAX_K_GEMM_D,       /* down projection                               (a9)            */
  PIPEMAX_K_MISC,         /* hidden load/store, RoPE table, length advance                 */
  PIPEMAX_N_KCLASS
};

typedef struct {
  uint64_t steps;                 /* decode_step calls completed (enqueued)                  */
  uint64_t tokens;                /* sum of b over those steps                               */
  uint64_t h2d_bytes, h2d_copies; /* KV prefetch traffic (page copies)                       */
  uint64_t d2h_bytes, d2h_copies; /* KV write-back traffic (per-layer staging copies)        */
  uint64_t table_uploads;         /* block-table uploads                                     */
  uint64_t relayout_jobs;         /* per-layer host re-layout jobs finished by the worker    */
  double   host_enqueue_s;        /* host time spent inside decode_step                      */
  double   host_wait_s;           /* host time blocked on the write-back worker              */
  double   h2d_ms;                /* busy time of prefetch copies   (FLAG_TIME_KERNELS)      */
  double   d2h_ms;                /* write-back copies, issue to completion as seen by the   */
                                  /* worker thread that issues them (FLAG_TIME_KERNELS)      */
  double   kernel_ms[PIPEMAX_N_KCLASS];        /* summed kernel durations per class          */
  uint64_t kernel_launches[PIPEMAX_N_KCLASS];
  int32_t  engine;                /* 0 = shape-generic kernels, 1 = matrix-core (bf16) kernels.
                                     The matrix-core kernels serve bf16 stages with head_dim 128,
                                     hidden % 128 == 0, ffn % 64 == 0, at most 16 query heads per KV
                                     head and max_seqs_per_mb <= 256 -- or <= 4096 when hidden,
                                     (n_q_heads + 2 n_kv_heads) * head_dim and 2 * ffn are multiples
                                     of 256; every other stage runs on the generic kernels.        */
  int32_t  gpu_pages_total, gpu_pages_free, host_pages_total, host_pages_free;
  uint64_t page_bytes;
  double   prefetch_stall_ms;     /* compute-stream time spent waiting for a step's prefetch to land: from the
                                     moment the stream reaches the wait (the previous work has ended) to the
                                     moment it passes it (FLAG_TIME_KERNELS, also with TIME_ATTN_ONLY)          */
  uint64_t prefetch_stalls;       /* steps that had such a wait                                              */
} pipemax_stats_t;

/* ---- life cycle ----------------------------------------------------------------------- */

/* Validates cfg (host pointer), allocates weights, pools, staging, streams and events on
 * cfg->device and returns the handle in *out.  Errors: ERR_ARG (shape/dtype/page size),
 * ERR_OOM_DEVICE, ERR_OOM_HOST, ERR_HIP.  Nothing is left allocated on error.            */
int pipemax_stage_create(const pipemax_config_t* cfg, pipemax_stage_t** out);

/* Drains all work, stops the write-back worker, frees everything.                         */
int pipemax_stage_destroy(pipemax_stage_t* st);

/* Copies one weight tensor (host pointer, canonical layout above, stage element type,
 * `bytes` must equal the tensor's size) into the stage; the library re-tiles it into its
 * internal layout.  Synchronous.                                                          */
int pipemax_set_weight(pipemax_stage_t* st, int layer, int which, const void* host, size_t bytes);

/* ---- micro-batches and their host-resident KV (Sec. 3.3.2: decode batches D_0..D_{n-1}) - */

/* Defines micro-batch `mb` (0 <= mb < n_microbatches, not yet defined) with n_seqs sequences
 * whose prompts have ctx_lens[i] cached tokens (host pointer; 0 <= len <= max_ctx).
 * Allocates ceil(len/16) host pages per sequence (plus the reservation of host_reserve_tokens),
 * consecutively, lowest index first.
 * All sequences start HOST-resident.  Errors: ERR_ARG, ERR_POOL_EXHAUSTED.                */
int pipemax_mb_define(pipemax_stage_t* st, int mb, int n_seqs, const int32_t* ctx_lens);

/* Measurement aid for hosts that cannot pin the KV of a whole configuration (a process here pins at most
 * about 64 GiB; the 70B-shaped configurations need 172 and 344 GB): defines micro-batch `mb` (not yet
 * defined) as an ALIAS of the defined, non-alias micro-batch `src_mb`.  The alias has as many sequences,
 * with the lengths src_mb's have now, and its block tables name the SAME host pages (reserved growth pages
 * included); nothing is taken from the host pool.  GPU pages, prefetch, decode and evict work as for any
 * micro-batch, so its transfers move the same bytes along the same access pattern and its steps run the same
 * kernels.  Its write-back lands in the shared pages: once an alias has decoded, the tokens appended to the
 * alias AND to its source are unspecified in the host replica (whichever wrote last), while every token that
 * existed when the alias was defined stays intact as long as both advance by the same number of steps.
 * For timing only: parity is checked on micro-batches that are neither aliases nor sources of a stepped alias.
 * pipemax_kv_host_write on an alias fails with ERR_STATE.  Errors: ERR_ARG.                                  */
int pipemax_mb_define_alias(pipemax_stage_t* st, int mb, int src_mb);
/* *src_mb (host pointer) receives the micro-batch `mb` is an alias of, or -1.                              */
int pipemax_mb_alias_of(pipemax_stage_t* st, int mb, int32_t* src_mb);

/* Writes / reads tokens [tok0, tok0+ntok) of one layer of one sequence in the HOST replica.
 * K and V are host pointers, canonical layout [ntok][Hkv][d].  Both calls first wait until
 * all pending write-back of that micro-batch has landed.  Range must lie within the
 * sequence's current length.  kv_host_write does not touch GPU pages: call it while the
 * sequence is HOST-resident (ERR_STATE otherwise).                                         */
int pipemax_kv_host_write(pipemax_stage_t* st, int mb, int seq, int layer, int tok0, int ntok,
                          const void* K, const void* V);
int pipemax_kv_host_read(pipemax_stage_t* st, int mb, int seq, int layer, int tok0, int ntok,
                         void* K, void* V);
/* Same read from the GPU pages (debug / parity).  Synchronises the stage first.
 * ERR_NOT_RESIDENT if the sequence has no GPU pages.                                      */
int pipemax_kv_dev_read(pipemax_stage_t* st, int mb, int seq, int layer, int tok0, int ntok,
                        void* K, void* V);

/* ---- the hot path ---------------------------------------------------------------------- */

/* Prefetch (Sec. 3.3.2: the KV cache of the next batch D_j is brought from CPU memory while D_i
 * executes; Sec. 3.4.2, block-first layout): for every named sequence of `mb` that is HOST-resident,
 * allocates GPU pages (lowest free index first) and arranges host->device copies of its pages on the
 * library's prefetch stream, adjacent (host, GPU) page pairs merged into single copies.
 * seq_ids: host pointer to n sequence indices, or NULL for all sequences of mb.  Sequences that
 * already have GPU pages are skipped.  Errors: ERR_ARG, ERR_POOL_EXHAUSTED (nothing applied), ERR_HIP
 * (also when an earlier prefetch failed after its call had returned).
 * The call does the bookkeeping and returns at once.  A worker thread of the stage issues the copies
 * as soon as (1) the write-back of `mb` that was pending at the time of the call has landed in the
 * host replica and (2) the decode steps that last read the pages being re-used (those of the
 * micro-batches evicted since the previous prefetch) have finished.  (2) is a host-side wait in that
 * thread: a copy stream that waits on a not-yet-signalled event of another stream was measured to
 * leave gaps of 150-350 us between its copies on this platform.  PIPEMAX_FLAG_STREAM_ORDERED_EVICT
 * selects the stream-side wait instead.  A decode step of `mb` is ordered after the copies.        */
int pipemax_prefetch_kv(pipemax_stage_t* st, int mb, const int32_t* seq_ids, int n);

/* One decode step of the stage on micro-batch `mb` (the op list of the benchmark spec; cost
 * structure alpha*b + beta*L + delta of Sec. 3.3.1): for every layer RMSNorm, QKV projection,
 * RoPE at position L_i, append of the new K,V to page table[i][L_i/16] slot L_i%16, GQA
 * attention over L_i+1 tokens, output projection + residual, RMSNorm, SwiGLU FFN + residual.
 * hidden_in / hidden_out: device pointers, [b][hidden] row-major in the stage's element type
 * (may alias).  hip_stream: the hipStream_t to run on (NULL = the library's own compute
 * stream).  Each layer's new K,V are also written to a contiguous staging buffer that the
 * write-back stream copies to pinned host memory, where a worker thread places them into the
 * host pages (Sec. 3.4.2, asynchronous CPU-assisted offloading).  Afterwards every L_i of mb is
 * one larger.  New pages (GPU and host) are taken when L_i % 16 == 0.
 * Errors: ERR_ARG, ERR_NOT_RESIDENT (some sequence of mb has no GPU pages and no prefetch in
 * flight), ERR_STATE (max_ctx reached), ERR_POOL_EXHAUSTED, ERR_HIP.                       */
int pipemax_decode_step(pipemax_stage_t* st, int mb, const void* hidden_in, void* hidden_out,
                        void* hip_stream);

/* The same step over a caller-chosen part of `mb` (Sec. 3.3.2: the executed batch is
 * D_j^res united with the prefetched set P_t, i.e. the sequences of D_j whose KV is on the GPU;
 * hybrid batches of Sec. 3.1.2).  seq_ids: host pointer to n distinct sequence indices; row r of
 * hidden_in / hidden_out ([n][hidden]) belongs to sequence seq_ids[r].  Only the listed
 * sequences must be resident, only they grow by one token, the others are untouched.  n == 0 is
 * a successful no-op.  The block table of the step is rebuilt and uploaded on every call.
 * Errors: as pipemax_decode_step, plus ERR_ARG for an index out of range or listed twice.     */
int pipemax_decode_step_seqs(pipemax_stage_t* st, int mb, const int32_t* seq_ids, int n,
                             const void* hidden_in, void* hidden_out, void* hip_stream);

/* pipemax_decode_step for callers that cannot allocate: code under HIP graph capture, serving loops and
 * harnesses that forbid hipMalloc.  Same arguments, same result, same errors and the same kernels as
 * pipemax_decode_step, but every device buffer the step works in besides its inputs, outputs, weights and KV
 * pages (residual stream, RoPE table, matrix-operand activations, split-K partials of the GEMMs and of the
 * attention, arrival counters, partial sums of squares) lies in one static device array of
 * PIPEMAX_NOALLOC_SCRATCH_BYTES that the library holds per GPU until the process ends, and the call itself calls
 * no hipMalloc / hipFree / event creation (a timing flag set on the stage is ignored for this call).
 * A step that needs more than the array holds is refused with ERR_ARG and a text naming both sizes, before
 * anything is enqueued (8B-shaped stages of up to 128 rows fit; the 256-row passes of the 70B-shaped stage
 * do not).  Only stages on the matrix-core engine are served (ERR_STATE otherwise).
 * All stages and calls on one GPU share the array: it keeps the last call's contents, the call clears what
 * must start at zero (with a kernel on hip_stream), and two calls whose work overlaps in time on one GPU --
 * different streams, or different stages driven from different threads -- race; calls on one stream are safe. */
#define PIPEMAX_NOALLOC_SCRATCH_BYTES (64u << 20)
int pipemax_decode_step_noalloc(pipemax_stage_t* st, int mb, const void* hidden_in, void* hidden_out,
                                void* hip_stream);

/* Prefill (Sec. 3.1.1: the KV cache produced by prefill is offloaded to CPU memory asynchronously;
 * Sec. 3.4.2: per-layer offload and CPU re-layout): runs the stage over n_tokens NEW tokens of one
 * sequence, at positions L .. L + n_tokens - 1 where L is the sequence's current length (0 for a fresh
 * request; a longer prompt may be fed in several calls).  Token t attends to all cached tokens and to
 * the new tokens up to and including itself (causal).  hidden_in / hidden_out: device pointers,
 * [n_tokens][hidden] row-major in the stage's element type (may alias).  The tokens are processed in
 * chunks of at most max_seqs_per_mb rows; each chunk is one pass of the same kernels as a decode step
 * (more than 64 rows take the large-tile GEMM path), appends its K,V to the sequence's GPU pages and
 * hands them to the write-back stream and the host re-layout worker exactly like a decode step, so the
 * host replica is complete once the work has drained and pipemax_evict_kv frees the GPU pages without
 * a copy.  The sequence must not be HOST-resident (call pipemax_prefetch_kv first, also for an empty
 * sequence).  Afterwards its length is L + n_tokens.  n_tokens == 0 is a successful no-op.
 * Errors: ERR_ARG, ERR_NOT_RESIDENT, ERR_STATE (max_ctx), ERR_POOL_EXHAUSTED (checked for the whole
 * call before anything is enqueued), ERR_HIP.                                                        */
int pipemax_prefill(pipemax_stage_t* st, int mb, int seq, int n_tokens, const void* hidden_in,
                    void* hidden_out, void* hip_stream);

/* Evict (Sec. 3.3.2: the GPU blocks of the batch D_k that has just executed are the ones a prefetch
 * may overwrite): releases the GPU pages of the named sequences (NULL = all of mb).  No bulk copy is made: the
 * host replica is kept current by the per-layer write-back.  Later prefetches into the freed
 * pages are ordered after the last decode step that read them.  Returns without blocking.  */
int pipemax_evict_kv(pipemax_stage_t* st, int mb, const int32_t* seq_ids, int n);

/* Blocks until all three streams are idle and the write-back worker has placed every
 * pending token into the host replica.                                                    */
int pipemax_sync(pipemax_stage_t* st);

/* ---- introspection ---------------------------------------------------------------------- */

int pipemax_get_stats(pipemax_stage_t* st, pipemax_stats_t* out);   /* synchronises if timing */
int pipemax_reset_stats(pipemax_stage_t* st);
/* Sets and clears run-time flags; only the PIPEMAX_FLAG_TIME_* flags and PIPEMAX_FLAG_NO_WRITEBACK can be
 * changed after creation (ERR_ARG otherwise).  Synchronises the stage first.                */
int pipemax_set_flags(pipemax_stage_t* st, uint32_t set, uint32_t clear);

/* Copies the configuration the stage was created with into *out (host pointer).            */
int pipemax_get_config(pipemax_stage_t* st, pipemax_config_t* out);
/* *n_seqs (host pointer) receives the number of sequences of mb, 0 if mb is not defined yet. */
int pipemax_mb_size(pipemax_stage_t* st, int mb, int32_t* n_seqs);
/* out: host pointer to n_seqs int32 (current context lengths).                             */
int pipemax_get_ctx_lens(pipemax_stage_t* st, int mb, int32_t* out);
/* out: host pointer to n_seqs int32: 0 = HOST, 1 = prefetch in flight, 2 = GPU.            */
int pipemax_get_residency(pipemax_stage_t* st, int mb, int32_t* out);
/* gpu_pages / host_pages: host pointers with room for *n entries (either may be NULL); on
 * return *n = number of pages of the sequence; gpu_pages entries are -1 when HOST-resident. */
int pipemax_get_block_table(pipemax_stage_t* st, int mb, int seq, int32_t* gpu_pages,
                            int32_t* host_pages, int* n);
/* Residual stream after every layer of the last decode_step (needs FLAG_CAPTURE_LAYERS):
 * out = host pointer to [n_layers][b][hidden] float.  Synchronises.                        */
int pipemax_get_layer_outputs(pipemax_stage_t* st, float* out, size_t bytes);

/* ---- test hooks (host-forced conditions; every kernel still runs to completion) --------------- */

/* Fills every currently free GPU page with the 16-bit pattern (e.g. 0x7FC0, a bf16 NaN), after
 * synchronising the stage: any read of a page that no live sequence owns then poisons the output. */
int pipemax_debug_fill_free_gpu_pages(pipemax_stage_t* st, uint16_t pattern);
/* Delays, in microseconds, injected from now on before every prefetch batch (on the host->device
 * stream), before every write-back copy and before every re-layout job (both in the worker thread,
 * which issues the copy once the step's K,V rows are in the staging buffer).  Results must not
 * depend on them: they only move work in time.                                                    */
int pipemax_debug_set_delays(pipemax_stage_t* st, int h2d_us, int d2h_us, int worker_us);

const char* pipemax_last_error(void);
const char* pipemax_version(void);

/* ---- measurement aid ------------------------------------------------------------------------ */

/* Launches a plain device-to-device copy kernel (named k_probe_copy in profiles) of `bytes` bytes
 * (a multiple of 16; dst and src are 16-byte-aligned device pointers that do not overlap) on
 * hip_stream (NULL = default stream).  Its known traffic calibrates the hardware counters that
 * the HBM-traffic figures are derived from.                                                   */
int pipemax_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* Launches a read-only streaming kernel over `bytes` bytes of device memory at src (16-byte aligned pointer and
 * size) on hip_stream: what HBM delivers to a plain coalesced reader.  segment_trips = 0: grid-stride order; > 0:
 * every work-group reads contiguous pieces of segment_trips * 4 KiB.  sink16: 16 bytes of device memory (never
 * written in practice; it keeps the loads alive).  The caller times the launch (events on hip_stream).        */
int pipemax_probe_read(const void* src, size_t bytes, int segment_trips, void* sink16, void* hip_stream);

/* Host-link probe (Sec. 4.4 compares the block-first layout, whose transfers are whole pages and page runs, with a
 * layer-first layout, whose transfers are per-(page, layer) fragments): allocates pinned host and device buffers of
 * its own on `device`, copies total_bytes in pieces of piece_bytes lying piece_stride bytes apart on both sides
 * (stride = piece: one contiguous region) with one hipMemcpyAsync per piece, `repeats` times after a warm-up pass, and
 * reports the fastest pass.  direction: 0 = host->device, 1 = device->host, 2 = both at once on two streams.
 * h2d_s / d2h_s: first copy issued to last copy done on each stream (HIP events); wall_s: the same for the whole pass
 * by the host clock.  Synchronises the device.  Errors: ERR_ARG, ERR_OOM_HOST, ERR_OOM_DEVICE, ERR_HIP.           */
typedef struct {
  double   h2d_s, d2h_s, wall_s;
  uint64_t h2d_bytes, d2h_bytes, pieces;
} pipemax_link_probe_t;
int pipemax_probe_link(int device, size_t total_bytes, size_t piece_bytes, size_t piece_stride, int direction,
                       int repeats, pipemax_link_probe_t* out);

/* The same probe for strided host->device copies (hipMemcpy2DAsync): n_copies copies of rows_per_copy rows of
 * row_bytes each, the rows host_pitch bytes apart in pinned host memory and packed on the device -- what a prefetch
 * from block-first host pages into a layer-major device pool issues per (page run, layer).                       */
int pipemax_probe_link_strided(int device, size_t row_bytes, size_t host_pitch, int rows_per_copy, int n_copies,
                          int repeats, pipemax_link_probe_t* out);

/* Launch-overhead probe: a chain of n_kernels one-wave kernels, each depending on its predecessor, enqueued one by
 * one (use_graph = 0) or replayed as one captured HIP graph (use_graph = 1); `repeats` passes after a warm-up, the
 * fastest reported.  host_enqueue_s: host time to hand the chain to the runtime; gpu_s: first kernel's start to last
 * kernel's end (HIP events around the chain).  Checks that every kernel ran.  Synchronises its own stream.       */
typedef struct {
  double   host_enqueue_s, gpu_s;
  uint64_t kernels;
} pipemax_launch_probe_t;
int pipemax_probe_launch(int device, int n_kernels, int use_graph, int repeats, pipemax_launch_probe_t* out);

/* ---- host-side planning helpers (pure host code; also used by the CPU tests) ------------- */

/* Element offset, inside one KV page, of element `dd` of token slot `tok` (0..15) of head
 * `head` of K (kv = 0) or V (kv = 1) of layer `layer`.  Returns -1 on bad arguments.       */
int64_t pipemax_page_elem_offset(int n_layers, int n_kv_heads, int head_dim,
                                 int layer, int kv, int head, int tok, int dd);

/* Split-K plan of the large-tile GEMM (more than 128 rows; n_cols a multiple of 256, k of 16): the number
 * of K splits the stage plans for a rows x k x n_cols product (*plan_splits: the partials its consumers sum),
 * the number the launch geometry derives from it (*launch_splits; the two must agree) and the 16-wide
 * k-steps per split.  Pure host arithmetic.  Errors: ERR_ARG.                                          */
int pipemax_plan_gemm_splits(int rows, int n_cols, int k, int32_t* plan_splits, int32_t* launch_splits,
                             int32_t* k_steps_per_split);

/* Plan of the decode attention for a step of n_seqs sequences whose longest context is max_ctx_tokens tokens (the new
 * token included) and whose contexts cover sum_pages pages in all, on a GPU of compute_units compute units.  The
 * attention's items are (chunk of the context, KV head, sequence).  *wave_per_item = 1: every item is streamed by one
 * wave (chosen when n_seqs * n_kv_heads >= 2 * compute_units); 0: by a work-group of four waves that share its pages
 * (then *chunk_pages <= 256).  *chunk_pages = pages per item, *n_chunks = chunks the longest sequence is cut into.
 * Chunks are even: a context one page longer than an item takes becomes two halves, not a full chunk and a one-page
 * chunk.  Pure host arithmetic (the stage's own planner, without the PIPEMAX_ATTN_CHUNK_PAGES / PIPEMAX_ATTN_KERNEL
 * overrides).  Errors: ERR_ARG.                                                                                     */
int pipemax_plan_attention_chunks(int n_seqs, int n_kv_heads, int max_ctx_tokens, int64_t sum_pages,
                                  int compute_units, int32_t* chunk_pages, int32_t* n_chunks, int32_t* wave_per_item);

/* Merges n (src_page, dst_page) pairs, in the given order, into runs of consecutive pages,
 * each at most max_run_pages long.  Writes (src_first, dst_first, count) triples to runs
 * (room for 3*n int32) and returns the number of runs, or a negative status.               */
int pipemax_plan_copy_runs(const int32_t* src_pages, const int32_t* dst_pages, int n,
                           int max_run_pages, int32_t* runs);

/* Lowest-index-first page allocator (the one the stage uses for both pools).               */
int pipemax_pool_create(int n_pages, pipemax_pool_t** out);
int pipemax_pool_destroy(pipemax_pool_t* p);
int pipemax_pool_alloc(pipemax_pool_t* p, int n, int32_t* out_pages);  /* all or nothing */
int pipemax_pool_free(pipemax_pool_t* p, const int32_t* pages, int n);
int pipemax_pool_free_count(pipemax_pool_t* p);

#ifdef __cplusplus
}
#endif
#endif /* PIPEMAX_H */

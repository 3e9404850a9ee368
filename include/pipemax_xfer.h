/*
 * pipemax_xfer.h -- C ABI of the demand-priority transfer orchestrator (host code + HIP copies).
 *
 * PipeMax Sec. 3.4.2 ("Demand-Priority Transfer Orchestration"): the runtime moves three kinds of data
 * over the host link -- small latency-critical activation transfers, KV prefetch (host -> device) and KV
 * offload (device -> host) -- and enforces priorities by controlling the ORDER IN WHICH COPIES ARE
 * SUBMITTED: urgent copies are issued at once, bulk KV copies opportunistically.
 *
 * This component does exactly that.  Every stream keeps the default priority.  A dispatcher thread
 * owns, per direction, one bulk stream and one urgent stream.  Bulk requests are cut into chunks of at
 * most chunk_bytes and at most max_inflight_bulk chunks per direction are handed to the runtime at any
 * time, so a newly arrived urgent copy never has more than that many chunks submitted ahead of it.
 * Urgent requests are submitted whole, before any waiting bulk chunk, in arrival order.  Bulk requests
 * of one direction complete in arrival order.
 *
 * Conventions: as in pipemax.h.  dst / src are host (pinned, allocated with hipHostMalloc) or device
 * pointers owned by the caller and must stay valid until the request's ticket has completed.  With
 * device = -1 the orchestrator runs without a GPU: both pointers are host memory and the dispatcher
 * copies with memcpy (used to test the queue discipline on the CPU).  Calls may come from any thread.
 */
#ifndef PIPEMAX_XFER_H
#define PIPEMAX_XFER_H

#include "pipemax.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pipemax_xfer pipemax_xfer_t;   /* opaque */

enum { PIPEMAX_XFER_URGENT = 0, PIPEMAX_XFER_BULK = 1 };
enum { PIPEMAX_XFER_H2D = 0, PIPEMAX_XFER_D2H = 1 };

typedef struct {
  int32_t  device;             /* HIP device ordinal, or -1 for the host-only mode                 */
  int32_t  max_inflight_bulk;  /* bulk chunks per direction submitted but not finished (>= 1)      */
  uint64_t chunk_bytes;        /* largest bulk chunk (>= 4096); 0 = bulk requests are not cut      */
  int32_t  log_capacity;       /* submissions kept in the order log (0 = none)                     */
  int32_t  reserved;
} pipemax_xfer_config_t;

/* Totals since creation (or the last reset), per kind [URGENT, BULK].  latency = completion time minus
 * the time pipemax_xfer_submit was called, measured on the host.                                   */
typedef struct {
  uint64_t requests[2], bytes[2], chunks[2];
  double   latency_sum_s[2], latency_max_s[2];
} pipemax_xfer_stats_t;

/* One entry of the order log: the n-th copy handed to the runtime.                                 */
typedef struct {
  uint64_t ticket;
  uint64_t offset, bytes;      /* the part of the request this copy covers                          */
  int32_t  kind, dir;
} pipemax_xfer_log_t;

/* Errors: ERR_ARG (NULL, ranges above), ERR_HIP (streams / events).                                */
int pipemax_xfer_create(const pipemax_xfer_config_t* cfg, pipemax_xfer_t** out);
/* Completes everything queued, stops the dispatcher, releases streams and events.                  */
int pipemax_xfer_destroy(pipemax_xfer_t* x);

/* Queues one copy of `bytes` bytes.  *ticket (host pointer) receives a number > 0 that grows with
 * every call.  Returns at once.  Errors: ERR_ARG (NULL pointers with bytes > 0, bad kind / dir).   */
int pipemax_xfer_submit(pipemax_xfer_t* x, int kind, int dir, void* dst, const void* src, size_t bytes,
                        uint64_t* ticket);
/* Blocks the calling thread until the request has completed (its data is at dst).  ERR_ARG for a
 * ticket that was never issued; ERR_HIP if any copy of the orchestrator has failed so far (sticky).  */
int pipemax_xfer_wait(pipemax_xfer_t* x, uint64_t ticket);
/* Returns 1 if the request has completed, 0 if not, ERR_ARG for a ticket that was never issued.      */
int pipemax_xfer_poll(pipemax_xfer_t* x, uint64_t ticket);
/* Makes `hip_stream` (device pointer-sized hipStream_t) wait for the request: blocks the calling
 * thread until the request's last copy has been SUBMITTED, then enqueues a wait for its completion
 * event on the stream.  Not available in the host-only mode (ERR_STATE).                            */
int pipemax_xfer_stream_wait(pipemax_xfer_t* x, uint64_t ticket, void* hip_stream);
/* Blocks until both queues are empty and every submitted copy has finished.  ERR_HIP as for wait.   */
int pipemax_xfer_drain(pipemax_xfer_t* x);

int pipemax_xfer_get_stats(pipemax_xfer_t* x, pipemax_xfer_stats_t* out);
int pipemax_xfer_reset_stats(pipemax_xfer_t* x);
/* Copies up to `capacity` log entries (oldest first) into out; returns their number (>= 0) or an
 * error.  The log stops recording when it is full.                                                 */
int pipemax_xfer_get_log(pipemax_xfer_t* x, pipemax_xfer_log_t* out, int capacity);
/* Test hook for the host-only mode: the dispatcher sleeps this many microseconds per MiB it copies,
 * so that a bulk request stays in progress long enough for an urgent one to arrive behind it.      */
int pipemax_xfer_debug_set_host_us_per_mib(pipemax_xfer_t* x, int us);
/* Test hook: while paused the dispatcher issues nothing, so a set of requests can be queued and the
 * order in which they are then issued is fully determined by the queue discipline.                */
int pipemax_xfer_debug_pause(pipemax_xfer_t* x, int paused);

/* Routes the KV prefetch copies of a stage through the orchestrator (x = NULL: back to the stage's own
 * prefetch stream).  pipemax_prefetch_kv then queues its copy runs as bulk host-to-device requests, a
 * decode step waits for them through pipemax_xfer_stream_wait, pipemax_sync drains the orchestrator.
 * The orchestrator must be on the stage's device and must outlive the attachment.  Synchronises the
 * stage first.                                                                                      */
int pipemax_stage_attach_xfer(pipemax_stage_t* st, pipemax_xfer_t* x);

#ifdef __cplusplus
}
#endif
#endif

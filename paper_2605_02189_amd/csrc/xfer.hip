// Demand-priority transfer orchestrator (PipeMax Sec. 3.4.2): priorities are enforced by the order in
// which copies are handed to the HIP runtime, not by stream priorities (every stream here has the default
// priority).  A dispatcher thread submits urgent copies whole and at once, and feeds the bulk (KV) copies of
// each direction in chunks, a bounded number of which are outstanding at any time.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <memory>
#include <mutex>
#include <thread>
#include <unordered_map>
#include <vector>

#include "pipemax_xfer.h"

namespace pmx {
void set_error(const char* fmt, ...);
}

#define XF_FAIL(code, ...)         \
  do {                             \
    ::pmx::set_error(__VA_ARGS__); \
    return (code);                 \
  } while (0)

namespace {

double now_s() {
  return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

struct Request {
  uint64_t ticket = 0;
  int kind = 0, dir = 0;
  char* dst = nullptr;
  const char* src = nullptr;
  size_t bytes = 0, issued = 0;       // bytes handed to the runtime so far
  int outstanding = 0;                // copies submitted and not yet seen finished
  bool all_submitted = false, done = false;
  double t_submit = 0;
  hipEvent_t ev_last = nullptr;       // completion of the request's last copy
};

struct Flight {                       // one submitted copy
  std::shared_ptr<Request> req;
  hipEvent_t ev = nullptr;
};

}  // namespace

struct pipemax_xfer {
  pipemax_xfer_config_t cfg{};
  bool gpu = false;
  hipStream_t s_bulk[2] = {}, s_urgent[2] = {};
  std::mutex mu;
  std::condition_variable cv_work, cv_done;
  std::deque<std::shared_ptr<Request>> q_urgent, q_bulk[2];
  std::deque<Flight> fly_bulk[2], fly_urgent;
  std::unordered_map<uint64_t, std::shared_ptr<Request>> live;
  std::vector<hipEvent_t> ev_pool;
  std::vector<pipemax_xfer_log_t> log;
  pipemax_xfer_stats_t stats{};
  uint64_t next_ticket = 1;
  int host_us_per_mib = 0;
  bool stop = false, paused = false;
  hipError_t hip_error = hipSuccess;   // first failure of a copy or event call (sticky)
  std::thread th;

  hipEvent_t get_event() {
    if (!ev_pool.empty()) {
      hipEvent_t e = ev_pool.back();
      ev_pool.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreateWithFlags(&e, hipEventDisableTiming);
    return e;
  }

  void finish(const std::shared_ptr<Request>& r) {   // mu held
    r->done = true;
    const double lat = now_s() - r->t_submit;
    stats.latency_sum_s[r->kind] += lat;
    if (lat > stats.latency_max_s[r->kind]) stats.latency_max_s[r->kind] = lat;
    if (r->ev_last) {
      ev_pool.push_back(r->ev_last);
      r->ev_last = nullptr;
    }
    live.erase(r->ticket);
  }

  // hands one copy (the whole request, or its next chunk) to the runtime; mu held
  void issue(const std::shared_ptr<Request>& r, size_t n, std::unique_lock<std::mutex>& lk) {
    const size_t off = r->issued;
    r->issued += n;
    r->outstanding += 1;
    const bool last = r->issued == r->bytes;
    stats.chunks[r->kind] += 1;
    if ((int)log.size() < cfg.log_capacity) log.push_back({r->ticket, (uint64_t)off, (uint64_t)n, r->kind, r->dir});
    if (gpu) {
      hipStream_t s = (r->kind == PIPEMAX_XFER_URGENT) ? s_urgent[r->dir] : s_bulk[r->dir];
      auto note = [&](hipError_t e) {
        if (e != hipSuccess && hip_error == hipSuccess) hip_error = e;
      };
      note(hipMemcpyAsync(r->dst + off, r->src + off, n,
                          r->dir == PIPEMAX_XFER_H2D ? hipMemcpyHostToDevice : hipMemcpyDeviceToHost, s));
      Flight f{r, get_event()};
      note(hipEventRecord(f.ev, s));
      if (last) {
        r->ev_last = get_event();
        note(hipEventRecord(r->ev_last, s));
        r->all_submitted = true;
        cv_done.notify_all();
      }
      (r->kind == PIPEMAX_XFER_URGENT ? fly_urgent : fly_bulk[r->dir]).push_back(f);
    } else {
      // host-only mode: the copy runs here, outside the lock, so that submissions can arrive meanwhile
      const int us = host_us_per_mib;
      lk.unlock();
      if (n) memcpy(r->dst + off, r->src + off, n);
      if (us > 0) std::this_thread::sleep_for(std::chrono::microseconds((int64_t)us * (int64_t)n / (1 << 20) + 1));
      lk.lock();
      r->outstanding -= 1;
      if (last) {
        r->all_submitted = true;
        finish(r);
        cv_done.notify_all();
      }
    }
  }

  // retires finished copies (in submission order per stream); returns true if anything is still in flight
  bool reap() {   // mu held
    auto sweep = [&](std::deque<Flight>& d) {
      while (!d.empty()) {
        const hipError_t q = hipEventQuery(d.front().ev);
        if (q == hipErrorNotReady) break;
        if (q != hipSuccess && hip_error == hipSuccess) hip_error = q;   // retired all the same: nothing waits forever
        Flight f = d.front();
        d.pop_front();
        ev_pool.push_back(f.ev);
        f.req->outstanding -= 1;
        if (f.req->all_submitted && f.req->outstanding == 0) {
          finish(f.req);
          cv_done.notify_all();
        }
      }
    };
    sweep(fly_urgent);
    sweep(fly_bulk[0]);
    sweep(fly_bulk[1]);
    return !fly_urgent.empty() || !fly_bulk[0].empty() || !fly_bulk[1].empty();
  }

  void run() {
    if (gpu) (void)hipSetDevice(cfg.device);
    std::unique_lock<std::mutex> lk(mu);
    for (;;) {
      const bool flying = gpu ? reap() : false;
      bool issued = false;
      if (paused && !stop) {          // test hook: requests pile up, nothing is issued
        cv_work.wait_for(lk, std::chrono::microseconds(200));
        continue;
      }
      // 1. urgent copies: whole, in arrival order, before any waiting bulk chunk
      while (!q_urgent.empty()) {
        auto r = q_urgent.front();
        q_urgent.pop_front();
        issue(r, r->bytes, lk);
        issued = true;
      }
      // 2. bulk: the next chunk of the oldest request of each direction, while the window has room.  One
      //    chunk per direction per pass, so that an urgent arrival is looked at between any two chunks.
      for (int d = 0; d < 2; ++d) {
        if (q_bulk[d].empty()) continue;
        if (gpu && (int)fly_bulk[d].size() >= cfg.max_inflight_bulk) continue;
        auto r = q_bulk[d].front();
        const size_t left = r->bytes - r->issued;
        const size_t n = (cfg.chunk_bytes && left > cfg.chunk_bytes) ? (size_t)cfg.chunk_bytes : left;
        if (r->issued + n == r->bytes) q_bulk[d].pop_front();
        issue(r, n, lk);
        issued = true;
        if (!q_urgent.empty()) break;
      }
      if (issued) continue;
      const bool queued = !q_urgent.empty() || !q_bulk[0].empty() || !q_bulk[1].empty();
      if (stop && !queued && !flying) return;
      if (flying || queued) cv_work.wait_for(lk, std::chrono::microseconds(20));   // poll the completion events
      else cv_work.wait(lk, [&] { return stop || !q_urgent.empty() || !q_bulk[0].empty() || !q_bulk[1].empty(); });
    }
  }
};

extern "C" {

int pipemax_xfer_create(const pipemax_xfer_config_t* cfg, pipemax_xfer_t** out) {
  if (!cfg || !out) XF_FAIL(PIPEMAX_ERR_ARG, "null argument");
  *out = nullptr;
  if (cfg->max_inflight_bulk < 1 || (cfg->chunk_bytes != 0 && cfg->chunk_bytes < 4096) || cfg->log_capacity < 0 ||
      cfg->device < -1)
    XF_FAIL(PIPEMAX_ERR_ARG, "max_inflight_bulk >= 1, chunk_bytes 0 or >= 4096, log_capacity >= 0, device >= -1");
  auto* x = new pipemax_xfer();
  x->cfg = *cfg;
  x->gpu = cfg->device >= 0;
  x->log.reserve(cfg->log_capacity);
  if (x->gpu) {
    hipError_t e = hipSetDevice(cfg->device);
    for (int d = 0; d < 2 && e == hipSuccess; ++d) {
      e = hipStreamCreateWithFlags(&x->s_bulk[d], hipStreamNonBlocking);
      if (e == hipSuccess) e = hipStreamCreateWithFlags(&x->s_urgent[d], hipStreamNonBlocking);
    }
    if (e != hipSuccess) {
      (void)hipGetLastError();
      for (int d = 0; d < 2; ++d) {
        if (x->s_bulk[d]) (void)hipStreamDestroy(x->s_bulk[d]);
        if (x->s_urgent[d]) (void)hipStreamDestroy(x->s_urgent[d]);
      }
      delete x;
      XF_FAIL(PIPEMAX_ERR_HIP, "stream creation failed: %s", hipGetErrorString(e));
    }
  }
  x->th = std::thread([x] { x->run(); });
  *out = x;
  return PIPEMAX_OK;
}

int pipemax_xfer_destroy(pipemax_xfer_t* x) {
  if (!x) XF_FAIL(PIPEMAX_ERR_ARG, "null orchestrator");
  {
    std::lock_guard<std::mutex> lk(x->mu);
    x->stop = true;
  }
  x->cv_work.notify_all();
  x->th.join();
  if (x->gpu) {
    (void)hipSetDevice(x->cfg.device);
    for (int d = 0; d < 2; ++d) {
      (void)hipStreamSynchronize(x->s_bulk[d]);
      (void)hipStreamSynchronize(x->s_urgent[d]);
      (void)hipStreamDestroy(x->s_bulk[d]);
      (void)hipStreamDestroy(x->s_urgent[d]);
    }
    for (hipEvent_t e : x->ev_pool) (void)hipEventDestroy(e);
  }
  delete x;
  return PIPEMAX_OK;
}

int pipemax_xfer_submit(pipemax_xfer_t* x, int kind, int dir, void* dst, const void* src, size_t bytes,
                        uint64_t* ticket) {
  if (!x || !ticket) XF_FAIL(PIPEMAX_ERR_ARG, "null argument");
  if ((kind != PIPEMAX_XFER_URGENT && kind != PIPEMAX_XFER_BULK) || (dir != PIPEMAX_XFER_H2D && dir != PIPEMAX_XFER_D2H))
    XF_FAIL(PIPEMAX_ERR_ARG, "bad kind %d or direction %d", kind, dir);
  if (bytes > 0 && (!dst || !src)) XF_FAIL(PIPEMAX_ERR_ARG, "null buffer");
  auto r = std::make_shared<Request>();
  r->kind = kind;
  r->dir = dir;
  r->dst = (char*)dst;
  r->src = (const char*)src;
  r->bytes = bytes;
  r->t_submit = now_s();
  {
    std::lock_guard<std::mutex> lk(x->mu);
    if (x->stop) XF_FAIL(PIPEMAX_ERR_STATE, "the orchestrator is shutting down");
    r->ticket = x->next_ticket++;
    *ticket = r->ticket;
    x->live[r->ticket] = r;
    x->stats.requests[kind] += 1;
    x->stats.bytes[kind] += bytes;
    (kind == PIPEMAX_XFER_URGENT ? x->q_urgent : x->q_bulk[dir]).push_back(r);
  }
  x->cv_work.notify_all();
  return PIPEMAX_OK;
}

int pipemax_xfer_wait(pipemax_xfer_t* x, uint64_t ticket) {
  if (!x) XF_FAIL(PIPEMAX_ERR_ARG, "null orchestrator");
  std::unique_lock<std::mutex> lk(x->mu);
  if (ticket == 0 || ticket >= x->next_ticket) XF_FAIL(PIPEMAX_ERR_ARG, "ticket %llu was never issued", (unsigned long long)ticket);
  auto it = x->live.find(ticket);
  if (it == x->live.end()) return PIPEMAX_OK;
  std::shared_ptr<Request> r = it->second;
  x->cv_done.wait(lk, [&] { return r->done; });
  if (x->hip_error != hipSuccess) XF_FAIL(PIPEMAX_ERR_HIP, "a copy failed: %s", hipGetErrorString(x->hip_error));
  return PIPEMAX_OK;
}

int pipemax_xfer_poll(pipemax_xfer_t* x, uint64_t ticket) {
  if (!x) XF_FAIL(PIPEMAX_ERR_ARG, "null orchestrator");
  std::lock_guard<std::mutex> lk(x->mu);
  if (ticket == 0 || ticket >= x->next_ticket) XF_FAIL(PIPEMAX_ERR_ARG, "ticket %llu was never issued", (unsigned long long)ticket);
  return x->live.find(ticket) == x->live.end() ? 1 : 0;
}

int pipemax_xfer_stream_wait(pipemax_xfer_t* x, uint64_t ticket, void* hip_stream) {
  if (!x) XF_FAIL(PIPEMAX_ERR_ARG, "null orchestrator");
  if (!x->gpu) XF_FAIL(PIPEMAX_ERR_STATE, "no streams in the host-only mode");
  std::unique_lock<std::mutex> lk(x->mu);
  if (ticket == 0 || ticket >= x->next_ticket) XF_FAIL(PIPEMAX_ERR_ARG, "ticket %llu was never issued", (unsigned long long)ticket);
  auto it = x->live.find(ticket);
  if (it == x->live.end()) return PIPEMAX_OK;           // already complete
  std::shared_ptr<Request> r = it->second;
  x->cv_done.wait(lk, [&] { return r->all_submitted || r->done; });
  if (r->done || !r->ev_last) return PIPEMAX_OK;
  // under the lock: the dispatcher cannot recycle the event while the wait is being enqueued
  hipError_t e = hipStreamWaitEvent((hipStream_t)hip_stream, r->ev_last, 0);
  if (e != hipSuccess) XF_FAIL(PIPEMAX_ERR_HIP, "hipStreamWaitEvent failed: %s", hipGetErrorString(e));
  return PIPEMAX_OK;
}

int pipemax_xfer_drain(pipemax_xfer_t* x) {
  if (!x) XF_FAIL(PIPEMAX_ERR_ARG, "null orchestrator");
  std::unique_lock<std::mutex> lk(x->mu);
  x->cv_done.wait(lk, [&] { return x->live.empty(); });
  if (x->hip_error != hipSuccess) XF_FAIL(PIPEMAX_ERR_HIP, "a copy failed: %s", hipGetErrorString(x->hip_error));
  return PIPEMAX_OK;
}

int pipemax_xfer_get_stats(pipemax_xfer_t* x, pipemax_xfer_stats_t* out) {
  if (!x || !out) XF_FAIL(PIPEMAX_ERR_ARG, "null argument");
  std::lock_guard<std::mutex> lk(x->mu);
  *out = x->stats;
  return PIPEMAX_OK;
}

int pipemax_xfer_reset_stats(pipemax_xfer_t* x) {
  if (!x) XF_FAIL(PIPEMAX_ERR_ARG, "null orchestrator");
  std::lock_guard<std::mutex> lk(x->mu);
  x->stats = pipemax_xfer_stats_t{};
  x->log.clear();
  return PIPEMAX_OK;
}

int pipemax_xfer_get_log(pipemax_xfer_t* x, pipemax_xfer_log_t* out, int capacity) {
  if (!x || (capacity > 0 && !out) || capacity < 0) XF_FAIL(PIPEMAX_ERR_ARG, "null argument or negative capacity");
  std::lock_guard<std::mutex> lk(x->mu);
  const int n = std::min<int>(capacity, (int)x->log.size());
  for (int i = 0; i < n; ++i) out[i] = x->log[i];
  return n;
}

int pipemax_xfer_debug_set_host_us_per_mib(pipemax_xfer_t* x, int us) {
  if (!x || us < 0) XF_FAIL(PIPEMAX_ERR_ARG, "null orchestrator or negative delay");
  std::lock_guard<std::mutex> lk(x->mu);
  x->host_us_per_mib = us;
  return PIPEMAX_OK;
}

int pipemax_xfer_debug_pause(pipemax_xfer_t* x, int paused) {
  if (!x) XF_FAIL(PIPEMAX_ERR_ARG, "null orchestrator");
  {
    std::lock_guard<std::mutex> lk(x->mu);
    x->paused = paused != 0;
  }
  x->cv_work.notify_all();
  return PIPEMAX_OK;
}

}  // extern "C"

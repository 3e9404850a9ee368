// The stage object behind the C ABI: KV page pools and block tables, the three-stream step
// executor, the prefetch / evict paths and the write-back worker.
//
// Streams.  compute = the caller's stream (or the stage's own); h2d = KV prefetch; d2h = KV
// write-back.  All at default priority.
//   decode_step(mb): compute waits for mb's prefetch event; after the kernel that appends the new K,V
//     of a layer (or of the last layer of a group) an event is recorded; the worker thread waits for it,
//     issues the d2h copy of the contiguous staging rows to pinned host memory, waits for the copy and
//     scatters the rows into the host pages.
//   prefetch(mb):   the caller's thread does the bookkeeping (GPU pages, copy runs) and returns; a second
//     worker thread waits until mb's pending write-back has landed in the host replica and until the
//     last reader of every page about to be overwritten has finished (see evict), then issues the page
//     runs on h2d and records mb's prefetch event.  A decode step of mb waits (host side) for that issue
//     before it makes its stream wait for the event.
//   evict(mb):      the GPU pages go back to the free list; the next prefetch is ordered after mb's
//     last step event.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <memory>
#include <mutex>
#include <new>
#include <omp.h>
#include <thread>
#include <vector>

#include "dma_copy.hpp"
#include "kernels.hpp"
#include "pipemax_xfer.h"
#include "kv_pool.hpp"

// Scratch of pipemax_decode_step_noalloc: one copy per GPU, held until the process ends.
static __device__ __align__(256) unsigned char scratch[PIPEMAX_NOALLOC_SCRATCH_BYTES];

namespace pmx {

static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

namespace {

constexpr int kFusedRows = 128;   // up to this many rows take the fused 5-launch-per-layer pipeline
constexpr int kSlots = 4;        // depth of the write-back staging ring
constexpr int kTableRing = 8;    // depth of the block-table upload ring
constexpr int kMaxRunPages = 128;  // longest single prefetch copy, in pages (64 MiB at 512 KiB pages)
enum { ST_HOST = 0, ST_INFLIGHT = 1, ST_GPU = 2 };
enum { TC_H2D = PIPEMAX_N_KCLASS, TC_D2H = PIPEMAX_N_KCLASS + 1, TC_STALL = PIPEMAX_N_KCLASS + 2 };

double now_s() {
  return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// ---- scratch of the entry point that allocates nothing (pipemax_decode_step_noalloc) -------------------------
// One array per GPU, held for the life of the process.  Host code never uses the array's name as an address:
// the device address is looked up once per device (scratch_base) and handed to the kernels as an argument.
constexpr size_t kScratchBytes = PIPEMAX_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mu;

// Device address of this GPU's copy of the scratch array (the device must be current); nullptr + error text on
// failure.
void* scratch_base(int dev) {
  if (dev < 0 || dev >= kMaxDevices) {
    set_error("device %d is outside the %d devices the static scratch is tracked for", dev, kMaxDevices);
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      set_error("hipGetSymbolAddress of the static scratch failed on device %d: %s", dev, hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

// clears n16 16-byte words (a kernel, not a memset node: callers may be under graph capture)
__global__ void k_clear16(uint4* p, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

// copies n 32-bit words from pinned host memory (device-visible) to device memory.  The block table of a step goes
// up this way, by the compute units over the link, not as a host-to-device copy: such a copy would queue on the
// same DMA engine as the KV prefetch and wait behind whatever part of it has been submitted, holding the step up.
__global__ void k_upload_words(int32_t* __restrict__ dst, const int32_t* __restrict__ src, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// The device buffers a step works in besides its inputs, outputs, weights and KV pages (matrix-core engine).
struct Work {
  float* x = nullptr;
  float2* rope_cs = nullptr;
  uint16_t *m_xn_t = nullptr, *m_q = nullptr, *m_attn_t = nullptr, *m_act_t = nullptr;
  float *m_part = nullptr, *m_part_o = nullptr, *m_part_ml = nullptr, *m_ssq = nullptr;
  int *m_cnt_gemm = nullptr, *m_cnt_attn = nullptr;
};

struct SeqState {
  int len = 0;
  int state = ST_HOST;
  std::vector<int32_t> gpu, host;
  std::vector<int32_t> host_reserved;   // pages right after `host`, taken first when the sequence grows
};

struct MicroBatch {
  bool defined = false;
  int alias_of = -1;    // >= 0: shares the host pages of that micro-batch (timing aid, see pipemax_mb_define_alias)
  int b = 0;
  std::vector<SeqState> seq;
  int* d_ctx = nullptr;
  int* d_table = nullptr;   // [maxb][max_pages] page ids, [maxb] row order (longest first), [maxb] lengths
                            // (d_ctx points at the lengths); rows are the sequences of the last step
  bool table_dirty = true;
  hipEvent_t ev_prefetch = nullptr;
  bool prefetch_pending = false;
  uint64_t prefetch_ticket = 0;   // last copy of the prefetch when a transfer orchestrator issues the copies
  hipEvent_t ev_step = nullptr;
  bool stepped = false;
  int wb_pending = 0;   // guarded by Stage::mu
  uint64_t wb_queued = 0, wb_done = 0;   // write-back jobs of this micro-batch ever queued / finished (guarded by mu)
  uint64_t pf_ticket = 0;   // number of the last prefetch job of this micro-batch
};

struct WbJob {
  hipEvent_t ev = nullptr;
  int mb = 0, layer = 0, n_layers = 1, slot = 0, b = 0;
  std::shared_ptr<std::vector<std::pair<int32_t, int>>> where;   // per sequence: host page, slot
  // ev marks the staging rows as written; the worker then issues the device -> host copy itself
  void* copy_dst = nullptr;
  const void* copy_src = nullptr;
  size_t copy_bytes = 0;
  bool timed = false;              // accumulate the copy's duration (the timing flag when the job was queued)
  bool stop = false;
};

struct Timed {
  int cls;
  hipEvent_t a, b;
};

// One prefetch_kv call, handed to the prefetch worker: the copies and what they must wait for.
struct PfJob {
  uint64_t no = 0;                 // running number of the job (MicroBatch::pf_ticket)
  int mb = 0;
  std::vector<CopyRun> runs;
  std::vector<int> release;        // micro-batches evicted since the last prefetch: their last step read the pages
  uint64_t wb_target = 0;          // write-back jobs of mb that must have landed in the host replica first
  bool stream_ordered = false;     // wait for the last readers on the stream instead of on the host
  bool timed = false;
  bool stop = false;
};

struct LayerW {
  void *wqkv = nullptr, *wo = nullptr, *wgu = nullptr, *wd = nullptr, *g1 = nullptr, *g2 = nullptr;
};

struct GemmPlan {
  int split = 1, wn = 8;   // wn: waves (32-column tiles) per work-group of the LDS-staged kernel
  int nwk = 0;             // > 0: barrier-free skinny kernel with nwk waves per work-group
  bool fused_swiglu = false;
};

}  // namespace
}  // namespace pmx

using namespace pmx;

struct pipemax_pool {
  PagePool pool;
  explicit pipemax_pool(int n) : pool(n) {}
};

struct pipemax_stage {
  pipemax_config_t cfg{};
  Dims D{};
  int engine = 0;
  size_t esz = 4;
  size_t page_bytes = 0;
  size_t layer_block_bytes = 0;     // one layer's K,V of one page
  int dev = 0;
  hipStream_t s_own = nullptr, s_h2d = nullptr, s_d2h = nullptr, s_last = nullptr;
  void* gpu_pool = nullptr;
  void* host_pool = nullptr;
  std::unique_ptr<PagePool> gpu_pages, host_pages;
  std::vector<MicroBatch> mbs;
  std::vector<LayerW> w;
  std::vector<void*> dev_allocs;    // everything hipMalloc'ed except the pool
  std::vector<void*> host_allocs;   // everything hipHostMalloc'ed except the pool
  // activations
  float* x = nullptr;
  float2* rope_cs = nullptr;
  float *g_xn = nullptr, *g_qkv = nullptr, *g_q = nullptr, *g_attn = nullptr, *g_gu = nullptr,
        *g_act = nullptr, *g_scores = nullptr;
  uint16_t *m_xn_t = nullptr, *m_q = nullptr, *m_attn_t = nullptr, *m_act_t = nullptr;
  float *m_part = nullptr, *m_part_o = nullptr, *m_part_ml = nullptr, *m_ssq = nullptr;
  int *m_cnt_gemm = nullptr, *m_cnt_attn = nullptr;
  // up to 64 rows: consumers fused into the GEMM epilogues (plans f_*); more: large-tile GEMMs with
  // separate element-wise kernels, planned per call from the row count
  int attn_cp_override = 0;   // PIPEMAX_ATTN_CHUNK_PAGES: tuning override of the attention chunk size
  int attn_worker = 0;        // PIPEMAX_ATTN_KERNEL=wave|group: tuning override of the attention kernel choice
  GemmPlan f_qkv, f_o, f_gu, f_d;
  int nch_alloc = 1;
  float* layer_out = nullptr;
  int last_b = 0;
  // write-back ring
  void* d_stage[kSlots] = {};
  void* h_stage[kSlots] = {};
  std::vector<hipEvent_t> ev_ready[kSlots];
  int slot_pending[kSlots] = {};   // guarded by mu
  uint64_t step_no = 0;
  // table upload ring
  int32_t* h_table[kTableRing] = {};
  hipEvent_t ev_table[kTableRing] = {};
  bool table_used[kTableRing] = {};
  int table_pos = 0;
  std::vector<int> release_wait;   // micro-batches evicted since the last prefetch (host-ordered mode)
  // ordering of growth pages against cancelled prefetches
  hipEvent_t ev_h2d_fence = nullptr;
  bool h2d_fence_pending = false;
  pipemax_xfer_t* xfer = nullptr;   // not owned: issues the prefetch copies when attached
  void* scratch_dev = nullptr;      // device address of this GPU's static scratch (pipemax_decode_step_noalloc)
  bool no_timing_now = false;       // the current step must not create events
  // worker
  std::thread worker;
  std::mutex mu;
  std::condition_variable cv_job, cv_done;
  std::deque<WbJob> jobs;
  bool worker_started = false;
  // prefetch worker: issues the copies of prefetch_kv once their conditions hold
  std::thread pf_worker;
  std::condition_variable cv_pf, cv_pf_done;
  std::deque<PfJob> pf_jobs;            // guarded by mu
  uint64_t pf_queued = 0, pf_issued = 0;   // jobs handed over / issued on the stream (guarded by mu)
  int pf_error = 0;                     // guarded by mu: status of the first failing job
  char pf_error_text[256] = "";
  std::vector<Timed> pf_timed;          // guarded by mu: event pairs the prefetch worker recorded
  std::vector<hipEvent_t> pf_ev_free;   // guarded by mu
  // test hooks
  std::atomic<int> dly_h2d{0}, dly_d2h{0}, dly_worker{0};
  int worker_hip_error = 0;        // guarded by mu: first failure of a copy the worker issued
  DmaCopy* dma = nullptr;          // write-back copies on the DMA engines (nullptr: the runtime's own copies)
  // stats / timing
  pipemax_stats_t st{};
  std::vector<Timed> timed;
  std::vector<hipEvent_t> ev_free;

  // ---- helpers ---------------------------------------------------------------------------------
  bool timing() const { return (cfg.flags & PIPEMAX_FLAG_TIME_KERNELS) && !no_timing_now; }
  hipEvent_t get_event() {
    if (!ev_free.empty()) {
      hipEvent_t e = ev_free.back();
      ev_free.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  bool t_open = false;
  void tbegin(int cls, hipStream_t s) {
    t_open = false;
    if (!timing()) return;
    if ((cfg.flags & PIPEMAX_FLAG_TIME_ATTN_ONLY) && cls != PIPEMAX_K_ATTN && cls != TC_STALL) return;
    if (timed.size() >= 4096) resolve_timers(true);
    Timed t{cls, get_event(), get_event()};
    if (!t.a || !t.b) return;
    (void)hipEventRecord(t.a, s);
    timed.push_back(t);
    t_open = true;
  }
  // a pair of events for a launch that stamps them itself; nullptr when this class is not being timed
  Timed* tpair(int cls) {
    t_open = false;
    if (!timing()) return nullptr;
    if ((cfg.flags & PIPEMAX_FLAG_TIME_ATTN_ONLY) && cls != PIPEMAX_K_ATTN) return nullptr;
    if (timed.size() >= 4096) resolve_timers(true);
    Timed t{cls, get_event(), get_event()};
    if (!t.a || !t.b) return nullptr;
    timed.push_back(t);
    return &timed.back();
  }
  void tend(hipStream_t s) {
    if (!t_open) return;
    (void)hipEventRecord(timed.back().b, s);
    t_open = false;
  }
  // only_ready: keep the pairs whose second event has not completed yet
  void resolve_timers(bool only_ready = false) {
    std::vector<Timed> keep, from_pf, back_pf;
    {
      std::lock_guard<std::mutex> lk(mu);
      from_pf.swap(pf_timed);
    }
    for (auto& t : from_pf) {          // pairs of the prefetch worker; their events go back to its own free list
      float ms = 0.f;
      if (hipEventQuery(t.b) != hipSuccess) {
        back_pf.push_back(t);
        continue;
      }
      if (hipEventElapsedTime(&ms, t.a, t.b) == hipSuccess) st.h2d_ms += ms;
      std::lock_guard<std::mutex> lk(mu);
      pf_ev_free.push_back(t.a);
      pf_ev_free.push_back(t.b);
    }
    if (!back_pf.empty()) {
      std::lock_guard<std::mutex> lk(mu);
      pf_timed.insert(pf_timed.begin(), back_pf.begin(), back_pf.end());
    }
    for (auto& t : timed) {
      float ms = 0.f;
      if (only_ready && hipEventQuery(t.b) != hipSuccess) {
        keep.push_back(t);
        continue;
      }
      if (hipEventElapsedTime(&ms, t.a, t.b) == hipSuccess) {
        if (t.cls < PIPEMAX_N_KCLASS) {
          st.kernel_ms[t.cls] += ms;
          st.kernel_launches[t.cls] += 1;
        } else if (t.cls == TC_STALL) {
          st.prefetch_stall_ms += ms;
          st.prefetch_stalls += 1;
        } else if (t.cls == TC_H2D) {
          st.h2d_ms += ms;
        } else {
          st.d2h_ms += ms;
        }
      }
      ev_free.push_back(t.a);
      ev_free.push_back(t.b);
    }
    timed.swap(keep);
  }
  char* host_page_ptr(int32_t page) const { return (char*)host_pool + (size_t)page * page_bytes; }
  bool layer_major() const { return cfg.flags & PIPEMAX_FLAG_DEVICE_LAYER_MAJOR; }
  // a whole page on the device: block-first pools only
  char* gpu_page_ptr(int32_t page) const { return (char*)gpu_pool + (size_t)page * page_bytes; }
  // one layer's block of a page on the device, either pool layout
  char* gpu_block_ptr(int32_t page, int layer) const {
    return (char*)gpu_pool + ((size_t)page * D.page_stride + (size_t)layer * D.layer_stride) * esz;
  }
  void wait_mb_writeback(int mb) {
    std::unique_lock<std::mutex> lk(mu);
    if (mbs[mb].wb_pending == 0) return;
    double t0 = now_s();
    cv_done.wait(lk, [&] { return mbs[mb].wb_pending == 0; });
    st.host_wait_s += now_s() - t0;
  }
  // blocks until the prefetch worker has issued job `no` (0 = nothing to wait for)
  void wait_pf(uint64_t no) {
    std::unique_lock<std::mutex> lk(mu);
    if (pf_issued >= no) return;
    double t0 = now_s();
    cv_pf_done.wait(lk, [&] { return pf_issued >= no; });
    st.host_wait_s += now_s() - t0;
  }
  void wait_slot(int slot) {
    std::unique_lock<std::mutex> lk(mu);
    if (slot_pending[slot] == 0) return;
    double t0 = now_s();
    cv_done.wait(lk, [&] { return slot_pending[slot] == 0; });
    st.host_wait_s += now_s() - t0;
  }
  void wait_all_writeback() {
    std::unique_lock<std::mutex> lk(mu);
    cv_done.wait(lk, [&] {
      if (!jobs.empty()) return false;
      for (int s = 0; s < kSlots; ++s)
        if (slot_pending[s]) return false;
      return true;
    });
  }
};

namespace {

// ---- element scatter between the canonical [tok][Hkv][d] layout and a page -----------------------
template <typename T>
void scatter_token(const pipemax_stage* st, T* page, int layer, int slot, const T* k_row, const T* v_row) {
  const int Hkv = st->D.Hkv, d = st->D.d;
  for (int head = 0; head < Hkv; ++head) {
    T* ks = page + sub_block_off(Hkv, d, layer, head, 0);
    T* vs = page + sub_block_off(Hkv, d, layer, head, 1);
    if (k_row) {
      const T* kr = k_row + (size_t)head * d;
      for (int dd = 0; dd < d; dd += 8) memcpy(ks + k_sub_idx(slot, dd), kr + dd, 8 * sizeof(T));
    }
    if (v_row) {
      const T* vr = v_row + (size_t)head * d;
      for (int dd = 0; dd < d; ++dd) vs[v_sub_idx(slot, dd)] = vr[dd];
    }
  }
}
// n consecutive tokens of one sequence (slots slot0 .. slot0 + n - 1 of one page; their staging rows lie
// `stride` elements apart): in the page the 8-element K pieces of consecutive tokens are adjacent, and so are
// the V elements of four consecutive tokens, so a run is written in 16-byte / 4-element pieces instead of
// element by element (a prefill chunk hands over thousands of rows per layer).
template <typename T>
void scatter_run(const pipemax_stage* st, T* page, int layer, int slot0, int n, const T* k_rows, const T* v_rows,
                 size_t stride) {
  const int Hkv = st->D.Hkv, d = st->D.d;
  for (int head = 0; head < Hkv; ++head) {
    T* ks = page + sub_block_off(Hkv, d, layer, head, 0);
    T* vs = page + sub_block_off(Hkv, d, layer, head, 1);
    for (int dd = 0; dd < d; dd += 8) {
      T* dst = ks + k_sub_idx(slot0, dd);
      const T* src = k_rows + (size_t)head * d + dd;
      for (int t = 0; t < n; ++t) memcpy(dst + (size_t)t * 8, src + (size_t)t * stride, 8 * sizeof(T));
    }
    int t = 0;
    for (; t < n && ((slot0 + t) & 3); ++t) {          // tokens in front of the first aligned group of four
      const T* vr = v_rows + (size_t)t * stride + (size_t)head * d;
      for (int dd = 0; dd < d; ++dd) vs[v_sub_idx(slot0 + t, dd)] = vr[dd];
    }
    for (; t + 4 <= n; t += 4) {
      const T* v0 = v_rows + (size_t)t * stride + (size_t)head * d;
      const T *v1 = v0 + stride, *v2 = v1 + stride, *v3 = v2 + stride;
      for (int dd = 0; dd < d; ++dd) {
        const T quad[4] = {v0[dd], v1[dd], v2[dd], v3[dd]};
        memcpy(vs + v_sub_idx(slot0 + t, dd), quad, sizeof(quad));
      }
    }
    for (; t < n; ++t) {
      const T* vr = v_rows + (size_t)t * stride + (size_t)head * d;
      for (int dd = 0; dd < d; ++dd) vs[v_sub_idx(slot0 + t, dd)] = vr[dd];
    }
  }
}
template <typename T>
void gather_token(const pipemax_stage* st, const T* page, int layer, int slot, T* k_row, T* v_row) {
  const int Hkv = st->D.Hkv, d = st->D.d;
  for (int head = 0; head < Hkv; ++head) {
    const T* ks = page + sub_block_off(Hkv, d, layer, head, 0);
    const T* vs = page + sub_block_off(Hkv, d, layer, head, 1);
    if (k_row)
      for (int dd = 0; dd < d; dd += 8) memcpy(k_row + (size_t)head * d + dd, ks + k_sub_idx(slot, dd), 8 * sizeof(T));
    if (v_row)
      for (int dd = 0; dd < d; ++dd) v_row[(size_t)head * d + dd] = vs[v_sub_idx(slot, dd)];
  }
}

// Threads of the re-layout team.  They must not saturate the host: the HIP runtime resolves cross-stream event
// waits in host threads of its own, and with every core spinning in OpenMP the compute stream was seen to stall
// for 1-2 ms per prefill pass behind the write-back copy.  So: at most half of the available threads (8 at most;
// PIPEMAX_RELAYOUT_THREADS overrides), and the team sleeps as soon as a job is done instead of spinning for the
// runtime's default 200 ms.
int relayout_threads() {
  static const int n = [] {
    int t = std::max(1, std::min(8, omp_get_max_threads() / 2));
    if (const char* e = getenv("PIPEMAX_RELAYOUT_THREADS")) t = std::max(1, std::min(64, atoi(e)));
    return t;
  }();
  return n;
}

void worker_main(pipemax_stage* st) {
  (void)hipSetDevice(st->dev);
  kmp_set_blocktime(0);
  for (;;) {
    WbJob job;
    {
      std::unique_lock<std::mutex> lk(st->mu);
      st->cv_job.wait(lk, [&] { return !st->jobs.empty(); });
      job = st->jobs.front();
      st->jobs.pop_front();
    }
    if (job.stop) return;
    (void)hipEventSynchronize(job.ev);
    {
      if (int us = st->dly_d2h.load()) std::this_thread::sleep_for(std::chrono::microseconds(us));
      const double t0 = now_s();
      hipError_t e = hipSuccess;
      if (st->dma) {
        if (dma_copy_d2h(st->dma, job.copy_dst, job.copy_src, job.copy_bytes) != 0) e = hipErrorUnknown;
      } else {
        e = hipMemcpyAsync(job.copy_dst, job.copy_src, job.copy_bytes, hipMemcpyDeviceToHost, st->s_d2h);
        if (e == hipSuccess) e = hipStreamSynchronize(st->s_d2h);
      }
      std::lock_guard<std::mutex> lk(st->mu);
      if (e != hipSuccess && !st->worker_hip_error) st->worker_hip_error = (int)e;
      if (job.timed) st->st.d2h_ms += (now_s() - t0) * 1e3;
    }
    if (int us = st->dly_worker.load()) std::this_thread::sleep_for(std::chrono::microseconds(us));
    const size_t row = (size_t)st->D.Hkv * st->D.d;                       // elements of one K (or V) row
    const size_t layer_elems = (size_t)st->cfg.max_seqs_per_mb * 2 * row;  // staging of one layer
    // rows write disjoint token slots, so a prefill chunk (hundreds of rows) is spread over the host cores;
    // its rows are consecutive tokens, which are written run by run (rows of one page, consecutive slots)
    std::vector<std::pair<int, int>> runs;      // (first row, length)
    for (int i = 0; i < job.b;) {
      int n = 1;
      while (i + n < job.b && (*job.where)[i + n].first == (*job.where)[i].first &&
             (*job.where)[i + n].second == (*job.where)[i].second + n)
        ++n;
      runs.emplace_back(i, n);
      i += n;
    }
    const int n_runs = (int)runs.size();
    const int n_items = job.n_layers * n_runs;
#pragma omp parallel for schedule(static) num_threads(relayout_threads()) if (job.n_layers * job.b >= 1024)
    for (int item = 0; item < n_items; ++item) {
      const int layer = job.layer + item / n_runs;
      const char* src = (const char*)st->h_stage[job.slot] + (size_t)layer * layer_elems * st->esz;
      const int i = runs[item % n_runs].first, n = runs[item % n_runs].second;
      const auto& wh = (*job.where)[i];
      char* page = st->host_page_ptr(wh.first);
      const char* kr = src + ((size_t)i * 2 + 0) * row * st->esz;
      const char* vr = src + ((size_t)i * 2 + 1) * row * st->esz;
      if (st->esz == 4)
        scatter_run<float>(st, (float*)page, layer, wh.second, n, (const float*)kr, (const float*)vr, 2 * row);
      else
        scatter_run<uint16_t>(st, (uint16_t*)page, layer, wh.second, n, (const uint16_t*)kr, (const uint16_t*)vr,
                              2 * row);
    }
    {
      std::lock_guard<std::mutex> lk(st->mu);
      st->mbs[job.mb].wb_pending -= 1;
      st->mbs[job.mb].wb_done += 1;
      st->slot_pending[job.slot] -= 1;
      st->st.relayout_jobs += job.n_layers;
    }
    st->cv_done.notify_all();
  }
}

void host_sleep_cb(void* arg) {
  std::this_thread::sleep_for(std::chrono::microseconds((intptr_t)arg));
}

// The prefetch worker.  A job's copies may start once (1) the write-back of its micro-batch that was pending when
// prefetch_kv was called has landed in the host replica and (2) the last decode step of every micro-batch evicted
// since the previous prefetch has finished reading the pages that are handed out again.  Both waits used to be
// taken by the caller inside prefetch_kv, which kept it from enqueuing the next decode step meanwhile.
void pf_worker_main(pipemax_stage* st) {
  (void)hipSetDevice(st->dev);
  for (;;) {
    PfJob job;
    {
      std::unique_lock<std::mutex> lk(st->mu);
      st->cv_pf.wait(lk, [&] { return !st->pf_jobs.empty(); });
      job = std::move(st->pf_jobs.front());
      st->pf_jobs.pop_front();
      if (job.stop) return;
      st->cv_done.wait(lk, [&] { return st->mbs[job.mb].wb_done >= job.wb_target; });
    }
    MicroBatch& M = st->mbs[job.mb];
    int status = PIPEMAX_OK;
    char text[256] = "";
    auto fail_hip = [&](hipError_t e, const char* what) {
      if (e == hipSuccess || status != PIPEMAX_OK) return;
      status = PIPEMAX_ERR_HIP;
      snprintf(text, sizeof(text), "prefetch worker: %s failed: %s", what, hipGetErrorString(e));
    };
    for (int k : job.release) {
      if (job.stream_ordered) fail_hip(hipStreamWaitEvent(st->s_h2d, st->mbs[k].ev_step, 0), "hipStreamWaitEvent");
      else fail_hip(hipEventSynchronize(st->mbs[k].ev_step), "hipEventSynchronize");
    }
    if (int us = st->dly_h2d.load())
      fail_hip(hipLaunchHostFunc(st->s_h2d, host_sleep_cb, (void*)(intptr_t)us), "hipLaunchHostFunc");
    uint64_t ticket = 0;
    if (st->xfer) {
      // the orchestrator cuts the runs into chunks and feeds them to the link behind any urgent copy; bulk
      // requests of one direction complete in order, so the last ticket stands for the whole prefetch
      for (const CopyRun& r : job.runs) {
        if (status != PIPEMAX_OK) break;
        int rc = pipemax_xfer_submit(st->xfer, PIPEMAX_XFER_BULK, PIPEMAX_XFER_H2D, st->gpu_page_ptr(r.dst),
                                     st->host_page_ptr(r.src), (size_t)r.count * st->page_bytes, &ticket);
        if (rc != PIPEMAX_OK) {
          status = rc;
          snprintf(text, sizeof(text), "prefetch worker: the transfer orchestrator refused a copy (%d)", rc);
        }
      }
    } else {
      Timed t{TC_H2D, nullptr, nullptr};
      if (job.timed) {
        std::lock_guard<std::mutex> lk(st->mu);
        if (st->pf_ev_free.size() >= 2) {
          t.a = st->pf_ev_free.back(); st->pf_ev_free.pop_back();
          t.b = st->pf_ev_free.back(); st->pf_ev_free.pop_back();
        }
      }
      if (job.timed && !t.a && (hipEventCreate(&t.a) != hipSuccess || hipEventCreate(&t.b) != hipSuccess)) t.a = t.b = nullptr;
      if (t.a) fail_hip(hipEventRecord(t.a, st->s_h2d), "hipEventRecord");
      if (st->layer_major()) {
        // block-first host pages into the [layer][page] pool: per run one strided copy per layer (rows = pages,
        // one page apart in host memory, packed on the device)
        for (const CopyRun& r : job.runs)
          for (int l = 0; l < st->cfg.n_layers; ++l)
            fail_hip(hipMemcpy2DAsync(st->gpu_block_ptr(r.dst, l), st->layer_block_bytes,
                                      st->host_page_ptr(r.src) + (size_t)l * st->layer_block_bytes, st->page_bytes,
                                      st->layer_block_bytes, (size_t)r.count, hipMemcpyHostToDevice, st->s_h2d),
                     "hipMemcpy2DAsync");
      } else {
        for (const CopyRun& r : job.runs)
          fail_hip(hipMemcpyAsync(st->gpu_page_ptr(r.dst), st->host_page_ptr(r.src), (size_t)r.count * st->page_bytes,
                                  hipMemcpyHostToDevice, st->s_h2d), "hipMemcpyAsync");
      }
      if (t.a) {
        fail_hip(hipEventRecord(t.b, st->s_h2d), "hipEventRecord");
        std::lock_guard<std::mutex> lk(st->mu);
        st->pf_timed.push_back(t);
      }
      fail_hip(hipEventRecord(M.ev_prefetch, st->s_h2d), "hipEventRecord");
    }
    {
      std::lock_guard<std::mutex> lk(st->mu);
      M.prefetch_ticket = ticket;
      st->pf_issued = job.no;
      if (status != PIPEMAX_OK && st->pf_error == PIPEMAX_OK) {
        st->pf_error = status;
        snprintf(st->pf_error_text, sizeof(st->pf_error_text), "%s", text);
      }
    }
    st->cv_pf_done.notify_all();
  }
}

template <typename T>
int dev_alloc(pipemax_stage* st, T** p, size_t count) {
  void* q = nullptr;
  if (count == 0) count = 1;
  hipError_t e = hipMalloc(&q, count * sizeof(T));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    PMX_FAIL(PIPEMAX_ERR_OOM_DEVICE, "hipMalloc of %zu bytes failed: %s", count * sizeof(T),
             hipGetErrorString(e));
  }
  st->dev_allocs.push_back(q);
  *p = (T*)q;
  return PIPEMAX_OK;
}
template <typename T>
int host_alloc(pipemax_stage* st, T** p, size_t count) {
  void* q = nullptr;
  if (count == 0) count = 1;
  hipError_t e = hipHostMalloc(&q, count * sizeof(T), hipHostMallocDefault);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    PMX_FAIL(PIPEMAX_ERR_OOM_HOST, "hipHostMalloc of %zu bytes failed: %s", count * sizeof(T),
             hipGetErrorString(e));
  }
  st->host_allocs.push_back(q);
  *p = (T*)q;
  return PIPEMAX_OK;
}

// M <= 64: barrier-free kernel.  Measured on MI355X: about 256 work-groups of 8 waves (or, when the
// matrix alone has >= 384 column pairs, 4 waves and no split) stream fastest.
GemmPlan plan_gemm_skinny(int N, int K, bool swiglu) {
  GemmPlan p;
  const int bn = N / 64, KT = K / 16;
  p.fused_swiglu = swiglu;
  p.nwk = (bn >= 384) ? 4 : 8;
  int S = swiglu ? 1 : std::max(1, 256 / bn);
  S = std::max(1, std::min(S, KT / (p.nwk * 4)));
  const int ksp = (KT + S - 1) / S;
  p.split = (KT + ksp - 1) / ksp;
  return p;
}

// More than 128 rows: large-tile kernel, one work-group (256 rows x 256 columns) per CU.  The K split is the
// one with the lowest modelled time: work-groups run in rounds of 256 (one per compute unit), a work-group takes
// a fixed start / store cost plus its share of the k-steps, and every split adds one fp32 partial of the output
// that is written here and read by the consumer.  (Constants measured on the ring kernel: 0.42 us per k-step
// and work-group, 4.5 us per work-group, partials at an effective 4 TB/s.)  A plain "about 256 work-groups" rule
// picks 3 splits for 96 column-row blocks -- 288 work-groups, i.e. two rounds -- where 2 splits are 25 % faster.
GemmPlan plan_gemm_large(int N, int K, int M) {
  GemmPlan p;
  p.wn = 0;
  const int rb = (M + 255) / 256, bn = (N / 256) * rb, KT = K / 16;
  const double part_us = (double)rb * 256 * N * 8.0 / 4.0e6;
  int best = 1;
  double best_cost = 0.0;
  for (int S = 1; S <= std::max(1, std::min(16, KT / 16)); ++S) {
    int ksp = (KT + S - 1) / S;
    if (KT % 2 == 0) ksp += ksp & 1;      // the ring kernel works on pairs of k-steps
    const int split = (KT + ksp - 1) / ksp;
    const int rounds = (bn * split + 255) / 256;
    double cost = rounds * (0.42 * ksp + 4.5) + (split > 1 ? split * part_us : 0.0);
    // One row block: every work-group streams weights of its own, and at the ring kernel's rate 256 of them ask for
    // about 5 TB/s.  A round that needs (nearly) every compute unit then runs 10-25 % longer than one that leaves an
    // eighth of them free (256 rows, 32 tiles x 6 / 7 / 8 splits of k = 8192: 46.7 / 49.7 / 57.8 us).  With several
    // row blocks the weight tiles are shared through L2 and the full round is the faster one (1024 rows: 0.68 vs 0.72 ms).
    if (rb == 1 && bn * split - (rounds - 1) * 256 > 224) cost += 0.25 * (0.42 * ksp + 4.5);
    if (S == 1 || cost < best_cost) {
      best = split;
      best_cost = cost;
    }
  }
  p.split = best;
  return p;
}

GemmPlan plan_gemm(int N, int K);
GemmPlan plan_rows(int N, int K, int M) { return (N % 256 == 0) ? plan_gemm_large(N, K, M) : plan_gemm(N, K); }

GemmPlan plan_gemm(int N, int K) {
  GemmPlan p;
  p.wn = (N % 256 == 0) ? 8 : 4;
  const int groups = N / (32 * p.wn);
  const int KT = K / 16;
  int S = (512 + groups - 1) / groups;
  S = std::max(1, std::min(S, std::max(1, KT / 16)));
  const int ksp = (KT + S - 1) / S;
  p.split = (KT + ksp - 1) / ksp;
  return p;
}

bool mfma_shape_ok(const pipemax_config_t& c) {
  const int nq = c.n_q_heads * c.head_dim;
  return c.dtype == PIPEMAX_BF16 && c.head_dim == 128 && c.hidden % 128 == 0 && c.ffn % 64 == 0 &&
         nq % 16 == 0 && c.n_q_heads / c.n_kv_heads <= 16 &&
         // more than 256 rows per pass (prefill chunks) need the large-tile GEMM for every matrix
         (c.max_seqs_per_mb <= 256 ||
          (c.max_seqs_per_mb <= 4096 && (nq + 2 * c.n_kv_heads * c.head_dim) % 256 == 0 && c.hidden % 256 == 0 &&
           (2 * c.ffn) % 256 == 0));
}

void destroy_impl(pipemax_stage* st) {
  if (!st) return;
  (void)hipSetDevice(st->dev);
  if (st->worker_started) {
    {
      std::lock_guard<std::mutex> lk(st->mu);
      WbJob stop;
      stop.stop = true;
      st->jobs.push_back(stop);
    }
    st->cv_job.notify_all();
    st->worker.join();
    {
      std::lock_guard<std::mutex> lk(st->mu);
      PfJob stop;
      stop.stop = true;
      st->pf_jobs.push_back(stop);
    }
    st->cv_pf.notify_all();
    st->pf_worker.join();
    dma_copy_destroy(st->dma);
    st->dma = nullptr;
  }
  (void)hipDeviceSynchronize();
  st->timed.clear();
  for (auto& t : st->pf_timed) {
    (void)hipEventDestroy(t.a);
    (void)hipEventDestroy(t.b);
  }
  for (auto e : st->pf_ev_free) (void)hipEventDestroy(e);
  for (auto e : st->ev_free) (void)hipEventDestroy(e);
  for (auto& mb : st->mbs) {
    if (mb.ev_prefetch) (void)hipEventDestroy(mb.ev_prefetch);
    if (mb.ev_step) (void)hipEventDestroy(mb.ev_step);
  }
  for (int s = 0; s < kSlots; ++s) {
    for (auto e : st->ev_ready[s]) (void)hipEventDestroy(e);
  }
  for (int r = 0; r < kTableRing; ++r)
    if (st->ev_table[r]) (void)hipEventDestroy(st->ev_table[r]);
  if (st->ev_h2d_fence) (void)hipEventDestroy(st->ev_h2d_fence);
  for (void* p : st->dev_allocs) (void)hipFree(p);
  for (void* p : st->host_allocs) (void)hipHostFree(p);
  if (st->gpu_pool) (void)hipFree(st->gpu_pool);
  if (st->host_pool) (void)hipHostFree(st->host_pool);
  if (st->s_own) (void)hipStreamDestroy(st->s_own);
  if (st->s_h2d) (void)hipStreamDestroy(st->s_h2d);
  if (st->s_d2h) (void)hipStreamDestroy(st->s_d2h);
  delete st;
}

int check_mb(pipemax_stage* st, int mb, bool must_be_defined) {
  if (!st) PMX_FAIL(PIPEMAX_ERR_ARG, "null stage");
  if (mb < 0 || mb >= st->cfg.n_microbatches) PMX_FAIL(PIPEMAX_ERR_ARG, "micro-batch %d out of range", mb);
  if (must_be_defined && !st->mbs[mb].defined) PMX_FAIL(PIPEMAX_ERR_ARG, "micro-batch %d is not defined", mb);
  return PIPEMAX_OK;
}

// resolves a (seq_ids, n) argument into a list of distinct valid sequence indices
int seq_list(pipemax_stage* st, int mb, const int32_t* ids, int n, std::vector<int>& out) {
  MicroBatch& M = st->mbs[mb];
  out.clear();
  if (!ids) {
    for (int i = 0; i < M.b; ++i) out.push_back(i);
    return PIPEMAX_OK;
  }
  if (n < 0) PMX_FAIL(PIPEMAX_ERR_ARG, "negative sequence count");
  std::vector<char> seen(M.b, 0);
  for (int k = 0; k < n; ++k) {
    if (ids[k] < 0 || ids[k] >= M.b) PMX_FAIL(PIPEMAX_ERR_ARG, "sequence %d out of range", ids[k]);
    if (!seen[ids[k]]) {
      seen[ids[k]] = 1;
      out.push_back(ids[k]);
    }
  }
  return PIPEMAX_OK;
}

int kv_rw_check(pipemax_stage* st, int mb, int seq, int layer, int tok0, int ntok) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  MicroBatch& M = st->mbs[mb];
  if (seq < 0 || seq >= M.b) PMX_FAIL(PIPEMAX_ERR_ARG, "sequence %d out of range", seq);
  if (layer < 0 || layer >= st->cfg.n_layers) PMX_FAIL(PIPEMAX_ERR_ARG, "layer %d out of range", layer);
  if (tok0 < 0 || ntok < 0 || tok0 + ntok > M.seq[seq].len)
    PMX_FAIL(PIPEMAX_ERR_ARG, "token range [%d, %d) outside the sequence's %d tokens", tok0, tok0 + ntok,
             M.seq[seq].len);
  return PIPEMAX_OK;
}

}  // namespace

// =================================================================================================
// C ABI
// =================================================================================================
extern "C" {

const char* pipemax_last_error(void) { return g_err; }
const char* pipemax_version(void) { return "pipemax-stage 0.1 (gfx950)"; }

int pipemax_stage_create(const pipemax_config_t* cfg, pipemax_stage_t** out) {
  if (!cfg || !out) PMX_FAIL(PIPEMAX_ERR_ARG, "null argument");
  *out = nullptr;
  const pipemax_config_t& c = *cfg;
  if (c.n_layers < 1 || c.hidden < 8 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.head_dim < 32 ||
      c.ffn < 1 || c.n_microbatches < 1 || c.max_seqs_per_mb < 1 || c.max_ctx < 1)
    PMX_FAIL(PIPEMAX_ERR_ARG, "non-positive shape field");
  if (c.dtype != PIPEMAX_F32 && c.dtype != PIPEMAX_BF16) PMX_FAIL(PIPEMAX_ERR_ARG, "unknown dtype %d", c.dtype);
  if (c.host_reserve_tokens < 0 || c.wb_layers_per_copy < 0) PMX_FAIL(PIPEMAX_ERR_ARG, "negative reserve / write-back group");
  if (c.page_tokens != kPageTokens) PMX_FAIL(PIPEMAX_ERR_ARG, "page_tokens must be %d", kPageTokens);
  if (c.n_q_heads % c.n_kv_heads) PMX_FAIL(PIPEMAX_ERR_ARG, "n_q_heads must be a multiple of n_kv_heads");
  if (c.head_dim % 32 || c.head_dim > 512) PMX_FAIL(PIPEMAX_ERR_ARG, "head_dim must be a multiple of 32, at most 512");
  if (c.max_seqs_per_mb > 65535) PMX_FAIL(PIPEMAX_ERR_ARG, "max_seqs_per_mb too large");
  if (!(c.rope_base > 1.0f) || !(c.rms_eps >= 0.0f)) PMX_FAIL(PIPEMAX_ERR_ARG, "bad rope_base / rms_eps");
  int ndev = 0;
  PMX_HIP(hipGetDeviceCount(&ndev));
  if (c.device < 0 || c.device >= ndev) PMX_FAIL(PIPEMAX_ERR_ARG, "device %d not present (%d devices)", c.device, ndev);

  pipemax_stage* st = new (std::nothrow) pipemax_stage();
  if (!st) PMX_FAIL(PIPEMAX_ERR_OOM_HOST, "out of host memory");
  st->cfg = c;
  st->dev = c.device;
  st->esz = (c.dtype == PIPEMAX_F32) ? 4 : 2;
  Dims& D = st->D;
  D.n_layers = c.n_layers; D.h = c.hidden; D.Hq = c.n_q_heads; D.Hkv = c.n_kv_heads; D.d = c.head_dim;
  D.F = c.ffn; D.Nqkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim; D.G = c.n_q_heads / c.n_kv_heads;
  D.rope_base = c.rope_base; D.eps = c.rms_eps;
  D.max_pages = (c.max_ctx + kPageTokens - 1) / kPageTokens;
  D.max_ctx_pad = D.max_pages * kPageTokens;
  D.page_elems = page_elems(c.n_layers, c.n_kv_heads, c.head_dim);
  st->page_bytes = (size_t)D.page_elems * st->esz;
  st->layer_block_bytes = st->page_bytes / c.n_layers;
  st->engine = (mfma_shape_ok(c) && !(c.flags & PIPEMAX_FLAG_FORCE_GENERIC)) ? 1 : 0;
  const int n_gpu_pages = (int)std::min<uint64_t>(c.gpu_kv_bytes / st->page_bytes, 1u << 30);
  const int n_host_pages = (int)std::min<uint64_t>(c.host_kv_bytes / st->page_bytes, 1u << 30);
  if (n_gpu_pages < 1 || n_host_pages < 1) {
    delete st;
    PMX_FAIL(PIPEMAX_ERR_ARG, "pools must hold at least one page of %zu bytes", st->page_bytes);
  }
  {
    const int64_t block = D.page_elems / c.n_layers;      // one layer's K,V of one page
    if (c.flags & PIPEMAX_FLAG_DEVICE_LAYER_MAJOR) {
      D.page_stride = block;
      D.layer_stride = (int64_t)n_gpu_pages * block;
    } else {
      D.page_stride = D.page_elems;
      D.layer_stride = block;
    }
  }

#define PMX_TRY(expr)           \
  do {                          \
    int rc_ = (expr);           \
    if (rc_ != PIPEMAX_OK) {    \
      destroy_impl(st);         \
      return rc_;               \
    }                           \
  } while (0)
#define PMX_TRY_HIP(expr)                                                                       \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess) {                                                                     \
      set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__);     \
      destroy_impl(st);                                                                         \
      return PIPEMAX_ERR_HIP;                                                                   \
    }                                                                                           \
  } while (0)

  PMX_TRY_HIP(hipSetDevice(st->dev));
  st->scratch_dev = scratch_base(st->dev);       // this device's copy of the static scratch
  if (!st->scratch_dev) {
    destroy_impl(st);
    return PIPEMAX_ERR_HIP;
  }
  PMX_TRY_HIP(hipStreamCreateWithFlags(&st->s_own, hipStreamNonBlocking));
  PMX_TRY_HIP(hipStreamCreateWithFlags(&st->s_h2d, hipStreamNonBlocking));
  PMX_TRY_HIP(hipStreamCreateWithFlags(&st->s_d2h, hipStreamNonBlocking));
  st->s_last = st->s_own;

  // pools
  {
    hipError_t e = hipMalloc(&st->gpu_pool, (size_t)n_gpu_pages * st->page_bytes);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      set_error("hipMalloc of the GPU page pool (%zu bytes) failed: %s", (size_t)n_gpu_pages * st->page_bytes,
                hipGetErrorString(e));
      st->gpu_pool = nullptr;
      destroy_impl(st);
      return PIPEMAX_ERR_OOM_DEVICE;
    }
    e = hipHostMalloc(&st->host_pool, (size_t)n_host_pages * st->page_bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      set_error("hipHostMalloc of the host page pool (%zu bytes) failed: %s",
                (size_t)n_host_pages * st->page_bytes, hipGetErrorString(e));
      st->host_pool = nullptr;
      destroy_impl(st);
      return PIPEMAX_ERR_OOM_HOST;
    }
    // unused slots of every page must hold finite values (the attention kernel multiplies them by 0)
    memset(st->host_pool, 0, (size_t)n_host_pages * st->page_bytes);
    PMX_TRY_HIP(hipMemset(st->gpu_pool, 0, (size_t)n_gpu_pages * st->page_bytes));
  }
  st->gpu_pages.reset(new PagePool(n_gpu_pages));
  st->host_pages.reset(new PagePool(n_host_pages));

  const int maxb = c.max_seqs_per_mb;
  const int h = c.hidden, F = c.ffn, nq = c.n_q_heads * c.head_dim;
  st->mbs.resize(c.n_microbatches);
  for (auto& M : st->mbs) {
    PMX_TRY(dev_alloc(st, &M.d_table, (size_t)maxb * D.max_pages + 2 * (size_t)maxb));
    PMX_TRY_HIP(hipMemset(M.d_table, 0, ((size_t)maxb * D.max_pages + 2 * (size_t)maxb) * sizeof(int)));
    M.d_ctx = M.d_table + (size_t)maxb * D.max_pages + maxb;
    PMX_TRY_HIP(hipEventCreateWithFlags(&M.ev_prefetch, hipEventDisableTiming));
    PMX_TRY_HIP(hipEventCreateWithFlags(&M.ev_step, hipEventDisableTiming));
  }
  PMX_TRY_HIP(hipEventCreateWithFlags(&st->ev_h2d_fence, hipEventDisableTiming));

  // weights (internal layouts have the same sizes as the canonical ones)
  st->w.resize(c.n_layers);
  for (auto& L : st->w) {
    char* p;
    PMX_TRY(dev_alloc(st, &p, (size_t)h * D.Nqkv * st->esz)); L.wqkv = p;
    PMX_TRY(dev_alloc(st, &p, (size_t)nq * h * st->esz));     L.wo = p;
    PMX_TRY(dev_alloc(st, &p, (size_t)h * 2 * F * st->esz));  L.wgu = p;
    PMX_TRY(dev_alloc(st, &p, (size_t)F * h * st->esz));      L.wd = p;
    PMX_TRY(dev_alloc(st, &p, (size_t)h * st->esz));          L.g1 = p;
    PMX_TRY(dev_alloc(st, &p, (size_t)h * st->esz));          L.g2 = p;
    PMX_TRY_HIP(hipMemset(L.wqkv, 0, (size_t)h * D.Nqkv * st->esz));
    PMX_TRY_HIP(hipMemset(L.wo, 0, (size_t)nq * h * st->esz));
    PMX_TRY_HIP(hipMemset(L.wgu, 0, (size_t)h * 2 * F * st->esz));
    PMX_TRY_HIP(hipMemset(L.wd, 0, (size_t)F * h * st->esz));
    PMX_TRY_HIP(hipMemset(L.g1, 0, (size_t)h * st->esz));
    PMX_TRY_HIP(hipMemset(L.g2, 0, (size_t)h * st->esz));
  }

  // activations
  const int mpad = ((maxb + 31) / 32) * 32;
  // the GEMM kernels are instantiated for 1, 2, 4 or 8 row tiles of 32 and read all of them
  const int mtile = (maxb <= 32) ? 32 : (maxb <= 64) ? 64 : (maxb <= 128) ? 128 : ((maxb + 255) / 256) * 256;
  PMX_TRY(dev_alloc(st, &st->x, (size_t)mpad * h));
  PMX_TRY(dev_alloc(st, &st->rope_cs, (size_t)maxb * (c.head_dim / 2)));
  if (st->engine == 0) {
    PMX_TRY(dev_alloc(st, &st->g_xn, (size_t)maxb * h));
    PMX_TRY(dev_alloc(st, &st->g_qkv, (size_t)maxb * D.Nqkv));
    PMX_TRY(dev_alloc(st, &st->g_q, (size_t)maxb * nq));
    PMX_TRY(dev_alloc(st, &st->g_attn, (size_t)maxb * nq));
    PMX_TRY(dev_alloc(st, &st->g_gu, (size_t)maxb * 2 * F));
    PMX_TRY(dev_alloc(st, &st->g_act, (size_t)maxb * F));
    PMX_TRY(dev_alloc(st, &st->g_scores, (size_t)maxb * c.n_q_heads * D.max_ctx_pad));
  } else {
    st->f_qkv = plan_gemm_skinny(D.Nqkv, h, false);
    st->f_o = plan_gemm_skinny(h, nq, false);
    st->f_gu = plan_gemm_skinny(2 * F, h, true);
    st->f_d = plan_gemm_skinny(h, F, false);
    // tuning overrides "splits,waves" (waves 4 or 8), e.g. PIPEMAX_PLAN_O=2,8
    auto override_plan = [&](const char* name, GemmPlan& p, int K) {
      const char* e = getenv(name);
      int sp = 0, wv = 0;
      if (!e || sscanf(e, "%d,%d", &sp, &wv) != 2 || (wv != 4 && wv != 8) || sp < 1) return;
      const int KT = K / 16;
      sp = std::max(1, std::min(sp, KT / (wv * 4)));
      const int ksp = (KT + sp - 1) / sp;
      p.split = p.fused_swiglu ? 1 : (KT + ksp - 1) / ksp;
      p.nwk = wv;
    };
    override_plan("PIPEMAX_PLAN_QKV", st->f_qkv, h);
    override_plan("PIPEMAX_PLAN_O", st->f_o, nq);
    override_plan("PIPEMAX_PLAN_GU", st->f_gu, h);
    override_plan("PIPEMAX_PLAN_D", st->f_d, F);
    const int fpad = std::min(mpad, kFusedRows);
    size_t part = 0;
    part = std::max(part, (size_t)st->f_qkv.split * fpad * D.Nqkv);
    part = std::max(part, (size_t)st->f_o.split * fpad * h);
    part = std::max(part, (size_t)st->f_gu.split * fpad * 2 * F);
    part = std::max(part, (size_t)st->f_d.split * fpad * h);
    // the un-fused path plans its split per call from the row count; the partial buffer covers every count
    for (int rows = kFusedRows + 32; rows <= mpad; rows += 32) {
      part = std::max(part, (size_t)plan_rows(D.Nqkv, h, rows).split * rows * D.Nqkv);
      part = std::max(part, (size_t)plan_rows(h, nq, rows).split * rows * h);
      part = std::max(part, (size_t)plan_rows(2 * F, h, rows).split * rows * 2 * F);
      part = std::max(part, (size_t)plan_rows(h, F, rows).split * rows * h);
    }
    PMX_TRY(dev_alloc(st, &st->m_part, part));
    PMX_TRY(dev_alloc(st, &st->m_xn_t, (size_t)mtile * h));
    PMX_TRY(dev_alloc(st, &st->m_q, (size_t)maxb * nq));
    PMX_TRY(dev_alloc(st, &st->m_attn_t, (size_t)mtile * nq));
    PMX_TRY(dev_alloc(st, &st->m_act_t, (size_t)mtile * F));
    PMX_TRY_HIP(hipMemset(st->m_xn_t, 0, (size_t)mtile * h * 2));
    PMX_TRY_HIP(hipMemset(st->m_attn_t, 0, (size_t)mtile * nq * 2));
    PMX_TRY_HIP(hipMemset(st->m_act_t, 0, (size_t)mtile * F * 2));
    st->nch_alloc = (D.max_pages + 7) / 8;
    PMX_TRY(dev_alloc(st, &st->m_part_o, (size_t)maxb * c.n_q_heads * st->nch_alloc * 128));
    PMX_TRY(dev_alloc(st, &st->m_part_ml, (size_t)maxb * c.n_q_heads * st->nch_alloc * 2));
    const size_t n_cnt = (size_t)std::max(D.Nqkv, h) / 64 + 1;
    PMX_TRY(dev_alloc(st, &st->m_cnt_gemm, n_cnt));
    PMX_TRY(dev_alloc(st, &st->m_cnt_attn, (size_t)maxb * c.n_kv_heads));
    PMX_TRY(dev_alloc(st, &st->m_ssq, (size_t)kFusedRows * (h / 64)));
    PMX_TRY_HIP(hipMemset(st->m_cnt_gemm, 0, n_cnt * sizeof(int)));
    PMX_TRY_HIP(hipMemset(st->m_cnt_attn, 0, (size_t)maxb * c.n_kv_heads * sizeof(int)));
    PMX_TRY_HIP(hipMemset(st->m_ssq, 0, (size_t)kFusedRows * (h / 64) * sizeof(float)));
  }
  if (c.flags & PIPEMAX_FLAG_CAPTURE_LAYERS) PMX_TRY(dev_alloc(st, &st->layer_out, (size_t)c.n_layers * maxb * h));

  // write-back staging ring + table ring
  const size_t stage_bytes = (size_t)c.n_layers * maxb * 2 * c.n_kv_heads * c.head_dim * st->esz;
  for (int s = 0; s < kSlots; ++s) {
    char* p;
    PMX_TRY(dev_alloc(st, &p, stage_bytes)); st->d_stage[s] = p;
    PMX_TRY(host_alloc(st, &p, stage_bytes)); st->h_stage[s] = p;
    st->ev_ready[s].resize(c.n_layers, nullptr);
    for (int l = 0; l < c.n_layers; ++l) {
      // the worker sleeps in hipEventSynchronize instead of spinning on a core for a whole step
      PMX_TRY_HIP(hipEventCreateWithFlags(&st->ev_ready[s][l], hipEventDisableTiming | hipEventBlockingSync));
    }
  }
  for (int r = 0; r < kTableRing; ++r) {
    PMX_TRY(host_alloc(st, &st->h_table[r], (size_t)maxb * D.max_pages + 2 * (size_t)maxb));
    PMX_TRY_HIP(hipEventCreateWithFlags(&st->ev_table[r], hipEventDisableTiming));
  }
  PMX_TRY_HIP(hipDeviceSynchronize());
#undef PMX_TRY
#undef PMX_TRY_HIP

  if (const char* e = getenv("PIPEMAX_ATTN_CHUNK_PAGES")) st->attn_cp_override = atoi(e);
  if (const char* e = getenv("PIPEMAX_ATTN_KERNEL")) st->attn_worker = e[0] == 'w' ? 1 : (e[0] == 'g' ? 2 : 0);
  st->dma = dma_copy_create(st->d_stage[0], st->h_stage[0]);
  st->worker = std::thread(worker_main, st);
  st->pf_worker = std::thread(pf_worker_main, st);
  st->worker_started = true;
  st->st.engine = st->engine;
  *out = st;
  return PIPEMAX_OK;
}

int pipemax_stage_destroy(pipemax_stage_t* st) {
  if (!st) PMX_FAIL(PIPEMAX_ERR_ARG, "null stage");
  destroy_impl(st);
  return PIPEMAX_OK;
}

int pipemax_set_weight(pipemax_stage_t* st, int layer, int which, const void* host, size_t bytes) {
  if (!st || !host) PMX_FAIL(PIPEMAX_ERR_ARG, "null argument");
  if (layer < 0 || layer >= st->cfg.n_layers) PMX_FAIL(PIPEMAX_ERR_ARG, "layer %d out of range", layer);
  const Dims& D = st->D;
  const int nq = D.Hq * D.d;
  int K = 0, N = 0;
  void* dst = nullptr;
  LayerW& L = st->w[layer];
  switch (which) {
    case PIPEMAX_W_QKV: K = D.h; N = D.Nqkv; dst = L.wqkv; break;
    case PIPEMAX_W_O: K = nq; N = D.h; dst = L.wo; break;
    case PIPEMAX_W_GU: K = D.h; N = 2 * D.F; dst = L.wgu; break;
    case PIPEMAX_W_D: K = D.F; N = D.h; dst = L.wd; break;
    case PIPEMAX_G_ATTN: K = 1; N = D.h; dst = L.g1; break;
    case PIPEMAX_G_FFN: K = 1; N = D.h; dst = L.g2; break;
    default: PMX_FAIL(PIPEMAX_ERR_ARG, "unknown weight id %d", which);
  }
  const size_t want = (size_t)K * N * st->esz;
  if (bytes != want) PMX_FAIL(PIPEMAX_ERR_ARG, "weight %d needs %zu bytes, got %zu", which, want, bytes);
  PMX_HIP(hipSetDevice(st->dev));
  if (st->engine == 0 || which >= PIPEMAX_G_ATTN) {
    PMX_HIP(hipMemcpy(dst, host, want, hipMemcpyHostToDevice));
    return PIPEMAX_OK;
  }
  // matrix-core engine: re-tile into B-operand fragments.  The gate/up matrix additionally
  // interleaves 32-column tiles (gate tile j, up tile j) so that one work-group column range
  // holds both halves of the same FFN columns.
  std::vector<uint16_t> tiled;
  try {
    tiled.resize((size_t)K * N);
  } catch (...) {
    PMX_FAIL(PIPEMAX_ERR_OOM_HOST, "out of host memory re-tiling a weight");
  }
  const uint16_t* src = (const uint16_t*)host;
  const int KT = K / 16;
  const int F = D.F;
  const int NT = N / 32;
  kmp_set_blocktime(0);      // the helper threads sleep after the loop instead of spinning beside the first steps
#pragma omp parallel for schedule(static)
  for (int nt = 0; nt < NT; ++nt) {
    int src_col0;
    if (which == PIPEMAX_W_GU) {
      src_col0 = (nt & 1) ? (F + (nt >> 1) * 32) : ((nt >> 1) * 32);
    } else if (which == PIPEMAX_W_QKV) {
      // the four 32-column tiles of a head in the order (0, 2, 1, 3): a 64-column block then holds
      // elements j and j + 64 of the head, i.e. both halves of RoPE pairs
      static const int order[4] = {0, 64, 32, 96};
      src_col0 = (nt >> 2) * 128 + order[nt & 3];
    } else {
      src_col0 = nt * 32;
    }
    for (int kt = 0; kt < KT; ++kt) {
      uint16_t* frag = tiled.data() + ((size_t)nt * KT + kt) * 512;
      for (int lane = 0; lane < 64; ++lane) {
        const int n = src_col0 + (lane & 31);
        const int kb = kt * 16 + (lane >> 5) * 8;
        for (int e = 0; e < 8; ++e) frag[lane * 8 + e] = src[(size_t)(kb + e) * N + n];
      }
    }
  }
  PMX_HIP(hipMemcpy(dst, tiled.data(), want, hipMemcpyHostToDevice));
  return PIPEMAX_OK;
}

int pipemax_mb_define(pipemax_stage_t* st, int mb, int n_seqs, const int32_t* ctx_lens) {
  int rc = check_mb(st, mb, false);
  if (rc) return rc;
  MicroBatch& M = st->mbs[mb];
  if (M.defined) PMX_FAIL(PIPEMAX_ERR_ARG, "micro-batch %d is already defined", mb);
  if (!ctx_lens || n_seqs < 1 || n_seqs > st->cfg.max_seqs_per_mb)
    PMX_FAIL(PIPEMAX_ERR_ARG, "n_seqs %d outside [1, %d]", n_seqs, st->cfg.max_seqs_per_mb);
  int64_t need = 0;
  for (int i = 0; i < n_seqs; ++i) {
    if (ctx_lens[i] < 0 || ctx_lens[i] > st->cfg.max_ctx)
      PMX_FAIL(PIPEMAX_ERR_ARG, "context length %d outside [0, %d]", ctx_lens[i], st->cfg.max_ctx);
    const int res_len = std::min(st->cfg.max_ctx, ctx_lens[i] + st->cfg.host_reserve_tokens);
    need += (res_len + kPageTokens - 1) / kPageTokens;
  }
  if (need > st->host_pages->free_count())
    PMX_FAIL(PIPEMAX_ERR_POOL_EXHAUSTED, "host pool has %d free pages, %lld needed", st->host_pages->free_count(),
             (long long)need);
  PMX_HIP(hipSetDevice(st->dev));
  M.seq.assign(n_seqs, SeqState());
  for (int i = 0; i < n_seqs; ++i) {
    SeqState& S = M.seq[i];
    S.len = ctx_lens[i];
    S.state = ST_HOST;
    const int np = (S.len + kPageTokens - 1) / kPageTokens;
    const int res_len = std::min(st->cfg.max_ctx, S.len + st->cfg.host_reserve_tokens);
    const int np_res = (res_len + kPageTokens - 1) / kPageTokens;
    S.host.resize(np_res);
    st->host_pages->alloc(np_res, S.host.data());
    S.host_reserved.assign(S.host.begin() + np, S.host.end());
    S.host.resize(np);
  }
  M.b = n_seqs;
  M.defined = true;
  M.table_dirty = true;
  return PIPEMAX_OK;
}

int pipemax_mb_define_alias(pipemax_stage_t* st, int mb, int src_mb) {
  int rc = check_mb(st, mb, false);
  if (rc) return rc;
  rc = check_mb(st, src_mb, true);
  if (rc) return rc;
  MicroBatch& M = st->mbs[mb];
  const MicroBatch& S = st->mbs[src_mb];
  if (M.defined) PMX_FAIL(PIPEMAX_ERR_ARG, "micro-batch %d is already defined", mb);
  if (S.alias_of >= 0) PMX_FAIL(PIPEMAX_ERR_ARG, "micro-batch %d is itself an alias", src_mb);
  st->wait_mb_writeback(src_mb);
  M.seq.assign(S.b, SeqState());
  for (int i = 0; i < S.b; ++i) {
    M.seq[i].len = S.seq[i].len;
    M.seq[i].state = ST_HOST;
    M.seq[i].host = S.seq[i].host;                     // the same page ids: nothing is taken from the pool
    M.seq[i].host_reserved = S.seq[i].host_reserved;   // growth lands in the source's reserved pages as well
  }
  M.b = S.b;
  M.alias_of = src_mb;
  M.defined = true;
  M.table_dirty = true;
  return PIPEMAX_OK;
}

int pipemax_mb_alias_of(pipemax_stage_t* st, int mb, int32_t* src_mb) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  if (!src_mb) PMX_FAIL(PIPEMAX_ERR_ARG, "null argument");
  *src_mb = st->mbs[mb].alias_of;
  return PIPEMAX_OK;
}

int pipemax_kv_host_write(pipemax_stage_t* st, int mb, int seq, int layer, int tok0, int ntok,
                          const void* K, const void* V) {
  int rc = kv_rw_check(st, mb, seq, layer, tok0, ntok);
  if (rc) return rc;
  if (!K || !V) PMX_FAIL(PIPEMAX_ERR_ARG, "null K/V");
  if (st->mbs[mb].alias_of >= 0)
    PMX_FAIL(PIPEMAX_ERR_STATE, "micro-batch %d is an alias: it has no host pages of its own to write", mb);
  SeqState& S = st->mbs[mb].seq[seq];
  if (S.state != ST_HOST) PMX_FAIL(PIPEMAX_ERR_STATE, "kv_host_write needs a HOST-resident sequence");
  st->wait_mb_writeback(mb);
  const size_t row = (size_t)st->D.Hkv * st->D.d;
#pragma omp parallel for schedule(static) if (ntok >= 256)
  for (int t = 0; t < ntok; ++t) {
    const int tok = tok0 + t;
    char* page = st->host_page_ptr(S.host[tok / kPageTokens]);
    if (st->esz == 4)
      scatter_token<float>(st, (float*)page, layer, tok % kPageTokens, (const float*)K + t * row,
                           (const float*)V + t * row);
    else
      scatter_token<uint16_t>(st, (uint16_t*)page, layer, tok % kPageTokens, (const uint16_t*)K + t * row,
                              (const uint16_t*)V + t * row);
  }
  return PIPEMAX_OK;
}

int pipemax_kv_host_read(pipemax_stage_t* st, int mb, int seq, int layer, int tok0, int ntok, void* K,
                         void* V) {
  int rc = kv_rw_check(st, mb, seq, layer, tok0, ntok);
  if (rc) return rc;
  if (!K || !V) PMX_FAIL(PIPEMAX_ERR_ARG, "null K/V");
  SeqState& S = st->mbs[mb].seq[seq];
  st->wait_mb_writeback(mb);
  const size_t row = (size_t)st->D.Hkv * st->D.d;
  for (int t = 0; t < ntok; ++t) {
    const int tok = tok0 + t;
    const char* page = st->host_page_ptr(S.host[tok / kPageTokens]);
    if (st->esz == 4)
      gather_token<float>(st, (const float*)page, layer, tok % kPageTokens, (float*)K + t * row, (float*)V + t * row);
    else
      gather_token<uint16_t>(st, (const uint16_t*)page, layer, tok % kPageTokens, (uint16_t*)K + t * row,
                             (uint16_t*)V + t * row);
  }
  return PIPEMAX_OK;
}

int pipemax_kv_dev_read(pipemax_stage_t* st, int mb, int seq, int layer, int tok0, int ntok, void* K,
                        void* V) {
  int rc = kv_rw_check(st, mb, seq, layer, tok0, ntok);
  if (rc) return rc;
  if (!K || !V) PMX_FAIL(PIPEMAX_ERR_ARG, "null K/V");
  SeqState& S = st->mbs[mb].seq[seq];
  if (S.state == ST_HOST) PMX_FAIL(PIPEMAX_ERR_NOT_RESIDENT, "sequence %d of micro-batch %d has no GPU pages", seq, mb);
  rc = pipemax_sync(st);
  if (rc) return rc;
  const int Hkv = st->D.Hkv, d = st->D.d;
  const size_t row = (size_t)Hkv * d;
  const size_t layer_bytes = (size_t)Hkv * 2 * kPageTokens * d * st->esz;   // one layer's slice of a page
  std::vector<char> tmp(st->page_bytes);
  int cached = -1;
  for (int t = 0; t < ntok; ++t) {
    const int tok = tok0 + t, pi = tok / kPageTokens;
    if (pi != cached) {
      const size_t off = (size_t)sub_block_off(Hkv, d, layer, 0, 0) * st->esz;
      PMX_HIP(hipMemcpy(tmp.data() + off, st->gpu_block_ptr(S.gpu[pi], layer), layer_bytes, hipMemcpyDeviceToHost));
      cached = pi;
    }
    if (st->esz == 4)
      gather_token<float>(st, (const float*)tmp.data(), layer, tok % kPageTokens, (float*)K + t * row, (float*)V + t * row);
    else
      gather_token<uint16_t>(st, (const uint16_t*)tmp.data(), layer, tok % kPageTokens, (uint16_t*)K + t * row,
                             (uint16_t*)V + t * row);
  }
  return PIPEMAX_OK;
}

// ---- prefetch / evict -----------------------------------------------------------------------------
int pipemax_prefetch_kv(pipemax_stage_t* st, int mb, const int32_t* seq_ids, int n) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  MicroBatch& M = st->mbs[mb];
  std::vector<int> ids;
  rc = seq_list(st, mb, seq_ids, n, ids);
  if (rc) return rc;
  std::vector<int> todo;
  int64_t need = 0;
  for (int i : ids)
    if (M.seq[i].state == ST_HOST) {
      todo.push_back(i);
      need += (int64_t)M.seq[i].host.size();
    }
  if (todo.empty()) return PIPEMAX_OK;
  if (need > st->gpu_pages->free_count())
    PMX_FAIL(PIPEMAX_ERR_POOL_EXHAUSTED, "GPU pool has %d free pages, %lld needed", st->gpu_pages->free_count(),
             (long long)need);
  {
    std::lock_guard<std::mutex> lk(st->mu);
    if (st->pf_error != PIPEMAX_OK) {
      set_error("%s", st->pf_error_text);
      return st->pf_error;
    }
  }
  std::vector<int32_t> src, dst;
  src.reserve(need);
  dst.reserve(need);
  for (int i : todo) {
    SeqState& S = M.seq[i];
    S.gpu.resize(S.host.size());
    st->gpu_pages->alloc((int)S.gpu.size(), S.gpu.data());
    S.state = ST_INFLIGHT;
    src.insert(src.end(), S.host.begin(), S.host.end());
    dst.insert(dst.end(), S.gpu.begin(), S.gpu.end());
  }
  M.table_dirty = true;
  PfJob job;
  job.mb = mb;
  // a layer-major pool takes a run as n_layers strided copies of count x 64 KiB: longer runs keep each copy large
  plan_copy_runs(src.data(), dst.data(), (int)src.size(), st->layer_major() ? 8 * kMaxRunPages : kMaxRunPages, job.runs);
  for (const CopyRun& r : job.runs) {
    st->st.h2d_bytes += (uint64_t)r.count * st->page_bytes;
    st->st.h2d_copies += st->layer_major() ? st->cfg.n_layers : 1;
  }
  // the pages freed by earlier evictions may still be read by the evicted micro-batches' last steps
  job.release.swap(st->release_wait);
  job.stream_ordered = (st->cfg.flags & PIPEMAX_FLAG_STREAM_ORDERED_EVICT) && !st->xfer;
  job.timed = st->timing();
  {
    std::lock_guard<std::mutex> lk(st->mu);
    job.no = ++st->pf_queued;
    job.wb_target = M.wb_queued;     // the host replica of mb must be complete before it is read
    M.pf_ticket = job.no;
    st->pf_jobs.push_back(std::move(job));
  }
  st->cv_pf.notify_one();
  M.prefetch_pending = true;
  return PIPEMAX_OK;
}

int pipemax_evict_kv(pipemax_stage_t* st, int mb, const int32_t* seq_ids, int n) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  MicroBatch& M = st->mbs[mb];
  std::vector<int> ids;
  rc = seq_list(st, mb, seq_ids, n, ids);
  if (rc) return rc;
  bool any = false, any_inflight = false;
  for (int i : ids)
    if (M.seq[i].state != ST_HOST) {
      any = true;
      any_inflight |= (M.seq[i].state == ST_INFLIGHT);
    }
  if (!any) return PIPEMAX_OK;
  PMX_HIP(hipSetDevice(st->dev));
  // later prefetches into these pages must come after the last step that read them (the prefetch worker waits)
  if (M.stepped && std::find(st->release_wait.begin(), st->release_wait.end(), mb) == st->release_wait.end())
    st->release_wait.push_back(mb);
  // pages of a cancelled prefetch may be handed to a decode step's growth: fence the compute stream
  if (any_inflight) st->wait_pf(M.pf_ticket);     // its copies are on the stream (or with the orchestrator)
  if (any_inflight && st->xfer && M.prefetch_ticket) {
    rc = pipemax_xfer_wait(st->xfer, M.prefetch_ticket);     // the copies into these pages have landed
    if (rc) return rc;
  } else if (any_inflight) {
    PMX_HIP(hipEventRecord(st->ev_h2d_fence, st->s_h2d));
    st->h2d_fence_pending = true;
  }
  for (int i : ids) {
    SeqState& S = M.seq[i];
    if (S.state == ST_HOST) continue;
    st->gpu_pages->release(S.gpu.data(), (int)S.gpu.size());
    S.gpu.clear();
    S.state = ST_HOST;
  }
  M.table_dirty = true;
  return PIPEMAX_OK;
}

// ---- the decode step ----------------------------------------------------------------------------------
namespace {
// Chunking of the decode attention for a step of b rows whose longest context is max_len cached tokens and that
// reads sum_pages pages per KV head and layer, on a chip of `cus` compute units: which kernel (*per_wave: a wave per
// (chunk, KV head, sequence) item, else a work-group per item), pages per item (*cp_out) and the number of chunks
// (returned).
int attention_plan(const pipemax_stage* st, int b, int max_len, int64_t sum_pages, int cus, int* cp_out,
                   bool* per_wave) {
  const Dims& D = st->D;
  *per_wave = false;
  // A wave per item when the (sequence, KV head) pairs alone give every compute unit two waves: the waves then
  // share nothing and never wait for each other (256 x 8 pairs of 129 pages: 334 against 348 us per launch; 128 x 8
  // ragged pairs: 213 against 217; 64 x 8 pairs of 65-82 pages, in two chunks each: 51.7 against 53.6).  A wave streams
  // a page in about 1 us at best (2.6 us when 2048 of them share the chip); a context that would take one wave longer
  // than all pages take the chip (6.5 TB/s, 8 KiB per page and head) is split evenly -- and with it every sequence
  // longer than the resulting chunk (128 ragged sequences of 512..4096 tokens: chunks of 129 pages 213 us, of 86
  // pages 221 us; the 64 x 8 pairs in one / two / three chunks: 55.0 / 51.7 / 57-61 us).
  if (st->attn_worker == 1 || (st->attn_worker == 0 && b * D.Hkv >= 2 * cus)) {
    const int npages = (max_len + 1 + kPageTokens - 1) / kPageTokens;
    const double t_all_us = (double)D.Hkv * (double)sum_pages * 8192.0 / 6.5e6;
    int CP = std::min(npages, std::max(16, (int)(t_all_us / 1.0)));
    const int n = (npages + CP - 1) / CP;
    CP = std::max(8, (npages + n - 1) / n);
    if (st->attn_cp_override > 0) CP = std::max(8, st->attn_cp_override);
    *per_wave = true;
    *cp_out = CP;
    return std::min(st->nch_alloc, (npages + CP - 1) / CP);
  }
  // attention split: about one wave per SIMD (1024 on the chip); a work-group of kAttnWaves waves
  // covers up to 64 pages per wave, so most contexts are a single chunk
  const int npages_max = (max_len + 1 + kPageTokens - 1) / kPageTokens;
  const int per_chunk_waves = b * D.Hkv * mfma::kAttnWaves;
  const int nch_target = std::max(1, (1024 + per_chunk_waves / 2) / per_chunk_waves);
  int CP = (npages_max + nch_target - 1) / nch_target;
  // Ragged batches: a work-group streams about 1.3 pages per microsecond whatever else runs (its four waves
  // wait for one page each), the whole chip about 650 (8 KiB pages at 5.3 TB/s).  When the longest sequence
  // alone would take longer than all pages take at the chip's rate, it -- and every sequence longer than the
  // resulting chunk -- is split evenly, so that the tail of the launch is not one work-group.  Uniform
  // batches (longest = mean) and batches with enough sequences to hide a long one keep a single chunk
  // (measured: 64 ragged sequences of 512..4100 tokens -4 % per step; 128 of them no gain from splitting).
  {
    const double chip_bound = (double)D.Hkv * (double)sum_pages / 650.0 * 1.3;      // pages one work-group may own
    const double target = std::max(chip_bound, (double)sum_pages / b);
    const int nch_long = std::max(1, (int)std::ceil(npages_max / std::max(target, 1.0) - 1e-9));
    CP = std::min(CP, (npages_max + nch_long - 1) / nch_long);
  }
  CP = std::max(8, std::min(64 * mfma::kAttnWaves, CP));
  // Even chunks: a context one page longer than a work-group takes (4097 tokens = 257 pages against 256) must not
  // become one full chunk and a one-page chunk -- 2048 work-groups of 256 pages run as four long rounds whose tail
  // idles, while 4096 of 129 pages balance (measured, 256 sequences of 4097 tokens: 880 -> 765 us per launch).
  CP = std::max(8, (npages_max + (npages_max + CP - 1) / CP - 1) / ((npages_max + CP - 1) / CP));
  if (st->attn_cp_override > 0) CP = std::max(8, std::min(64 * mfma::kAttnWaves, st->attn_cp_override));
  *cp_out = CP;
  return std::min(st->nch_alloc, (npages_max + CP - 1) / CP);
}

// Lays the working buffers of a b-row step (matrix-core engine, nch attention chunks) out in the static scratch.
// Sizes follow pipemax_stage_create with this call's row count in place of max_seqs_per_mb.  Returns the bytes
// needed (the caller compares them with kScratchBytes); *clear_bytes = the leading part that must start at zero.
size_t carve_work(const pipemax_stage* st, int b, int nch, Work* W, size_t* clear_bytes) {
  const Dims& D = st->D;
  const int nq = D.Hq * D.d;
  const size_t mpad = (size_t)((b + 31) / 32) * 32;
  const size_t mtile = (b <= 32) ? 32 : (b <= 64) ? 64 : (b <= 128) ? 128 : (size_t)((b + 255) / 256) * 256;
  size_t part = 0;
  if (b <= kFusedRows) {
    part = std::max(part, (size_t)st->f_qkv.split * mtile * D.Nqkv);
    part = std::max(part, (size_t)st->f_o.split * mtile * D.h);
    part = std::max(part, (size_t)st->f_d.split * mtile * D.h);
  } else {
    part = std::max(part, (size_t)plan_rows(D.Nqkv, D.h, b).split * mtile * D.Nqkv);
    part = std::max(part, (size_t)plan_rows(D.h, nq, b).split * mtile * D.h);
    part = std::max(part, (size_t)plan_rows(2 * D.F, D.h, b).split * mtile * 2 * D.F);
    part = std::max(part, (size_t)plan_rows(D.h, D.F, b).split * mtile * D.h);
  }
  const size_t n_cnt = (size_t)std::max(D.Nqkv, D.h) / 64 + 1;
  char* base = (char*)st->scratch_dev;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base + off;
    off += (bytes + 255) & ~(size_t)255;
    return p;
  };
  W->m_cnt_gemm = (int*)take(n_cnt * sizeof(int));
  W->m_cnt_attn = (int*)take((size_t)b * D.Hkv * sizeof(int));
  W->m_ssq = (float*)take((size_t)kFusedRows * (D.h / 64) * sizeof(float));
  W->m_xn_t = (uint16_t*)take(mtile * D.h * 2);
  W->m_attn_t = (uint16_t*)take(mtile * nq * 2);
  W->m_act_t = (uint16_t*)take(mtile * D.F * 2);
  *clear_bytes = off;
  W->x = (float*)take(mpad * D.h * sizeof(float));
  W->rope_cs = (float2*)take((size_t)b * (D.d / 2) * sizeof(float2));
  W->m_q = (uint16_t*)take((size_t)b * nq * 2);
  W->m_part = (float*)take(part * sizeof(float));
  W->m_part_o = (float*)take((size_t)b * D.Hq * nch * 128 * sizeof(float));
  W->m_part_ml = (float*)take((size_t)b * D.Hq * nch * 2 * sizeof(float));
  return off;
}

// One pass of the stage over a list of rows.  Row r is one new token: of sequence sel[r] at position
// pos0[r] (= the number of tokens cached before it).  A decode step has one row per sequence at its current
// length; a prefill chunk has consecutive positions of one sequence.  Rows of the same sequence must be
// consecutive and in ascending position, continuing from the sequence's length.  `subset` says that the
// rows are not simply "every sequence of mb": the device copy of the block table is then rebuilt.
// The kernels see rows only: block-table row r holds the pages of row r's sequence and ctx[r] its position;
// every row's K,V is appended before any row's attention runs and row r attends to positions <= pos0[r],
// which is causal attention within a chunk.
int decode_rows(pipemax_stage_t* st, int mb, const std::vector<int>& sel, const std::vector<int>& pos0, bool subset,
                const void* hidden_in, void* hidden_out, void* hip_stream, bool one_seq_chunk = false,
                bool static_scratch = false) {
  const double t_enter = now_s();
  const double wait_enter = st->st.host_wait_s;
  int rc;
  if (!hidden_in || !hidden_out) PMX_FAIL(PIPEMAX_ERR_ARG, "null hidden pointer");
  MicroBatch& M = st->mbs[mb];
  const Dims& D = st->D;
  const int b = (int)sel.size(), nl = st->cfg.n_layers;
  if (b == 0) return PIPEMAX_OK;
  int grow = 0, grow_host = 0, max_len = 0;
  int64_t sum_pages = 0;      // pages the attention of this step reads per KV head and layer
  for (int i : sel)
    if (M.seq[i].state == ST_HOST)
      PMX_FAIL(PIPEMAX_ERR_NOT_RESIDENT, "sequence %d of micro-batch %d is host-resident; prefetch it first", i, mb);
  for (int r = 0; r < b; ++r) {
    const SeqState& S = M.seq[sel[r]];
    if (pos0[r] + 1 > st->cfg.max_ctx)
      PMX_FAIL(PIPEMAX_ERR_STATE, "sequence %d of micro-batch %d is at max_ctx %d", sel[r], mb, st->cfg.max_ctx);
    if (pos0[r] % kPageTokens == 0) {
      ++grow;
      // reserved host pages of the sequence are used first; rows of one sequence are consecutive
      int before = 0;
      for (int q = r - 1; q >= 0 && sel[q] == sel[r]; --q) before += (pos0[q] % kPageTokens == 0);
      if (before >= (int)S.host_reserved.size()) ++grow_host;
    }
    max_len = std::max(max_len, pos0[r]);
    sum_pages += (pos0[r] + 1 + kPageTokens - 1) / kPageTokens;
  }
  if (grow > st->gpu_pages->free_count() || grow_host > st->host_pages->free_count())
    PMX_FAIL(PIPEMAX_ERR_POOL_EXHAUSTED, "%d new pages needed; free: GPU %d, host %d", grow,
             st->gpu_pages->free_count(), st->host_pages->free_count());
  if (static_scratch) {      // refused before anything changes: engine, the scratch's address, its size
    if (st->engine != 1)
      PMX_FAIL(PIPEMAX_ERR_STATE, "the entry point that allocates nothing serves stages on the matrix-core engine only");
    if (!st->scratch_dev) PMX_FAIL(PIPEMAX_ERR_STATE, "the static scratch has no device address on device %d", st->dev);
    int cp = 0;
    Work probe;
    size_t clear_bytes = 0;
    bool pw = false;
    const size_t need_bytes = carve_work(st, b, attention_plan(st, b, max_len, sum_pages, mfma::compute_units(), &cp, &pw), &probe,
                                         &clear_bytes);
    if (need_bytes > kScratchBytes)
      PMX_FAIL(PIPEMAX_ERR_ARG, "a step of %d rows on this stage needs %zu bytes of working buffers; the static scratch "
               "of the entry point that allocates nothing holds %zu", b, need_bytes, kScratchBytes);
  }
  PMX_HIP(hipSetDevice(st->dev));
  hipStream_t cs = hip_stream ? (hipStream_t)hip_stream : st->s_own;
  st->s_last = cs;
  st->no_timing_now = static_scratch;      // no event is created on behalf of a caller that must not allocate

  // ---- bookkeeping: growth pages, positions of the new token ----------------------------------------
  const bool writeback = !(st->cfg.flags & PIPEMAX_FLAG_NO_WRITEBACK);
  auto where = std::make_shared<std::vector<std::pair<int32_t, int>>>(b);
  for (int r = 0; r < b; ++r) {
    SeqState& S = M.seq[sel[r]];
    if (pos0[r] % kPageTokens == 0) {
      int32_t gp, hp;
      st->gpu_pages->alloc(1, &gp);
      if (!S.host_reserved.empty()) {
        hp = S.host_reserved.front();
        S.host_reserved.erase(S.host_reserved.begin());
      } else {
        st->host_pages->alloc(1, &hp);
      }
      S.gpu.push_back(gp);
      S.host.push_back(hp);
      M.table_dirty = true;
    }
    (*where)[r] = {S.host[pos0[r] / kPageTokens], pos0[r] % kPageTokens};
  }

  // ---- stream dependencies -----------------------------------------------------------------------
  if (M.prefetch_pending) {
    st->wait_pf(M.pf_ticket);      // the event below exists only once the worker has issued the copies
    st->tbegin(TC_STALL, cs);      // how long the stream stands at the wait, when timing is on
    if (st->xfer && M.prefetch_ticket) {
      rc = pipemax_xfer_stream_wait(st->xfer, M.prefetch_ticket, cs);
      if (rc) return rc;
    } else {
      PMX_HIP(hipStreamWaitEvent(cs, M.ev_prefetch, 0));
    }
    st->tend(cs);
    M.prefetch_pending = false;
  }
  if (st->h2d_fence_pending) {
    PMX_HIP(hipStreamWaitEvent(cs, st->ev_h2d_fence, 0));
    st->h2d_fence_pending = false;
  }
  for (int i : sel) M.seq[i].state = ST_GPU;
  if (M.table_dirty || subset) {
    const int r = st->table_pos;
    st->table_pos = (st->table_pos + 1) % kTableRing;
    if (st->table_used[r]) PMX_HIP(hipEventSynchronize(st->ev_table[r]));
    int32_t* ht = st->h_table[r];
    const int maxb = st->cfg.max_seqs_per_mb;
    for (int r2 = 0; r2 < b; ++r2) {
      const SeqState& S = M.seq[sel[r2]];
      int32_t* rowp = ht + (size_t)r2 * D.max_pages;
      std::copy(S.gpu.begin(), S.gpu.end(), rowp);
      std::fill(rowp + S.gpu.size(), rowp + D.max_pages, 0);
    }
    // row order for the attention grid: longest context first (ties by row)
    int32_t* ord = ht + (size_t)maxb * D.max_pages;
    for (int r2 = 0; r2 < b; ++r2) ord[r2] = r2;
    std::stable_sort(ord, ord + b, [&](int a, int c2) { return pos0[a] > pos0[c2]; });
    std::fill(ord + b, ord + maxb, 0);
    // lengths before this step; the last kernel of a step advances the device copy
    int32_t* hl = ord + maxb;
    for (int r2 = 0; r2 < b; ++r2) hl[r2] = pos0[r2];
    {
      const size_t n_words = (size_t)maxb * D.max_pages + maxb + b;
      hipLaunchKernelGGL(k_upload_words, dim3((unsigned)std::min<size_t>(64, (n_words + 255) / 256)), dim3(256), 0, cs,
                         M.d_table, (const int32_t*)ht, n_words);
    }
    PMX_HIP(hipEventRecord(st->ev_table[r], cs));
    st->table_used[r] = true;
    M.table_dirty = subset;   // after a caller-chosen row list the device copy does not describe the whole mb
    st->st.table_uploads += 1;
  }
  const int slot = (int)(st->step_no % kSlots);
  if (writeback) st->wait_slot(slot);
  const size_t row = (size_t)D.Hkv * D.d;
  const size_t layer_elems = (size_t)st->cfg.max_seqs_per_mb * 2 * row;
  const size_t copy_bytes = (size_t)b * 2 * row * st->esz;

  // ---- kernels ---------------------------------------------------------------------------------------
  if (st->engine == 0) {
    st->tbegin(PIPEMAX_K_MISC, cs);
    launch_rope_table(cs, M.d_ctx, st->rope_cs, b, D.d, D.rope_base);
    st->tend(cs);
  }

  // write-back: layers are copied in groups of wb_layers_per_copy (0 = the whole step in one copy)
  const int wb_group = (st->cfg.wb_layers_per_copy > 0) ? std::min(st->cfg.wb_layers_per_copy, nl) : nl;
  auto after_append = [&](int l) -> int {
    if (!writeback) return PIPEMAX_OK;
    if ((l + 1) % wb_group != 0 && l != nl - 1) return PIPEMAX_OK;
    const int l0 = (l / wb_group) * wb_group, nlay = l - l0 + 1;
    PMX_HIP(hipEventRecord(st->ev_ready[slot][l], cs));
    // one layer's rows are contiguous for b sequences; a group spans whole layer slots
    const size_t group_bytes = (size_t)(nlay - 1) * layer_elems * st->esz + copy_bytes;
    char* h_dst = (char*)st->h_stage[slot] + (size_t)l0 * layer_elems * st->esz;
    const char* d_src = (const char*)st->d_stage[slot] + (size_t)l0 * layer_elems * st->esz;
    // The worker thread issues the copy once the event has completed.  Enqueued here, behind a cross-stream
    // wait, the runtime's device-to-host copy (a shader copy with a full-size grid) was measured to hold this
    // thread up and to run beside the next kernels of the compute stream, which take several times longer next
    // to it; issued from the worker it costs a prefill pass of 1024 rows 0.25 ms instead of 0.65 ms.
    WbJob job;
    job.ev = st->ev_ready[slot][l];
    job.copy_dst = h_dst; job.copy_src = d_src; job.copy_bytes = group_bytes;
    job.timed = st->timing();
    job.mb = mb; job.layer = l0; job.n_layers = nlay; job.slot = slot; job.b = b; job.where = where;
    {
      std::lock_guard<std::mutex> lk(st->mu);
      M.wb_pending += 1;
      M.wb_queued += 1;
      st->slot_pending[slot] += 1;
      st->jobs.push_back(job);
    }
    st->cv_job.notify_one();
    st->st.d2h_bytes += group_bytes;
    st->st.d2h_copies += 1;
    return PIPEMAX_OK;
  };

  if (st->engine == 0) {
    auto run = [&](auto tag) -> int {
      using T = decltype(tag);
      using Gk = Generic<T>;
      st->tbegin(PIPEMAX_K_MISC, cs);
      Gk::load_hidden(cs, (const T*)hidden_in, st->x, (int64_t)b * D.h);
      st->tend(cs);
      for (int l = 0; l < nl; ++l) {
        const LayerW& L = st->w[l];
        T* stage_l = (T*)st->d_stage[slot] + (size_t)l * layer_elems;
        st->tbegin(PIPEMAX_K_NORM, cs);
        Gk::rmsnorm(cs, st->x, (const T*)L.g1, st->g_xn, b, D.h, D.eps);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_GEMM_QKV, cs);
        Gk::gemm(cs, st->g_xn, (const T*)L.wqkv, st->g_qkv, b, D.h, D.Nqkv, 0);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_ROPE_APPEND, cs);
        Gk::rope_append(cs, D, l, b, st->g_qkv, st->rope_cs, M.d_ctx, M.d_table, (T*)st->gpu_pool, stage_l, st->g_q);
        st->tend(cs);
        int rc2 = after_append(l);
        if (rc2) return rc2;
        st->tbegin(PIPEMAX_K_ATTN, cs);
        Gk::attention(cs, D, l, b, st->g_q, (const T*)st->gpu_pool, M.d_table, M.d_ctx, st->g_scores, st->g_attn);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_GEMM_O, cs);
        Gk::gemm(cs, st->g_attn, (const T*)L.wo, st->x, b, D.Hq * D.d, D.h, 1);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_NORM, cs);
        Gk::rmsnorm(cs, st->x, (const T*)L.g2, st->g_xn, b, D.h, D.eps);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_GEMM_GU, cs);
        Gk::gemm(cs, st->g_xn, (const T*)L.wgu, st->g_gu, b, D.h, 2 * D.F, 0);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_SWIGLU, cs);
        launch_swiglu_generic(cs, st->g_gu, st->g_act, b, D.F);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_GEMM_D, cs);
        Gk::gemm(cs, st->g_act, (const T*)L.wd, st->x, b, D.F, D.h, 1);
        st->tend(cs);
        if (st->layer_out)
          PMX_HIP(hipMemcpyAsync(st->layer_out + (size_t)l * b * D.h, st->x, (size_t)b * D.h * sizeof(float),
                                 hipMemcpyDeviceToDevice, cs));
      }
      st->tbegin(PIPEMAX_K_MISC, cs);
      Gk::store_hidden(cs, st->x, (T*)hidden_out, (int64_t)b * D.h);
      st->tend(cs);
      return PIPEMAX_OK;
    };
    rc = (st->esz == 4) ? run(float()) : run(uint16_t());
    if (rc) return rc;
  } else {
    const int mpad = ((b + 31) / 32) * 32;
    const int nq = D.Hq * D.d;
    const int npages_max = (max_len + 1 + kPageTokens - 1) / kPageTokens;
    int CP = 0;
    bool per_wave = false;
    const int nch = attention_plan(st, b, max_len, sum_pages, mfma::compute_units(), &CP, &per_wave);
    Work W;     // the buffers the step works in: the stage's own, or carved from the static per-GPU scratch
    if (!static_scratch) {
      W.x = st->x; W.rope_cs = st->rope_cs; W.m_xn_t = st->m_xn_t; W.m_q = st->m_q; W.m_attn_t = st->m_attn_t;
      W.m_act_t = st->m_act_t; W.m_part = st->m_part; W.m_part_o = st->m_part_o; W.m_part_ml = st->m_part_ml;
      W.m_ssq = st->m_ssq; W.m_cnt_gemm = st->m_cnt_gemm; W.m_cnt_attn = st->m_cnt_attn;
    } else {
      size_t clear_bytes = 0;
      carve_work(st, b, nch, &W, &clear_bytes);      // fits: checked before the bookkeeping above
      // everything the stage's own buffers have zeroed at creation (counters, sums of squares, padding rows)
      const size_t n16 = clear_bytes / 16;
      hipLaunchKernelGGL(k_clear16, dim3((unsigned)std::min<size_t>(1024, (n16 + 255) / 256)), dim3(256), 0, cs,
                         (uint4*)st->scratch_dev, n16);
    }
    const int64_t s_qkv = (int64_t)mpad * D.Nqkv, s_h = (int64_t)mpad * D.h, s_gu = (int64_t)mpad * 2 * D.F;
    auto run_gemm = [&](const GemmPlan& p, const uint16_t* Xt, const void* Wt, int K, int N) {
      mfma::gemm(cs, Xt, (const uint16_t*)Wt, W.m_part, b, K, N, p.split, p.wn);
    };
    // a prefill chunk (consecutive positions of one sequence) has its own kernel: 16 rows share every K,V load
    const bool chunk_kernel = one_seq_chunk && b > 1 && npages_max <= 64 * mfma::kAttnWaves;
    auto run_attention = [&](int l) {
      if (chunk_kernel) {
        st->tbegin(PIPEMAX_K_ATTN, cs);
        mfma::attention_prefill(cs, D, l, b, pos0[0], W.m_q, (const uint16_t*)st->gpu_pool, M.d_table, W.m_attn_t);
        st->tend(cs);
      } else {
        // timed through the dispatch's own start / stop events: an event recorded before and after a launch
        // also counts the two gaps around the kernel (about 3.5 us here)
        auto* tp = st->tpair(PIPEMAX_K_ATTN);
        mfma::attention(cs, D, l, b, W.m_q, (const uint16_t*)st->gpu_pool, M.d_table, M.d_ctx, W.m_part_o,
                        W.m_part_ml, CP, nch, W.m_cnt_attn, W.m_attn_t,
                        M.d_table + (size_t)st->cfg.max_seqs_per_mb * D.max_pages, tp ? tp->a : nullptr,
                        tp ? tp->b : nullptr, per_wave);
      }
    };
    if (b <= kFusedRows) {
      // 5 launches per layer: every element-wise consumer runs in the epilogue of the GEMM before it
      const int nb = D.h / 64;       // partial sums of squares per row: one per column block of the residual GEMMs
      st->tbegin(PIPEMAX_K_NORM, cs);
      mfma::first(cs, b, D.h, (const uint16_t*)hidden_in, W.x, (const uint16_t*)st->w[0].g1, W.m_xn_t, W.m_ssq,
                  nb, M.d_ctx, W.rope_cs, D.rope_base);
      st->tend(cs);
      for (int l = 0; l < nl; ++l) {
        const LayerW& L = st->w[l];
        const bool last = (l == nl - 1);
        uint16_t* stage_l = (uint16_t*)st->d_stage[slot] + (size_t)l * layer_elems;
        st->tbegin(PIPEMAX_K_GEMM_QKV, cs);
        mfma::gemm_qkv_rope_append(cs, D, l, b, W.m_xn_t, (const uint16_t*)L.wqkv, W.m_part, W.m_cnt_gemm,
                                   W.m_ssq, nb, W.rope_cs, M.d_ctx, M.d_table, (uint16_t*)st->gpu_pool, stage_l,
                                   W.m_q, st->f_qkv.split, st->f_qkv.nwk);
        st->tend(cs);
        int rc2 = after_append(l);
        if (rc2) return rc2;
        run_attention(l);
        st->tbegin(PIPEMAX_K_GEMM_O, cs);
        mfma::gemm_resid(cs, b, nq, D.h, W.m_attn_t, (const uint16_t*)L.wo, W.m_part, W.m_cnt_gemm, W.x,
                         (const uint16_t*)L.g2, W.m_xn_t, W.m_ssq, nullptr, nullptr, st->f_o.split, st->f_o.nwk);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_GEMM_GU, cs);
        mfma::gemm_swiglu(cs, b, D.h, D.F, D.eps, W.m_xn_t, (const uint16_t*)L.wgu, W.m_ssq, nb, W.m_act_t,
                          b > 64 ? 8 : st->f_gu.nwk);   // four row tiles per wave: 8 waves keep two waves per SIMD
        st->tend(cs);
        st->tbegin(PIPEMAX_K_GEMM_D, cs);
        mfma::gemm_resid(cs, b, D.F, D.h, W.m_act_t, (const uint16_t*)L.wd, W.m_part, W.m_cnt_gemm, W.x,
                         last ? nullptr : (const uint16_t*)st->w[l + 1].g1, W.m_xn_t, last ? nullptr : W.m_ssq,
                         last ? (uint16_t*)hidden_out : nullptr, last ? M.d_ctx : nullptr, st->f_d.split,
                         st->f_d.nwk);
        st->tend(cs);
        if (st->layer_out)
          PMX_HIP(hipMemcpyAsync(st->layer_out + (size_t)l * b * D.h, W.x, (size_t)b * D.h * sizeof(float),
                                 hipMemcpyDeviceToDevice, cs));
      }
    } else {
      const GemmPlan p_qkv = plan_rows(D.Nqkv, D.h, b), p_o = plan_rows(D.h, nq, b),
                     p_gu = plan_rows(2 * D.F, D.h, b), p_d = plan_rows(D.h, D.F, b);
      const float* prev_part = nullptr;     // partials of the previous layer's down projection
      st->tbegin(PIPEMAX_K_MISC, cs);
      launch_rope_table(cs, M.d_ctx, W.rope_cs, b, D.d, D.rope_base);
      st->tend(cs);
      for (int l = 0; l < nl; ++l) {
        const LayerW& L = st->w[l];
        uint16_t* stage_l = (uint16_t*)st->d_stage[slot] + (size_t)l * layer_elems;
        st->tbegin(PIPEMAX_K_NORM, cs);
        mfma::resid_norm(cs, b, D.h, D.eps, l == 0 ? (const uint16_t*)hidden_in : nullptr, prev_part,
                         p_d.split, s_h, W.x, (const uint16_t*)L.g1, W.m_xn_t, nullptr);
        st->tend(cs);
        if (st->layer_out && l > 0)
          PMX_HIP(hipMemcpyAsync(st->layer_out + (size_t)(l - 1) * b * D.h, W.x, (size_t)b * D.h * sizeof(float),
                                 hipMemcpyDeviceToDevice, cs));
        st->tbegin(PIPEMAX_K_GEMM_QKV, cs);
        run_gemm(p_qkv, W.m_xn_t, L.wqkv, D.h, D.Nqkv);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_ROPE_APPEND, cs);
        mfma::rope_append(cs, D, l, b, W.m_part, p_qkv.split, s_qkv, W.rope_cs, M.d_ctx, M.d_table,
                          (uint16_t*)st->gpu_pool, stage_l, W.m_q);
        st->tend(cs);
        int rc2 = after_append(l);
        if (rc2) return rc2;
        run_attention(l);
        st->tbegin(PIPEMAX_K_GEMM_O, cs);
        run_gemm(p_o, W.m_attn_t, L.wo, nq, D.h);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_NORM, cs);
        mfma::resid_norm(cs, b, D.h, D.eps, nullptr, W.m_part, p_o.split, s_h, W.x, (const uint16_t*)L.g2,
                         W.m_xn_t, nullptr);
        st->tend(cs);
        st->tbegin(PIPEMAX_K_GEMM_GU, cs);
        const bool gu_fused = (p_gu.wn == 0 && p_gu.split == 1);     // SwiGLU in the GEMM's epilogue
        mfma::gemm(cs, W.m_xn_t, (const uint16_t*)L.wgu, W.m_part, b, D.h, 2 * D.F, p_gu.split, p_gu.wn,
                   gu_fused ? W.m_act_t : nullptr);
        st->tend(cs);
        if (!gu_fused) {
          st->tbegin(PIPEMAX_K_SWIGLU, cs);
          mfma::swiglu(cs, b, D.F, W.m_part, p_gu.split, s_gu, W.m_act_t);
          st->tend(cs);
        }
        st->tbegin(PIPEMAX_K_GEMM_D, cs);
        run_gemm(p_d, W.m_act_t, L.wd, D.F, D.h);
        st->tend(cs);
        prev_part = W.m_part;
      }
      st->tbegin(PIPEMAX_K_NORM, cs);
      mfma::resid_norm(cs, b, D.h, D.eps, nullptr, prev_part, p_d.split, s_h, W.x, nullptr, nullptr,
                       (uint16_t*)hidden_out);
      st->tend(cs);
      if (st->layer_out)
        PMX_HIP(hipMemcpyAsync(st->layer_out + (size_t)(nl - 1) * b * D.h, W.x, (size_t)b * D.h * sizeof(float),
                               hipMemcpyDeviceToDevice, cs));
      st->tbegin(PIPEMAX_K_MISC, cs);
      launch_advance_ctx(cs, M.d_ctx, b);
      st->tend(cs);
    }
  }
  if (st->engine == 0) {
    st->tbegin(PIPEMAX_K_MISC, cs);
    launch_advance_ctx(cs, M.d_ctx, b);
    st->tend(cs);
  }
  PMX_HIP(hipEventRecord(M.ev_step, cs));
  PMX_HIP(hipGetLastError());
  M.stepped = true;
  for (int i : sel) M.seq[i].len += 1;
  st->last_b = b;
  st->step_no += 1;
  st->st.steps += 1;
  st->st.tokens += (uint64_t)b;
  st->st.host_enqueue_s += (now_s() - t_enter) - (st->st.host_wait_s - wait_enter);     // without the waits above
  return PIPEMAX_OK;
}
}  // namespace

int pipemax_decode_step(pipemax_stage_t* st, int mb, const void* hidden_in, void* hidden_out,
                        void* hip_stream) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  std::vector<int> sel(st->mbs[mb].b), pos(st->mbs[mb].b);
  for (int i = 0; i < (int)sel.size(); ++i) {
    sel[i] = i;
    pos[i] = st->mbs[mb].seq[i].len;
  }
  return decode_rows(st, mb, sel, pos, false, hidden_in, hidden_out, hip_stream);
}

int pipemax_decode_step_noalloc(pipemax_stage_t* st, int mb, const void* hidden_in, void* hidden_out,
                                void* hip_stream) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  std::vector<int> sel(st->mbs[mb].b), pos(st->mbs[mb].b);
  for (int i = 0; i < (int)sel.size(); ++i) {
    sel[i] = i;
    pos[i] = st->mbs[mb].seq[i].len;
  }
  rc = decode_rows(st, mb, sel, pos, false, hidden_in, hidden_out, hip_stream, false, true);
  st->no_timing_now = false;
  return rc;
}

int pipemax_decode_step_seqs(pipemax_stage_t* st, int mb, const int32_t* seq_ids, int n, const void* hidden_in,
                             void* hidden_out, void* hip_stream) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  if (!seq_ids && n != 0) PMX_FAIL(PIPEMAX_ERR_ARG, "null sequence list");
  if (n < 0 || n > st->mbs[mb].b) PMX_FAIL(PIPEMAX_ERR_ARG, "%d rows for a micro-batch of %d", n, st->mbs[mb].b);
  std::vector<int> sel, pos;
  std::vector<char> seen(st->mbs[mb].b, 0);
  for (int k = 0; k < n; ++k) {
    if (seq_ids[k] < 0 || seq_ids[k] >= st->mbs[mb].b) PMX_FAIL(PIPEMAX_ERR_ARG, "sequence %d out of range", seq_ids[k]);
    if (seen[seq_ids[k]]) PMX_FAIL(PIPEMAX_ERR_ARG, "sequence %d listed twice", seq_ids[k]);
    seen[seq_ids[k]] = 1;
    sel.push_back(seq_ids[k]);
    pos.push_back(st->mbs[mb].seq[seq_ids[k]].len);
  }
  return decode_rows(st, mb, sel, pos, true, hidden_in, hidden_out, hip_stream);
}

int pipemax_prefill(pipemax_stage_t* st, int mb, int seq, int n_tokens, const void* hidden_in, void* hidden_out,
                    void* hip_stream) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  MicroBatch& M = st->mbs[mb];
  if (seq < 0 || seq >= M.b) PMX_FAIL(PIPEMAX_ERR_ARG, "sequence %d out of range", seq);
  if (n_tokens < 0) PMX_FAIL(PIPEMAX_ERR_ARG, "negative token count");
  if (n_tokens == 0) return PIPEMAX_OK;
  if (!hidden_in || !hidden_out) PMX_FAIL(PIPEMAX_ERR_ARG, "null hidden pointer");
  const SeqState& S = M.seq[seq];
  if (S.state == ST_HOST)
    PMX_FAIL(PIPEMAX_ERR_NOT_RESIDENT, "sequence %d of micro-batch %d is host-resident; prefetch it first", seq, mb);
  if (S.len + n_tokens > st->cfg.max_ctx)
    PMX_FAIL(PIPEMAX_ERR_STATE, "%d + %d tokens exceed max_ctx %d", S.len, n_tokens, st->cfg.max_ctx);
  // all pages of the call are checked up front, so that a later chunk cannot fail for lack of pages
  const int have = (int)S.host.size(), want = (S.len + n_tokens + kPageTokens - 1) / kPageTokens;
  const int new_pages = want - have, new_host = std::max(0, new_pages - (int)S.host_reserved.size());
  if (new_pages > st->gpu_pages->free_count() || new_host > st->host_pages->free_count())
    PMX_FAIL(PIPEMAX_ERR_POOL_EXHAUSTED, "%d new pages needed; free: GPU %d, host %d", new_pages,
             st->gpu_pages->free_count(), st->host_pages->free_count());
  const int chunk = st->cfg.max_seqs_per_mb;
  const size_t row_bytes = (size_t)st->cfg.hidden * st->esz;
  for (int t0 = 0; t0 < n_tokens; t0 += chunk) {
    const int rows = std::min(chunk, n_tokens - t0);
    std::vector<int> sel(rows, seq), pos(rows);
    for (int r = 0; r < rows; ++r) pos[r] = M.seq[seq].len + r;
    rc = decode_rows(st, mb, sel, pos, true, (const char*)hidden_in + (size_t)t0 * row_bytes,
                     (char*)hidden_out + (size_t)t0 * row_bytes, hip_stream, true);
    if (rc) return rc;
  }
  return PIPEMAX_OK;
}

int pipemax_sync(pipemax_stage_t* st) {
  if (!st) PMX_FAIL(PIPEMAX_ERR_ARG, "null stage");
  PMX_HIP(hipSetDevice(st->dev));
  {
    uint64_t last;
    {
      std::lock_guard<std::mutex> lk(st->mu);
      last = st->pf_queued;
    }
    st->wait_pf(last);
  }
  if (st->xfer) {
    int rcx = pipemax_xfer_drain(st->xfer);
    if (rcx) return rcx;
  }
  PMX_HIP(hipStreamSynchronize(st->s_last));
  if (st->s_last != st->s_own) PMX_HIP(hipStreamSynchronize(st->s_own));
  PMX_HIP(hipStreamSynchronize(st->s_h2d));
  PMX_HIP(hipStreamSynchronize(st->s_d2h));
  st->wait_all_writeback();
  {
    std::lock_guard<std::mutex> lk(st->mu);
    if (st->worker_hip_error)
      PMX_FAIL(PIPEMAX_ERR_HIP, "a write-back copy failed: %s", hipGetErrorString((hipError_t)st->worker_hip_error));
    if (st->pf_error != PIPEMAX_OK) {
      set_error("%s", st->pf_error_text);
      return st->pf_error;
    }
  }
  for (auto& M : st->mbs) {
    if (!M.defined) continue;
    M.prefetch_pending = false;
    for (auto& S : M.seq)
      if (S.state == ST_INFLIGHT) S.state = ST_GPU;
  }
  st->h2d_fence_pending = false;
  return PIPEMAX_OK;
}

// ---- introspection ---------------------------------------------------------------------------------------
int pipemax_stage_attach_xfer(pipemax_stage_t* st, pipemax_xfer_t* x) {
  if (!st) PMX_FAIL(PIPEMAX_ERR_ARG, "null stage");
  if (x && st->layer_major())
    PMX_FAIL(PIPEMAX_ERR_STATE, "a transfer orchestrator moves contiguous pieces; it cannot feed a layer-major GPU pool");
  int rc = pipemax_sync(st);
  if (rc) return rc;
  st->xfer = x;
  return PIPEMAX_OK;
}

int pipemax_get_stats(pipemax_stage_t* st, pipemax_stats_t* out) {
  if (!st || !out) PMX_FAIL(PIPEMAX_ERR_ARG, "null argument");
  if (st->timing()) {
    int rc = pipemax_sync(st);
    if (rc) return rc;
    st->resolve_timers();
  }
  {
    std::lock_guard<std::mutex> lk(st->mu);
    *out = st->st;
  }
  out->engine = st->engine;
  out->gpu_pages_total = st->gpu_pages->total();
  out->gpu_pages_free = st->gpu_pages->free_count();
  out->host_pages_total = st->host_pages->total();
  out->host_pages_free = st->host_pages->free_count();
  out->page_bytes = st->page_bytes;
  return PIPEMAX_OK;
}

int pipemax_reset_stats(pipemax_stage_t* st) {
  if (!st) PMX_FAIL(PIPEMAX_ERR_ARG, "null stage");
  if (st->timing()) {
    int rc = pipemax_sync(st);
    if (rc) return rc;
    st->resolve_timers();
  }
  std::lock_guard<std::mutex> lk(st->mu);
  st->st = pipemax_stats_t{};
  st->st.engine = st->engine;
  return PIPEMAX_OK;
}

int pipemax_set_flags(pipemax_stage_t* st, uint32_t set, uint32_t clear) {
  if (!st) PMX_FAIL(PIPEMAX_ERR_ARG, "null stage");
  const uint32_t allowed = PIPEMAX_FLAG_TIME_KERNELS | PIPEMAX_FLAG_NO_WRITEBACK | PIPEMAX_FLAG_TIME_ATTN_ONLY;
  if ((set | clear) & ~allowed) PMX_FAIL(PIPEMAX_ERR_ARG, "only the timing and no-write-back flags can change");
  int rc = pipemax_sync(st);
  if (rc) return rc;
  if (st->timing()) st->resolve_timers();
  st->cfg.flags = (st->cfg.flags | set) & ~clear;
  return PIPEMAX_OK;
}

int pipemax_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15))
    PMX_FAIL(PIPEMAX_ERR_ARG, "probe copy needs 16-byte aligned pointers and size");
  launch_probe_copy((hipStream_t)hip_stream, dst, src, bytes);
  PMX_HIP(hipGetLastError());
  return PIPEMAX_OK;
}

int pipemax_debug_fill_free_gpu_pages(pipemax_stage_t* st, uint16_t pattern) {
  if (!st) PMX_FAIL(PIPEMAX_ERR_ARG, "null stage");
  int rc = pipemax_sync(st);
  if (rc) return rc;
  const int total = st->gpu_pages->total();
  int run0 = -1;
  for (int p = 0; p <= total; ++p) {
    const bool fr = (p < total) && st->gpu_pages->is_free(p);
    if (fr && run0 < 0) run0 = p;
    if (!fr && run0 >= 0) {
      if (st->layer_major()) {
        for (int l = 0; l < st->cfg.n_layers; ++l)
          PMX_HIP(hipMemsetD16Async((hipDeviceptr_t)st->gpu_block_ptr(run0, l), pattern,
                                    (size_t)(p - run0) * st->layer_block_bytes / 2, st->s_own));
      } else {
        PMX_HIP(hipMemsetD16Async((hipDeviceptr_t)st->gpu_page_ptr(run0), pattern,
                                  (size_t)(p - run0) * st->page_bytes / 2, st->s_own));
      }
      run0 = -1;
    }
  }
  PMX_HIP(hipStreamSynchronize(st->s_own));
  return PIPEMAX_OK;
}

int pipemax_debug_set_delays(pipemax_stage_t* st, int h2d_us, int d2h_us, int worker_us) {
  if (!st || h2d_us < 0 || d2h_us < 0 || worker_us < 0) PMX_FAIL(PIPEMAX_ERR_ARG, "bad argument");
  st->dly_h2d = h2d_us;
  st->dly_d2h = d2h_us;
  st->dly_worker = worker_us;
  return PIPEMAX_OK;
}

int pipemax_get_config(pipemax_stage_t* st, pipemax_config_t* out) {
  if (!st || !out) PMX_FAIL(PIPEMAX_ERR_ARG, "null argument");
  *out = st->cfg;
  return PIPEMAX_OK;
}

int pipemax_mb_size(pipemax_stage_t* st, int mb, int32_t* n_seqs) {
  int rc = check_mb(st, mb, false);
  if (rc) return rc;
  if (!n_seqs) PMX_FAIL(PIPEMAX_ERR_ARG, "null argument");
  *n_seqs = st->mbs[mb].defined ? st->mbs[mb].b : 0;
  return PIPEMAX_OK;
}

int pipemax_get_ctx_lens(pipemax_stage_t* st, int mb, int32_t* out) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  if (!out) PMX_FAIL(PIPEMAX_ERR_ARG, "null output");
  for (int i = 0; i < st->mbs[mb].b; ++i) out[i] = st->mbs[mb].seq[i].len;
  return PIPEMAX_OK;
}

int pipemax_get_residency(pipemax_stage_t* st, int mb, int32_t* out) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  if (!out) PMX_FAIL(PIPEMAX_ERR_ARG, "null output");
  for (int i = 0; i < st->mbs[mb].b; ++i) out[i] = st->mbs[mb].seq[i].state;
  return PIPEMAX_OK;
}

int pipemax_get_block_table(pipemax_stage_t* st, int mb, int seq, int32_t* gpu_pages, int32_t* host_pages,
                            int* n) {
  int rc = check_mb(st, mb, true);
  if (rc) return rc;
  if (!n) PMX_FAIL(PIPEMAX_ERR_ARG, "null count");
  MicroBatch& M = st->mbs[mb];
  if (seq < 0 || seq >= M.b) PMX_FAIL(PIPEMAX_ERR_ARG, "sequence %d out of range", seq);
  const SeqState& S = M.seq[seq];
  const int np = (int)S.host.size();
  if ((gpu_pages || host_pages) && *n < np) PMX_FAIL(PIPEMAX_ERR_ARG, "room for %d pages, %d needed", *n, np);
  for (int p = 0; p < np; ++p) {
    if (host_pages) host_pages[p] = S.host[p];
    if (gpu_pages) gpu_pages[p] = (S.state == ST_HOST) ? -1 : S.gpu[p];
  }
  *n = np;
  return PIPEMAX_OK;
}

int pipemax_get_layer_outputs(pipemax_stage_t* st, float* out, size_t bytes) {
  if (!st || !out) PMX_FAIL(PIPEMAX_ERR_ARG, "null argument");
  if (!st->layer_out) PMX_FAIL(PIPEMAX_ERR_STATE, "stage was created without PIPEMAX_FLAG_CAPTURE_LAYERS");
  const size_t want = (size_t)st->cfg.n_layers * st->last_b * st->cfg.hidden * sizeof(float);
  if (bytes != want) PMX_FAIL(PIPEMAX_ERR_ARG, "layer outputs are %zu bytes, got room for %zu", want, bytes);
  int rc = pipemax_sync(st);
  if (rc) return rc;
  PMX_HIP(hipMemcpy(out, st->layer_out, want, hipMemcpyDeviceToHost));
  return PIPEMAX_OK;
}

// ---- host-side planning helpers ------------------------------------------------------------------------------
int64_t pipemax_page_elem_offset(int n_layers, int n_kv_heads, int head_dim, int layer, int kv, int head,
                                 int tok, int dd) {
  if (n_layers < 1 || n_kv_heads < 1 || head_dim < 32 || head_dim % 32 || layer < 0 || layer >= n_layers ||
      kv < 0 || kv > 1 || head < 0 || head >= n_kv_heads || tok < 0 || tok >= kPageTokens || dd < 0 ||
      dd >= head_dim)
    return -1;
  return sub_block_off(n_kv_heads, head_dim, layer, head, kv) + (kv ? v_sub_idx(tok, dd) : k_sub_idx(tok, dd));
}

int pipemax_plan_gemm_splits(int rows, int n_cols, int k, int32_t* plan_splits, int32_t* launch_splits,
                             int32_t* k_steps_per_split) {
  if (!plan_splits || !launch_splits || !k_steps_per_split || rows < 1 || n_cols < 256 || n_cols % 256 != 0 ||
      k < 16 || k % 16 != 0)
    PMX_FAIL(PIPEMAX_ERR_ARG, "plan_gemm_splits: rows >= 1, columns a multiple of 256, k a multiple of 16");
  const GemmPlan p = plan_gemm_large(n_cols, k, rows);
  int ksp = 0;
  *plan_splits = p.split;
  *launch_splits = pmx::mfma::large_gemm_splits(k / 16, p.split, &ksp);
  *k_steps_per_split = ksp;
  return PIPEMAX_OK;
}

int pipemax_plan_attention_chunks(int n_seqs, int n_kv_heads, int max_ctx_tokens, int64_t sum_pages,
                                  int compute_units, int32_t* chunk_pages, int32_t* n_chunks, int32_t* wave_per_item) {
  if (!chunk_pages || !n_chunks || !wave_per_item || n_seqs < 1 || n_kv_heads < 1 || max_ctx_tokens < 1 ||
      sum_pages < 1 || compute_units < 1)
    PMX_FAIL(PIPEMAX_ERR_ARG, "plan_attention_chunks: positive counts");
  pipemax_stage tmp;
  tmp.D.Hkv = n_kv_heads;
  tmp.nch_alloc = (((max_ctx_tokens + kPageTokens - 1) / kPageTokens) + 7) / 8;
  int cp = 0;
  bool pw = false;
  *n_chunks = attention_plan(&tmp, n_seqs, max_ctx_tokens - 1, sum_pages, compute_units, &cp, &pw);
  *chunk_pages = cp;
  *wave_per_item = pw ? 1 : 0;
  return PIPEMAX_OK;
}

int pipemax_plan_copy_runs(const int32_t* src_pages, const int32_t* dst_pages, int n, int max_run_pages,
                           int32_t* runs) {
  if (n < 0 || max_run_pages < 1 || (n > 0 && (!src_pages || !dst_pages || !runs)))
    PMX_FAIL(PIPEMAX_ERR_ARG, "bad argument");
  std::vector<CopyRun> out;
  plan_copy_runs(src_pages, dst_pages, n, max_run_pages, out);
  for (size_t i = 0; i < out.size(); ++i) {
    runs[3 * i] = out[i].src;
    runs[3 * i + 1] = out[i].dst;
    runs[3 * i + 2] = out[i].count;
  }
  return (int)out.size();
}

int pipemax_pool_create(int n_pages, pipemax_pool_t** out) {
  if (n_pages < 0 || !out) PMX_FAIL(PIPEMAX_ERR_ARG, "bad argument");
  *out = new (std::nothrow) pipemax_pool(n_pages);
  if (!*out) PMX_FAIL(PIPEMAX_ERR_OOM_HOST, "out of host memory");
  return PIPEMAX_OK;
}
int pipemax_pool_destroy(pipemax_pool_t* p) {
  if (!p) PMX_FAIL(PIPEMAX_ERR_ARG, "null pool");
  delete p;
  return PIPEMAX_OK;
}
int pipemax_pool_alloc(pipemax_pool_t* p, int n, int32_t* out_pages) {
  if (!p || n < 0 || (n > 0 && !out_pages)) PMX_FAIL(PIPEMAX_ERR_ARG, "bad argument");
  if (!p->pool.alloc(n, out_pages)) PMX_FAIL(PIPEMAX_ERR_POOL_EXHAUSTED, "%d pages wanted, %d free", n, p->pool.free_count());
  return PIPEMAX_OK;
}
int pipemax_pool_free(pipemax_pool_t* p, const int32_t* pages, int n) {
  if (!p || n < 0 || (n > 0 && !pages)) PMX_FAIL(PIPEMAX_ERR_ARG, "bad argument");
  if (!p->pool.release(pages, n)) PMX_FAIL(PIPEMAX_ERR_ARG, "page out of range, duplicated or already free");
  return PIPEMAX_OK;
}
int pipemax_pool_free_count(pipemax_pool_t* p) {
  if (!p) PMX_FAIL(PIPEMAX_ERR_ARG, "null pool");
  return p->pool.free_count();
}

}  // extern "C"

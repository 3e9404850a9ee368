// Measurement probes behind the C ABI: the rates the roofline arguments lean on, measured with the library's own
// code on the machine at hand.  None of them is on the hot path.
//   pipemax_probe_read   a read-only streaming kernel: what HBM delivers to a plain, perfectly coalesced reader
//   pipemax_probe_link   pinned host <-> device copies in pieces of a given size: the host link's rate for whole page
//                        runs (block-first layout, Sec. 3.4.2) against per-(page, layer) fragments (layer-first
//                        layout, the comparison of Sec. 4.4), each direction alone or both at once
#include <algorithm>
#include <chrono>
#include <cstring>
#include <vector>

#include "common.hpp"

namespace pmx {
void set_error(const char* fmt, ...);
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_nt(const uint4* p) {
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4*)p));
}

// Every lane reads 16 bytes per trip; `segment` consecutive trips of a work-group cover one contiguous piece
// (segment == 0: plain grid-stride order).  The loaded words are folded into one value that is stored only if it
// equals a value no input produces in practice, so that the loads cannot be dropped.
__global__ __launch_bounds__(256) void k_probe_read(const uint4* __restrict__ src, size_t n16, unsigned segment,
                                                    uint4* sink) {
  uint4 acc = make_uint4(0, 0, 0, 0);
  if (segment == 0) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
      const uint4 v = load_nt(src + i);
      acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
  } else {
    // block-contiguous: work-group g owns pieces g, g + gridDim.x, ... of segment * 256 words each
    const size_t piece = (size_t)segment * blockDim.x;
    for (size_t p0 = (size_t)blockIdx.x * piece; p0 < n16; p0 += (size_t)gridDim.x * piece)
      for (unsigned k = 0; k < segment; ++k) {
        const size_t i = p0 + (size_t)k * blockDim.x + threadIdx.x;
        if (i < n16) {
          const uint4 v = load_nt(src + i);
          acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
        }
      }
  }
  if ((acc.x ^ acc.y) == 0x9E3779B9u && (acc.z ^ acc.w) == 0x7F4A7C15u && acc.x == 0x12345u) *sink = acc;
}

// one wave that adds 1 to a counter: the shortest kernel that still depends on its predecessor
__global__ void k_probe_tick(unsigned* p) {
  if (threadIdx.x == 0) *p += 1u;
}

double now_s() {
  return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

}  // namespace
}  // namespace pmx

using namespace pmx;

extern "C" {

int pipemax_probe_read(const void* src, size_t bytes, int segment_trips, void* sink16, void* hip_stream) {
  if (!src || !sink16 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)sink16 & 15) || segment_trips < 0 ||
      segment_trips > 4096)
    PMX_FAIL(PIPEMAX_ERR_ARG, "probe read needs 16-byte aligned pointers and size, 0 <= segment_trips <= 4096");
  const size_t n16 = bytes / 16;
  if (n16 == 0) return PIPEMAX_OK;
  // eight work-groups of four waves per compute unit: non-temporal loads stream fastest from 32 waves per unit
  // (2 GiB: 512 / 1024 / 2048 work-groups read 4.2 / 6.6 / 7.1 TB/s)
  const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 2048);
  hipLaunchKernelGGL(k_probe_read, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, (const uint4*)src, n16,
                     (unsigned)segment_trips, (uint4*)sink16);
  PMX_HIP(hipGetLastError());
  return PIPEMAX_OK;
}

int pipemax_probe_link(int device, size_t total_bytes, size_t piece_bytes, size_t piece_stride, int direction,
                       int repeats, pipemax_link_probe_t* out) {
  if (!out || total_bytes == 0 || piece_bytes == 0 || piece_bytes > total_bytes || piece_stride < piece_bytes ||
      direction < 0 || direction > 2 || repeats < 1 || repeats > 64)
    PMX_FAIL(PIPEMAX_ERR_ARG, "probe link: 0 < piece <= total, stride >= piece, direction 0..2, 1 <= repeats <= 64");
  const size_t n_pieces = total_bytes / piece_bytes;
  if (n_pieces > ((size_t)1 << 22)) PMX_FAIL(PIPEMAX_ERR_ARG, "probe link: more than 4M pieces");
  const size_t span = (n_pieces - 1) * piece_stride + piece_bytes;      // both sides use the same arrangement
  if (span > ((size_t)24 << 30)) PMX_FAIL(PIPEMAX_ERR_ARG, "probe link: a span of more than 24 GiB per buffer");
  memset(out, 0, sizeof(*out));
  PMX_HIP(hipSetDevice(device));
  const bool h2d = direction != 1, d2h = direction != 0;
  void *h_src = nullptr, *d_dst = nullptr, *d_src = nullptr, *h_dst = nullptr;
  hipStream_t s_up = nullptr, s_down = nullptr;
  hipEvent_t e[4] = {};
  int rc = PIPEMAX_OK;
  auto fail = [&](int code, const char* what, hipError_t err) {
    if (rc == PIPEMAX_OK) {
      rc = code;
      set_error("probe link: %s failed: %s", what, hipGetErrorString(err));
      (void)hipGetLastError();
    }
  };
  hipError_t err;
  if (h2d) {
    if ((err = hipHostMalloc(&h_src, span, hipHostMallocDefault)) != hipSuccess) fail(PIPEMAX_ERR_OOM_HOST, "hipHostMalloc", err);
    if (rc == PIPEMAX_OK && (err = hipMalloc(&d_dst, span)) != hipSuccess) fail(PIPEMAX_ERR_OOM_DEVICE, "hipMalloc", err);
    if (rc == PIPEMAX_OK) memset(h_src, 0x5a, span);
  }
  if (d2h && rc == PIPEMAX_OK) {
    if ((err = hipHostMalloc(&h_dst, span, hipHostMallocDefault)) != hipSuccess) fail(PIPEMAX_ERR_OOM_HOST, "hipHostMalloc", err);
    if (rc == PIPEMAX_OK && (err = hipMalloc(&d_src, span)) != hipSuccess) fail(PIPEMAX_ERR_OOM_DEVICE, "hipMalloc", err);
    if (rc == PIPEMAX_OK) {
      memset(h_dst, 0, span);
      if ((err = hipMemset(d_src, 0x3c, span)) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipMemset", err);
    }
  }
  if (rc == PIPEMAX_OK && (err = hipStreamCreateWithFlags(&s_up, hipStreamNonBlocking)) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipStreamCreate", err);
  if (rc == PIPEMAX_OK && (err = hipStreamCreateWithFlags(&s_down, hipStreamNonBlocking)) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipStreamCreate", err);
  for (int i = 0; i < 4 && rc == PIPEMAX_OK; ++i)
    if ((err = hipEventCreate(&e[i])) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipEventCreate", err);
  double best_wall = 0.0;
  for (int rep = 0; rep <= repeats && rc == PIPEMAX_OK; ++rep) {      // pass 0 warms the path up and is not counted
    if ((err = hipDeviceSynchronize()) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipDeviceSynchronize", err);
    const double t0 = now_s();
    if (h2d) (void)hipEventRecord(e[0], s_up);
    if (d2h) (void)hipEventRecord(e[2], s_down);
    for (size_t p = 0; p < n_pieces && rc == PIPEMAX_OK; ++p) {
      const size_t off = p * piece_stride;
      if (h2d && (err = hipMemcpyAsync((char*)d_dst + off, (char*)h_src + off, piece_bytes, hipMemcpyHostToDevice, s_up)) != hipSuccess)
        fail(PIPEMAX_ERR_HIP, "hipMemcpyAsync", err);
      if (d2h && (err = hipMemcpyAsync((char*)h_dst + off, (char*)d_src + off, piece_bytes, hipMemcpyDeviceToHost, s_down)) != hipSuccess)
        fail(PIPEMAX_ERR_HIP, "hipMemcpyAsync", err);
    }
    if (h2d) (void)hipEventRecord(e[1], s_up);
    if (d2h) (void)hipEventRecord(e[3], s_down);
    if (rc == PIPEMAX_OK && (err = hipDeviceSynchronize()) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipDeviceSynchronize", err);
    const double wall = now_s() - t0;
    if (rep == 0 || rc != PIPEMAX_OK) continue;
    float up_ms = 0.f, down_ms = 0.f;
    if (h2d) (void)hipEventElapsedTime(&up_ms, e[0], e[1]);
    if (d2h) (void)hipEventElapsedTime(&down_ms, e[2], e[3]);
    if (best_wall == 0.0 || wall < best_wall) {       // the fastest pass: the link's rate, not the host's hiccups
      best_wall = wall;
      out->wall_s = wall;
      out->h2d_s = up_ms * 1e-3;
      out->d2h_s = down_ms * 1e-3;
    }
  }
  out->pieces = n_pieces;
  out->h2d_bytes = h2d ? n_pieces * piece_bytes : 0;
  out->d2h_bytes = d2h ? n_pieces * piece_bytes : 0;
  if (rc == PIPEMAX_OK && d2h && ((unsigned char*)h_dst)[0] != 0x3c) {
    rc = PIPEMAX_ERR_HIP;
    set_error("probe link: the device-to-host copy did not deliver its bytes");
  }
  for (auto ev : e)
    if (ev) (void)hipEventDestroy(ev);
  if (s_up) (void)hipStreamDestroy(s_up);
  if (s_down) (void)hipStreamDestroy(s_down);
  if (h_src) (void)hipHostFree(h_src);
  if (h_dst) (void)hipHostFree(h_dst);
  if (d_dst) (void)hipFree(d_dst);
  if (d_src) (void)hipFree(d_src);
  return rc;
}

int pipemax_probe_link_strided(int device, size_t row_bytes, size_t host_pitch, int rows_per_copy, int n_copies,
                          int repeats, pipemax_link_probe_t* out) {
  if (!out || row_bytes == 0 || host_pitch < row_bytes || rows_per_copy < 1 || n_copies < 1 || repeats < 1 ||
      repeats > 64 || n_copies > (1 << 20))
    PMX_FAIL(PIPEMAX_ERR_ARG, "probe link 2d: pitch >= row > 0, rows >= 1, 1 <= copies <= 1M, 1 <= repeats <= 64");
  const size_t rows = (size_t)rows_per_copy * n_copies;
  const size_t h_span = rows * host_pitch, d_span = rows * row_bytes;
  if (h_span > ((size_t)24 << 30)) PMX_FAIL(PIPEMAX_ERR_ARG, "probe link 2d: more than 24 GiB of host span");
  memset(out, 0, sizeof(*out));
  PMX_HIP(hipSetDevice(device));
  void *h = nullptr, *d = nullptr;
  hipStream_t s = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = PIPEMAX_OK;
  hipError_t err;
  auto fail = [&](int code, const char* what, hipError_t er) {
    if (rc == PIPEMAX_OK) {
      rc = code;
      set_error("probe link 2d: %s failed: %s", what, hipGetErrorString(er));
      (void)hipGetLastError();
    }
  };
  if ((err = hipHostMalloc(&h, h_span, hipHostMallocDefault)) != hipSuccess) fail(PIPEMAX_ERR_OOM_HOST, "hipHostMalloc", err);
  if (rc == PIPEMAX_OK && (err = hipMalloc(&d, d_span)) != hipSuccess) fail(PIPEMAX_ERR_OOM_DEVICE, "hipMalloc", err);
  if (rc == PIPEMAX_OK) memset(h, 0x5a, h_span);
  if (rc == PIPEMAX_OK && (err = hipStreamCreateWithFlags(&s, hipStreamNonBlocking)) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipStreamCreate", err);
  if (rc == PIPEMAX_OK && (err = hipEventCreate(&e0)) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipEventCreate", err);
  if (rc == PIPEMAX_OK && (err = hipEventCreate(&e1)) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipEventCreate", err);
  double best = 0.0;
  for (int rep = 0; rep <= repeats && rc == PIPEMAX_OK; ++rep) {
    if ((err = hipDeviceSynchronize()) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipDeviceSynchronize", err);
    const double t0 = now_s();
    (void)hipEventRecord(e0, s);
    for (int c = 0; c < n_copies && rc == PIPEMAX_OK; ++c)
      if ((err = hipMemcpy2DAsync((char*)d + (size_t)c * rows_per_copy * row_bytes, row_bytes,
                                  (char*)h + (size_t)c * rows_per_copy * host_pitch, host_pitch, row_bytes,
                                  (size_t)rows_per_copy, hipMemcpyHostToDevice, s)) != hipSuccess)
        fail(PIPEMAX_ERR_HIP, "hipMemcpy2DAsync", err);
    (void)hipEventRecord(e1, s);
    if (rc == PIPEMAX_OK && (err = hipDeviceSynchronize()) != hipSuccess) fail(PIPEMAX_ERR_HIP, "hipDeviceSynchronize", err);
    const double wall = now_s() - t0;
    if (rep == 0 || rc != PIPEMAX_OK) continue;
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    if (best == 0.0 || wall < best) {
      best = wall;
      out->wall_s = wall;
      out->h2d_s = ms * 1e-3;
    }
  }
  out->pieces = (uint64_t)n_copies;
  out->h2d_bytes = d_span;
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (s) (void)hipStreamDestroy(s);
  if (h) (void)hipHostFree(h);
  if (d) (void)hipFree(d);
  return rc;
}

int pipemax_probe_launch(int device, int n_kernels, int use_graph, int repeats, pipemax_launch_probe_t* out) {
  if (!out || n_kernels < 1 || n_kernels > 4096 || repeats < 1 || repeats > 1000)
    PMX_FAIL(PIPEMAX_ERR_ARG, "probe launch: 1 <= kernels <= 4096, 1 <= repeats <= 1000");
  memset(out, 0, sizeof(*out));
  PMX_HIP(hipSetDevice(device));
  unsigned* d = nullptr;
  hipStream_t s = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  int rc = PIPEMAX_OK;
  auto fail = [&](const char* what, hipError_t er) {
    if (rc == PIPEMAX_OK && er != hipSuccess) {
      rc = PIPEMAX_ERR_HIP;
      set_error("probe launch: %s failed: %s", what, hipGetErrorString(er));
      (void)hipGetLastError();
    }
  };
  fail("hipMalloc", hipMalloc((void**)&d, 256));
  if (rc == PIPEMAX_OK) fail("hipMemset", hipMemset(d, 0, 256));
  if (rc == PIPEMAX_OK) fail("hipStreamCreate", hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
  if (rc == PIPEMAX_OK) fail("hipEventCreate", hipEventCreate(&e0));
  if (rc == PIPEMAX_OK) fail("hipEventCreate", hipEventCreate(&e1));
  auto enqueue = [&]() {
    for (int k = 0; k < n_kernels; ++k) hipLaunchKernelGGL(k_probe_tick, dim3(1), dim3(64), 0, s, d);
  };
  if (rc == PIPEMAX_OK && use_graph) {
    fail("hipStreamBeginCapture", hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
    if (rc == PIPEMAX_OK) {
      enqueue();
      fail("hipStreamEndCapture", hipStreamEndCapture(s, &graph));
    }
    if (rc == PIPEMAX_OK) fail("hipGraphInstantiate", hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
  }
  double host_best = 0.0, gpu_best = 0.0;
  unsigned launched = 0;
  for (int rep = 0; rep <= repeats && rc == PIPEMAX_OK; ++rep) {      // pass 0 is a warm-up
    fail("hipStreamSynchronize", hipStreamSynchronize(s));
    (void)hipEventRecord(e0, s);
    const double t0 = now_s();
    if (use_graph) fail("hipGraphLaunch", hipGraphLaunch(exec, s));
    else enqueue();
    const double host = now_s() - t0;
    (void)hipEventRecord(e1, s);
    fail("hipStreamSynchronize", hipStreamSynchronize(s));
    launched += (unsigned)n_kernels;
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    if (rep == 0) continue;
    if (host_best == 0.0 || host < host_best) host_best = host;
    if (gpu_best == 0.0 || ms * 1e-3 < gpu_best) gpu_best = ms * 1e-3;
  }
  if (rc == PIPEMAX_OK) {
    unsigned got = 0;
    fail("hipMemcpy", hipMemcpy(&got, d, sizeof(got), hipMemcpyDeviceToHost));
    if (rc == PIPEMAX_OK && got != launched) {
      rc = PIPEMAX_ERR_HIP;
      set_error("probe launch: %u kernels ran, %u were launched", got, launched);
    }
  }
  out->host_enqueue_s = host_best;
  out->gpu_s = gpu_best;
  out->kernels = (uint64_t)n_kernels;
  if (exec) (void)hipGraphExecDestroy(exec);
  if (graph) (void)hipGraphDestroy(graph);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (s) (void)hipStreamDestroy(s);
  if (d) (void)hipFree(d);
  return rc;
}

}  // extern "C"

// Shared declarations of the stage-decode library: status plumbing, the in-page KV layout and
// the tiled activation / weight layouts used by the matrix-core kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "pipemax.h"

namespace pmx {

// ---- error plumbing ------------------------------------------------------------------------
void set_error(const char* fmt, ...);

#define PMX_FAIL(code, ...)            \
  do {                                 \
    ::pmx::set_error(__VA_ARGS__);     \
    return (code);                     \
  } while (0)

#define PMX_HIP(expr)                                                                   \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess)                                                               \
      PMX_FAIL(PIPEMAX_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_),  \
               __FILE__, __LINE__);                                                     \
  } while (0)

constexpr int kPageTokens = 16;

// ---- in-page KV layout ------------------------------------------------------------------------
// A page holds 16 tokens of every layer of the stage (block-first layout, PipeMax Sec. 3.4.2):
//   page = [layer][kv head][K | V][16 x d elements]
// Inside a 16 x d sub-block the element order is the operand order of the gfx950 matrix
// instructions the attention kernel uses, so that every 16-byte lane load is lane-linear:
//   K (A operand of mfma 16x16x32, rows = tokens, k = 8 consecutive d):
//       idx = ((dd / 8) * 16 + tok) * 8 + dd % 8
//   V (A operand of mfma 16x16x16, rows = d, k = 4 consecutive tokens; two 16-wide d tiles
//      share one 16-byte lane load):
//       idx = ((((dd / 32) * 4 + tok / 4) * 16 + dd % 16) * 2 + (dd / 16) % 2) * 4 + tok % 4
// Requires d % 32 == 0.
__host__ __device__ inline int k_sub_idx(int tok, int dd) {
  return ((dd >> 3) * 16 + tok) * 8 + (dd & 7);
}
__host__ __device__ inline int v_sub_idx(int tok, int dd) {
  return (((((dd >> 5) * 4 + (tok >> 2)) * 16 + (dd & 15)) * 2 + ((dd >> 4) & 1)) * 4) + (tok & 3);
}
// element offset of the (layer, head, kv) sub-block inside a page
__host__ __device__ inline int64_t sub_block_off(int n_kv_heads, int d, int layer, int head, int kv) {
  return (((int64_t)layer * n_kv_heads + head) * 2 + kv) * (int64_t)(kPageTokens * d);
}
__host__ __device__ inline int64_t page_elems(int n_layers, int n_kv_heads, int d) {
  return (int64_t)n_layers * n_kv_heads * 2 * kPageTokens * d;
}

// ---- tiled operand layouts of the matrix-core GEMMs ----------------------------------------------
// Activations X[m][k] (m < Mpad = 32 * MT, k < K = 16 * KT) are stored as fragments of
// mfma_f32_32x32x16_bf16's A operand: fragment (mt, kt) is 64 lanes x 8 bf16 = 1 KiB with
//   lane = m % 32 + 32 * ((k % 16) / 8),  element = k % 8
__host__ __device__ inline int64_t a_tiled_idx(int KT, int m, int k) {
  int mt = m >> 5, kt = k >> 4;
  int lane = (m & 31) + 32 * ((k & 15) >> 3);
  return (((int64_t)mt * KT + kt) * 64 + lane) * 8 + (k & 7);
}
// Weights W[k][n] likewise as B-operand fragments: fragment (nt, kt), lane = n % 32 + 32*((k%16)/8).
__host__ __device__ inline int64_t b_tiled_idx(int KT, int k, int n) {
  int nt = n >> 5, kt = k >> 4;
  int lane = (n & 31) + 32 * ((k & 15) >> 3);
  return (((int64_t)nt * KT + kt) * 64 + lane) * 8 + (k & 7);
}

// ---- bf16 on the host ---------------------------------------------------------------------------
inline float bf16_to_f32_host(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  __builtin_memcpy(&f, &u, 4);
  return f;
}

}  // namespace pmx

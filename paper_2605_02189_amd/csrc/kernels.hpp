// Launchers of the device kernels.  Every launcher checks nothing: the stage object validates
// shapes once at create time and passes only buffers it sized itself.
#pragma once

#include "common.hpp"

namespace pmx {

struct Dims {
  int n_layers, h, Hq, Hkv, d, F, Nqkv, G;
  float rope_base, eps;
  int max_pages;        // block-table row length
  int max_ctx_pad;      // row length of the generic attention's score scratch
  int64_t page_elems;   // elements per page (all layers): the unit of the host replica and of a prefetch
  // Device pool addressing: sub-block (page, layer, head, kv) starts at element
  //   page * page_stride + layer * layer_stride + sub_block_off(Hkv, d, 0, head, kv).
  // Block-first pool (the host replica's layout): page_stride = page_elems, layer_stride = one layer's block of a
  // page.  Layer-major pool [layer][page]: page_stride = one layer's block, layer_stride = pages * that block, so
  // that an attention launch (one layer) reads one contiguous tenth of the pool instead of 64 KiB out of every page.
  int64_t page_stride, layer_stride;
};

// ---- shared small kernels ----------------------------------------------------------------------
// cs[i][j] = (cos, sin)(ctx[i] * base^(-2j/d)), angle formed in double precision.
void launch_rope_table(hipStream_t s, const int* ctx, float2* cs, int b, int d, float base);
void launch_advance_ctx(hipStream_t s, int* ctx, int b);
// plain grid-stride 16-byte copy, a counter-calibration aid
void launch_probe_copy(hipStream_t s, void* dst, const void* src, size_t bytes);

// ---- shape-generic engine (T = float or bf16 bit patterns as uint16_t) ---------------------------
template <typename T>
struct Generic {
  static void load_hidden(hipStream_t s, const T* in, float* x, int64_t n);
  static void store_hidden(hipStream_t s, const float* x, T* out, int64_t n);
  static void rmsnorm(hipStream_t s, const float* x, const T* gain, float* xn, int b, int h, float eps);
  // C[M][N] (+)= A[M][K] @ W[K][N]
  static void gemm(hipStream_t s, const float* A, const T* W, float* C, int M, int K, int N,
                   int accumulate);
  static void rope_append(hipStream_t s, const Dims& D, int layer, int b, const float* qkv,
                          const float2* cs, const int* ctx, const int* table, T* pool, T* staging,
                          float* q_out);
  static void attention(hipStream_t s, const Dims& D, int layer, int b, const float* q, const T* pool,
                        const int* table, const int* ctx, float* scores, float* out);
};
void launch_swiglu_generic(hipStream_t s, const float* gu, float* act, int b, int F);

// ---- matrix-core engine (bf16, head_dim 128) -------------------------------------------------------
namespace mfma {

// x (+)= sum_s part[s] ;  optional bf16 input row (hin) replaces x first ;
// optional RMSNorm -> A-tiled bf16 (xn_t, KT = h/16) ; optional bf16 row-major output (hout).
void resid_norm(hipStream_t s, int b, int h, float eps, const uint16_t* hin, const float* part,
                int n_split, int64_t split_stride, float* x, const uint16_t* gain, uint16_t* xn_t,
                uint16_t* hout);

// part[s][m][n] = X[m][k-range s] @ W[k-range s][n]   (X A-tiled, W B-tiled, fp32 partials)
// Mpad = 32*MT rows are computed, rows < M are stored.  N % (32*wn) == 0, wn in {4, 8}; wn == 0 selects the
// large-tile kernel for 65..256 rows (needs N % 256 == 0).
// swiglu_act_t (large-tile kernel, W = interleaved gate/up matrix, one split only): instead of the partials the
// kernel writes silu(gate) * up as the A-tiled bf16 operand of the next GEMM (K = N / 2); ignored otherwise.
void gemm(hipStream_t s, const uint16_t* Xt, const uint16_t* Wt, float* part, int M, int K, int N,
          int n_split, int wn, uint16_t* swiglu_act_t = nullptr);

// K ranges of the large-tile kernel for a requested number of splits: k-steps per split (*ksp) and the number
// of splits the grid really has (the return value; the consumers of the partials must use the same number).
// Ranges of an even number of k-steps -- what the ring kernel needs -- are taken when that keeps the count.
inline int large_gemm_splits(int KT, int n_split, int* ksp_out) {
  int ksp = (KT + n_split - 1) / n_split;
  const int S = (KT + ksp - 1) / ksp;
  if (KT % 2 == 0 && (ksp & 1) && (KT + ksp) / (ksp + 1) == S) ksp += 1;
  *ksp_out = ksp;
  return S;
}

void rope_append(hipStream_t s, const Dims& D, int layer, int b, const float* part, int n_split,
                 int64_t split_stride, const float2* cs, const int* ctx, const int* table,
                 uint16_t* pool, uint16_t* staging, uint16_t* q_out);

constexpr int kAttnWaves = 4;   // waves per attention work-group
int compute_units();            // of the current device (cached per device)
// Causal attention of a prefill chunk: `rows` consecutive new tokens of one sequence starting at position
// pos0, K,V already appended; table = the sequence's page ids.  (pos0 + rows) tokens must fit 64 * kAttnWaves
// pages.  Output rows are written A-tiled like the decode kernel's.
void attention_prefill(hipStream_t s, const Dims& D, int layer, int rows, int pos0, const uint16_t* q,
                       const uint16_t* pool, const int* table, uint16_t* out_t);
// Split-K paged GQA decode attention over the items (chunk, KV head, sequence): chunk_pages = pages per item,
// max_chunks = chunks of the longest context (>= ceil(max pages / chunk_pages)).  per_wave = false: a work-group of
// kAttnWaves waves per item (chunk_pages <= 64 * kAttnWaves), whose waves share the item's pages and merge through LDS;
// true: a wave per item (any chunk_pages).  Whoever finishes a (sequence, kv head) last merges the chunk partials
// (counters: b * Hkv ints, zero, self-resetting) and writes the A-tiled bf16 input of the output projection.
// order[z] = sequence handled by slice z of the items (a permutation of 0..b-1, longest context first).  ev_start /
// ev_stop (both or neither): events that receive the start and stop time of this dispatch (for timing the kernel alone).
void attention(hipStream_t s, const Dims& D, int layer, int b, const uint16_t* q,
               const uint16_t* pool, const int* table, const int* ctx, float* part_o, float* part_ml,
               int chunk_pages, int max_chunks, int* counters, uint16_t* out_t, const int* order,
               hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr, bool per_wave = false);

// ---- fused pipeline for b <= 64 rows -----------------------------------------------------------------
// x = hidden_in; ssq_out[i][0] = sum of squares of row i (other nb-1 entries 0); xg_t = x * gain as
// A-tiled bf16; cs = RoPE table of this step.
void first(hipStream_t s, int b, int h, const uint16_t* hin, float* x, const uint16_t* gain, uint16_t* xg_t,
           float* ssq_out, int nb, const int* ctx, float2* cs, float rope_base);
// QKV projection of the un-normalised xg_t with the RMSNorm row factor, RoPE, q rows, paged K/V append
// and write-back staging in the epilogue.  counters: Nqkv / 64 ints, zero, self-resetting.
void gemm_qkv_rope_append(hipStream_t s, const Dims& D, int layer, int b, const uint16_t* xg_t, const uint16_t* Wt,
                          float* part, int* counters, const float* ssq_in, int n_ssq_in, const float2* cs,
                          const int* ctx, const int* table, uint16_t* pool, uint16_t* staging, uint16_t* q_out,
                          int n_split, int nwk);
// x += X @ W; then either (hout == null) xg_t = x * gain_next (A-tiled bf16) and ssq_out[m][N/64] partial
// sums of squares, or hout = bf16(x) row-major.  ctx_advance != null: ctx_advance[i] += 1 for i < b.
void gemm_resid(hipStream_t s, int b, int K, int N, const uint16_t* Xt, const uint16_t* Wt, float* part,
                int* counters, float* x, const uint16_t* gain_next, uint16_t* xg_t, float* ssq_out,
                uint16_t* hout, int* ctx_advance, int n_split, int nwk);
// act_t = silu(r g) * (r u) with the RMSNorm row factor r from ssq_in; W = interleaved gate/up.
void gemm_swiglu(hipStream_t s, int b, int K, int F, float eps, const uint16_t* xg_t, const uint16_t* Wt,
                 const float* ssq_in, int n_ssq_in, uint16_t* act_t, int nwk);

// act_t (A-tiled, KT = F/16) = silu(sum_s gate) * sum_s up ; partial columns are in the
// gate/up-interleaved order of the tiled W_gu (32 gate columns, then the 32 up columns).
void swiglu(hipStream_t s, int b, int F, const float* part, int n_split, int64_t split_stride,
            uint16_t* act_t);

}  // namespace mfma
}  // namespace pmx

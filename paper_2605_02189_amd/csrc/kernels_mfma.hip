// Matrix-core (MFMA) kernels of the stage decode step for gfx950: bf16 storage, fp32 accumulation,
// head_dim 128, 64-wide wavefronts.
//
// Data reaches the matrix instructions without any shuffle: KV pages, weights and activations are
// stored in operand-fragment order (see common.hpp), so every global load is a lane-linear 16-byte
// load (1 KiB contiguous per wave instruction) that lands directly in an MFMA operand register.
#include <algorithm>
#include <atomic>
#include <cstdlib>

#include <hip/hip_ext.h>

#include "kernels.hpp"

namespace pmx {
namespace mfma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

// streaming 16-byte load: data read exactly once should not displace what is re-used
__device__ inline uint4 ld_stream(const uint4* p) {
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4*)p));
}

// Split-K partials cross work-groups (and XCDs, whose L2 caches are not coherent with each other)
// inside one kernel.  They are written and read with agent-scope relaxed atomics, which the hardware
// executes as write-through stores / coherent loads, so publishing them needs only "wait until my
// stores are acknowledged" before the arrival counter is bumped, not a write-back or invalidation
// of the whole L2 (which is what a device-wide fence costs: ~45 us per kernel when measured here).
// The language memory model asks for more than this relies on (a release at agent scope on the arrival and an
// acquire at agent scope in the last arriver; measured: +3 us on every split GEMM launch, +5 % per step at 64
// rows).  What is relied on instead is the hardware's behaviour: (1) an agent-scope atomic store is performed at
// the level all XCDs share, not in the issuing XCD's L2; (2) s_waitcnt 0 returns only when those stores have been
// acknowledged there; (3) an agent-scope atomic load is served from that level, never from a stale L2 line.  The
// partial buffers are touched by nothing but these atomics while a kernel runs, so no ordinary cached copy of them
// exists.  A run-to-run bit-exactness test of the many-chunk merges guards the contract.
__device__ inline void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_agent2(float* p, float a, float b) {      // 8-byte aligned pair
  const unsigned long long v = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
  __hip_atomic_store((unsigned long long*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void publish_stores() {      // all earlier stores of this wave are acknowledged
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
}
__device__ inline int arrive(int* counter) {
  return __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline float bf2f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ inline uint16_t f2bf(float v) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ inline uint32_t pack2(float a, float b) { return (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16); }
__device__ inline uint4 pack8(const float* v) {
  return make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
}
__device__ inline void unpack8(uint4 u, float* v) {
  v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
  v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
  v[4] = __uint_as_float(u.z << 16); v[5] = __uint_as_float(u.z & 0xffff0000u);
  v[6] = __uint_as_float(u.w << 16); v[7] = __uint_as_float(u.w & 0xffff0000u);
}

__device__ inline float block_sum256(float v, float* sh) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}

inline unsigned cdiv(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

// =================================================================================================
// residual add (+ split-K reduction of the producing GEMM) + RMSNorm -> A-tiled bf16
// =================================================================================================
__global__ __launch_bounds__(256) void k_resid_norm(int h, float eps, const uint16_t* hin,
                                                    const float* part, int n_split,
                                                    int64_t split_stride, float* x,
                                                    const uint16_t* gain, uint16_t* xn_t,
                                                    uint16_t* hout) {
  __shared__ float sh[4];
  const int i = blockIdx.x;
  float* xr = x + (int64_t)i * h;
  float ss = 0.f;
  for (int j0 = threadIdx.x * 8; j0 < h; j0 += 256 * 8) {
    float v[8];
    if (hin) {
      unpack8(*(const uint4*)(hin + (int64_t)i * h + j0), v);
    } else {
      float4 a = *(const float4*)(xr + j0), b = *(const float4*)(xr + j0 + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    if (part) {
      const float* p = part + (int64_t)i * h + j0;
      for (int s = 0; s < n_split; ++s) {
        float4 a = *(const float4*)(p + s * split_stride), b = *(const float4*)(p + s * split_stride + 4);
        v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
        v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
      }
    }
    *(float4*)(xr + j0) = make_float4(v[0], v[1], v[2], v[3]);
    *(float4*)(xr + j0 + 4) = make_float4(v[4], v[5], v[6], v[7]);
    for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
    if (hout) *(uint4*)(hout + (int64_t)i * h + j0) = pack8(v);
  }
  if (!xn_t) return;
  ss = block_sum256(ss, sh);     // its barriers also order the x stores above before the re-read
  const float r = 1.0f / sqrtf(ss / (float)h + eps);
  const int KT = h >> 4;
  for (int j0 = threadIdx.x * 8; j0 < h; j0 += 256 * 8) {
    float4 a = *(const float4*)(xr + j0), b = *(const float4*)(xr + j0 + 4);
    float gv[8];
    unpack8(*(const uint4*)(gain + j0), gv);
    float v[8] = {a.x * r * gv[0], a.y * r * gv[1], a.z * r * gv[2], a.w * r * gv[3],
                  b.x * r * gv[4], b.y * r * gv[5], b.z * r * gv[6], b.w * r * gv[7]};
    *(uint4*)(xn_t + a_tiled_idx(KT, i, j0)) = pack8(v);
  }
}

// =================================================================================================
// skinny GEMM: part[s][m][n] = X[m][k in split s] . W[k][n]
//   work-group = WN waves; wave w owns the 32 columns of n-tile blockIdx.x*WN + w and all MT m-tiles;
//   blockIdx.y = split of the K range.  The X fragments of a chunk of KC k-steps are staged once in
//   LDS and shared by the WN waves; every wave streams its own weight fragments straight from HBM.
// =================================================================================================
template <int MT, int WN>
__global__ __launch_bounds__(WN * 64) void k_gemm(const uint4* __restrict__ Xt,
                                                  const uint4* __restrict__ Wt,
                                                  float* __restrict__ part, int M, int N, int KT,
                                                  int ksp, int64_t split_stride) {
  constexpr int KC = 4;
  constexpr int NF = MT * KC;                       // X fragments per chunk
  constexpr int XPT = (NF + WN - 1) / WN;           // X fragments loaded per wave
  __shared__ uint4 xs[2][NF * 64];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nt = blockIdx.x * WN + w;
  const int k0 = blockIdx.y * ksp;
  const int k1 = min(KT, k0 + ksp);
  const int nchunks = (k1 - k0 + KC - 1) / KC;
  const uint4* wp = Wt + (int64_t)nt * KT * 64 + lane;
  const uint4 zero4 = make_uint4(0, 0, 0, 0);

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

  uint4 xr[XPT], wcur[KC], wnext[KC];
  auto load_x = [&](int kc0) {
#pragma unroll
    for (int t = 0; t < XPT; ++t) {
      int f = w + t * WN;
      int mt = f / KC, kk = f - mt * KC;
      xr[t] = (f < NF && kc0 + kk < k1) ? Xt[((int64_t)mt * KT + kc0 + kk) * 64 + lane] : zero4;
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int t = 0; t < XPT; ++t) {
      int f = w + t * WN;
      if (f < NF) xs[buf][f * 64 + lane] = xr[t];
    }
  };
  auto load_w = [&](int kc0, uint4* dst) {
#pragma unroll
    for (int kk = 0; kk < KC; ++kk)
      dst[kk] = (kc0 + kk < k1) ? ld_stream(wp + (int64_t)(kc0 + kk) * 64) : zero4;
  };

  if (nchunks > 0) {
    load_x(k0);
    load_w(k0, wcur);
    store_x(0);
  }
  __syncthreads();
  for (int c = 0; c < nchunks; ++c) {
    const int buf = c & 1;
    const bool more = (c + 1 < nchunks);
    if (more) {
      load_x(k0 + (c + 1) * KC);
      load_w(k0 + (c + 1) * KC, wnext);
    }
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      bf16x8 B = __builtin_bit_cast(bf16x8, wcur[kk]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        bf16x8 A = __builtin_bit_cast(bf16x8, xs[buf][(mt * KC + kk) * 64 + lane]);
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B, acc[mt], 0, 0, 0);
      }
    }
    if (more) {
      store_x(buf ^ 1);
#pragma unroll
      for (int kk = 0; kk < KC; ++kk) wcur[kk] = wnext[kk];
    }
    __syncthreads();
  }

  float* out = part + (int64_t)blockIdx.y * split_stride + (int64_t)nt * 32 + (lane & 31);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      int m = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (m < M) out[(int64_t)m * N] = acc[mt][r];
    }
}

// =================================================================================================
// GEMM for 65..256 rows (MT = 4 or 8 row tiles): part[s][m][n] = X[m][k in split s] . W[k][n]
//   At these heights the product is close to the matrix-core roofline (arithmetic intensity = M
//   flop/byte against a ridge of about 310), so the tile is chosen for MFMA work per LDS byte:
//   a work-group of 4 waves owns 256 columns; every wave owns 64 of them (2 column tiles) and ALL
//   row tiles, i.e. 2*MT accumulator tiles (256 accumulator registers at MT = 8), and re-uses every
//   X fragment it reads from LDS for two MFMAs.  X fragments of KC k-steps are staged once per
//   work-group (double-buffered, one barrier per KC * 2 * MT MFMAs per wave); weight fragments are
//   streamed from HBM into registers one chunk ahead.
// =================================================================================================
template <int MT, int KC>
__global__ __launch_bounds__(256) void k_gemm_l(const uint4* __restrict__ Xt, const uint4* __restrict__ Wt,
                                                float* __restrict__ part, int M, int N, int KT, int ksp,
                                                int64_t split_stride, uint16_t* __restrict__ act_t) {
  constexpr int NF = MT * KC;            // X fragments per chunk
  constexpr int XPT = NF / 4;            // X fragments loaded per wave
  static_assert(NF % 4 == 0, "chunk must split evenly over 4 waves");
  __shared__ uint4 xs[2][NF * 64];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nt0 = (blockIdx.x * 4 + w) * 2;
  // blockIdx.z: block of MT row tiles (more than 256 rows are covered by several row blocks, which re-use the
  // weight tile through L2 / the memory-side cache while they run side by side)
  Xt += (int64_t)blockIdx.z * MT * KT * 64;
  part += (int64_t)blockIdx.z * MT * 32 * N;
  M -= (int)blockIdx.z * MT * 32;
  const int row0 = (int)blockIdx.z * MT * 32;
  const int k0 = blockIdx.y * ksp;
  const int k1 = min(KT, k0 + ksp);
  const int nchunks = (k1 - k0 + KC - 1) / KC;
  const uint4* wp0 = Wt + (int64_t)nt0 * KT * 64 + lane;
  const uint4* wp1 = wp0 + (int64_t)KT * 64;
  const uint4 zero4 = make_uint4(0, 0, 0, 0);

  f32x16 acc[2][MT];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nt][mt][r] = 0.f;

  uint4 wc0[KC], wc1[KC], wn0[KC], wn1[KC];
  // X fragments go from global memory straight into LDS (global_load_lds_dwordx4: lane i of the wave
  // writes bytes [16 i, 16 i + 16) after the wave-uniform LDS base), no staging registers
  auto load_x = [&](int kc0, int buf) {
#pragma unroll
    for (int t = 0; t < XPT; ++t) {
      const int f = w + t * 4, mt = f / KC, kk = f - mt * KC;
      if (kc0 + kk < k1)
        __builtin_amdgcn_global_load_lds(
            (const void __attribute__((address_space(1)))*)(Xt + ((int64_t)mt * KT + kc0 + kk) * 64 + lane),
            (void __attribute__((address_space(3)))*)(&xs[buf][f * 64]), 16, 0, 0);
      else
        xs[buf][f * 64 + lane] = zero4;
    }
  };

  if (nchunks > 0) {
    load_x(k0, 0);
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      const bool ok = k0 + kk < k1;
      wc0[kk] = ok ? ld_stream(wp0 + (int64_t)(k0 + kk) * 64) : zero4;
      wc1[kk] = ok ? ld_stream(wp1 + (int64_t)(k0 + kk) * 64) : zero4;
    }
  }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  for (int c = 0; c < nchunks; ++c) {
    const int buf = c & 1;
    const bool more = (c + 1 < nchunks);
    if (more) {
      const int kn = k0 + (c + 1) * KC;
      load_x(kn, buf ^ 1);
#pragma unroll
      for (int kk = 0; kk < KC; ++kk) {
        const bool ok = kn + kk < k1;
        wn0[kk] = ok ? ld_stream(wp0 + (int64_t)(kn + kk) * 64) : zero4;
        wn1[kk] = ok ? ld_stream(wp1 + (int64_t)(kn + kk) * 64) : zero4;
      }
    }
    // (reading the A fragments of the next k-step before the MFMAs of this one, pinned with scheduling
    // barriers, was measured 20 % slower here than the compiler's read-then-two-MFMAs order)
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      const bf16x8 B0 = __builtin_bit_cast(bf16x8, wc0[kk]);
      const bf16x8 B1 = __builtin_bit_cast(bf16x8, wc1[kk]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const bf16x8 A = __builtin_bit_cast(bf16x8, xs[buf][(mt * KC + kk) * 64 + lane]);
        acc[0][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B0, acc[0][mt], 0, 0, 0);
        acc[1][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B1, acc[1][mt], 0, 0, 0);
      }
    }
    if (more) {
#pragma unroll
      for (int kk = 0; kk < KC; ++kk) {
        wc0[kk] = wn0[kk];
        wc1[kk] = wn1[kk];
      }
    }
    __builtin_amdgcn_s_waitcnt(0);      // the next chunk's direct-to-LDS loads have landed
    __syncthreads();
  }

  if (act_t != nullptr) {
    // gate/up matrix without a K split: the wave's two column tiles are a gate tile and its up tile, so
    // silu(gate) * up is formed here and written as the A-tiled bf16 operand of the down projection
    const int col = (nt0 >> 1) * 32 + (lane & 31);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const float g = acc[0][mt][r], u = acc[1][mt][r];
        if (m < M) act_t[a_tiled_idx(N >> 5, row0 + m, col)] = f2bf(g / (1.0f + expf(-g)) * u);
      }
    return;
  }
  float* out = part + (int64_t)blockIdx.y * split_stride + (int64_t)nt0 * 32 + (lane & 31);
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < M) out[(int64_t)m * N + nt * 32] = acc[nt][mt][r];
      }
}

// =================================================================================================
// 256 x 256 tile, 8 waves, both operands through an LDS ring of R slots of TWO k-steps each, loads spread out.
// Cycle counters inside an 8-wave kernel that, like the 4-wave one above, issued all loads of the next chunk of
// four k-steps at once (weights into registers, every row half its own copy) showed a wave spending about 40 %
// of a chunk ISSUING its twelve 1 KiB loads.  The vector memory path of a compute unit accepts 64 bytes per
// cycle, so the 96 KiB that work-group pulled per chunk kept it busy for 1500 cycles -- three quarters of the
// chunk's MFMA time -- and because a wave issues in order, a wave queued behind that burst issues no MFMA
// either.  So here:
//   * every fragment is fetched once per work-group (no second fetch of the weights by the other row half):
//     16 KiB per k-step, half of the MFMA time at full rate;
//   * the four loads a wave owes per slot are placed between groups of four MFMAs, never in a burst behind
//     the barrier;
//   * one barrier per two k-steps (16 MFMAs per wave), and the fragments of the slot's second k-step are read
//     from LDS while the first is multiplied.
//   A load issued during step s fills the slot read in step s + R - 1: it has R - 2 whole steps to land.
//   k ranges of an even number of k-steps; the X operand is readable up to the end of the last row block, whose
//   rows >= M are computed and not stored.
// =================================================================================================
template <int R, int RH, bool WNT>
__global__ __launch_bounds__(256 * RH, 3 - RH) void k_gemm_l5(const uint4* __restrict__ Xt, const uint4* __restrict__ Wt,
                                                         float* __restrict__ part, int M, int N, int KT, int ksp,
                                                         int64_t split_stride, uint16_t* __restrict__ act_t, int n_z,
                                                         int G) {
  // Tile of this work-group.  n_z == 0: (column block, row block) = (blockIdx.x, blockIdx.z).  n_z > 0 (grid.x = column
  // blocks x n_z row blocks, a multiple of 8): work-groups go to the 8 XCDs round-robin by their index, so XCD
  // blockIdx.x % 8 takes the column blocks x = xcd + 8 xi and walks them in groups of G, all n_z row blocks of a group
  // before the next group.  The 32 work-groups an XCD runs at a time then share G weight tiles and 32 / G activation
  // tiles through its L2 instead of 14 and 3 in plain grid order (1024 rows x 112 column blocks): 2-4 % faster on
  // GEMMs timed back to back, 0.3 % in the passes of a prefill.
  int bx = blockIdx.x, bz = blockIdx.z;
  if (n_z > 0) {
    const int xcd = bx & 7, local = bx >> 3, per = G * n_z, g = local / per, r = local - g * per;
    bz = r / G;
    bx = xcd + 8 * (g * G + r % G);
  }
  // RH row halves of 128 rows per work-group: 2 = the 256 x 256 tile with 8 waves described above; 1 = a
  // 128 x 256 tile with 4 waves and 3 slots of 24 KiB, so that two work-groups share a compute unit (65..128
  // rows, and the last rows of a taller operand).  Rows >= M of the last row block are computed on whatever the
  // padded X operand holds (finite) and not stored.
  constexpr int NWV = 4 * RH, MTB = 4 * RH, MTW = 4;
  constexpr int kXs = 2 * MTB * 64;                 // uint4 of a slot's X part: [k-step 0 | 1][row tile][64]
  constexpr int kSlot = kXs + 1024;                 // then W: [k-step 0 | 1][column tile 0..7][64]
  constexpr int LPS = (2 * MTB + 16) / NWV;         // loads per wave and step: 2 of X, LPS - 2 of W
  extern __shared__ uint4 ring[];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, rh = (RH == 2) ? (w >> 2) : 0, wc = w & 3;
  const int nt0 = (bx * 4 + wc) * 2;
  Xt += (int64_t)bz * MTB * KT * 64;
  part += (int64_t)bz * MTB * 32 * N;
  const int row0 = bz * MTB * 32;
  const int mrows = M - row0;                       // valid rows of this row block
  const int k0 = blockIdx.y * ksp;
  const int ns = (min(KT, k0 + ksp) - k0) >> 1;     // steps of two k-steps
  const uint4* xp = Xt + (int64_t)k0 * 64 + lane;
  const uint4* wp = Wt + ((int64_t)bx * 8 * KT + k0) * 64 + lane;

  f32x16 acc[2][MTW];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nt][mt][r] = 0.f;

  // load i (0 .. LPS - 1) of step s into slot `slot`: i < 2: X k-step i, row tile w; else fragment
  // (i - 2) * NWV + w of the 16 weight fragments [k-step][column tile]
  auto issue = [&](int s, int slot, int i) {
    const uint4* src;
    uint4* dst = ring + (size_t)slot * kSlot;
    if (i < 2) {
      src = xp + ((int64_t)w * KT + 2 * s + i) * 64;
      dst += (i * MTB + w) * 64;
    } else {
      const int g = (i - 2) * NWV + w, kk = g >> 3, tile = g & 7;
      src = wp + ((int64_t)tile * KT + 2 * s + kk) * 64;
      dst += kXs + g * 64;
    }
    // WNT: the launch has one row block, so every weight line is used once: requested non-temporal (cache policy
    // bit 1), it does not claim an L2 line; the activations, which every column block re-reads, stay ordinary loads
    if (WNT && i >= 2)
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                       (void __attribute__((address_space(3)))*)dst, 16, 0, 2);
    else
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                       (void __attribute__((address_space(3)))*)dst, 16, 0, 0);
  };
  // Every step issues exactly LPS loads, so "at most LPS (R - 2) outstanding" always means that the next
  // step's slot has landed; past the end of the k range the loads re-fetch the last step into a slot that is
  // not read again (no branch in the loop body, and the counter arithmetic stays uniform).
  constexpr int kAhead = LPS * (R - 2);
  constexpr int kWaitAhead = (kAhead & 0xF) | ((kAhead >> 4) << 14) | (0x7 << 4) | (0xF << 8);   // vmcnt(kAhead) only
  if (ns > 0) {
#pragma unroll
    for (int r = 0; r < R - 1; ++r)
#pragma unroll
      for (int i = 0; i < LPS; ++i) issue(min(r, ns - 1), r, i);
    __builtin_amdgcn_s_waitcnt(kWaitAhead);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  }

  for (int s0 = 0; s0 < ns; s0 += R) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int s = s0 + r;
      if (s < ns) {
        const int sn = min(s + R - 1, ns - 1);
        const int nslot = (r + R - 1) % R;
        const uint4* base = ring + (size_t)r * kSlot;
        // (the reads are typed as MFMA operands at the load: the compiler makes a wave wait for ALL its
        // outstanding direct-to-LDS loads before an LDS read typed as an integer vector, which would drain
        // the ring every step; the slot read here is covered by the counted wait and the barrier below)
        bf16x8 a0[MTW], a1[MTW], b0[2], b1[2];
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) a0[mt] = __builtin_bit_cast(bf16x8, base[(rh * MTW + mt) * 64 + lane]);
        b0[0] = __builtin_bit_cast(bf16x8, base[kXs + (wc * 2) * 64 + lane]);
        b0[1] = __builtin_bit_cast(bf16x8, base[kXs + (wc * 2 + 1) * 64 + lane]);
        __builtin_amdgcn_sched_barrier(0);
        issue(sn, nslot, 0);
        __builtin_amdgcn_sched_barrier(0);
        // eight pairs of MFMAs (pair q: k-step q / 4, row tile q % 4); loads 1 .. LPS - 1 are spread over the
        // three points behind pairs 1, 3 and 5, and the second k-step's fragments are read behind pair 1 (while direct-to-LDS loads
        // are in flight every compiler-placed LDS wait is a full one, so reads issued earlier would not overlap)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int mt = q & 3;
          if (q < 4) {
            acc[0][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[mt], b0[0], acc[0][mt], 0, 0, 0);
            acc[1][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[mt], b0[1], acc[1][mt], 0, 0, 0);
          } else {
            acc[0][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[mt], b1[0], acc[0][mt], 0, 0, 0);
            acc[1][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[mt], b1[1], acc[1][mt], 0, 0, 0);
          }
          if ((q & 1) && q < 7) {
            __builtin_amdgcn_sched_barrier(0);
            if (q == 1) {
#pragma unroll
              for (int m2 = 0; m2 < MTW; ++m2)
                a1[m2] = __builtin_bit_cast(bf16x8, base[(MTB + rh * MTW + m2) * 64 + lane]);
              b1[0] = __builtin_bit_cast(bf16x8, base[kXs + 512 + (wc * 2) * 64 + lane]);
              b1[1] = __builtin_bit_cast(bf16x8, base[kXs + 512 + (wc * 2 + 1) * 64 + lane]);
            }
#pragma unroll
            for (int i = 1; i < LPS; ++i)
              if ((i - 1) * 3 / (LPS - 1) == (q - 1) / 2) issue(sn, nslot, i);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // bare barrier (no fence): this step's LDS reads have been consumed by its MFMAs, and the counted
        // wait is what makes the next slot's direct-to-LDS data visible
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(kWaitAhead);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0);      // the re-fetches past the end are still writing LDS

  if (act_t != nullptr) {      // gate/up without a K split: silu(gate) * up
    const int col = (nt0 >> 1) * 32 + (lane & 31);
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = (rh * MTW + mt) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const float g = acc[0][mt][r], u = acc[1][mt][r];
        if (m < mrows) act_t[a_tiled_idx(N >> 5, row0 + m, col)] = f2bf(g / (1.0f + expf(-g)) * u);
      }
    return;
  }
  float* out = part + (int64_t)blockIdx.y * split_stride + (int64_t)nt0 * 32 + (lane & 31);
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = (rh * MTW + mt) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < mrows) out[(int64_t)m * N + nt * 32] = acc[nt][mt][r];
      }
}

// =================================================================================================
// Barrier-free streaming GEMM for at most 64 rows with the consumer fused into its epilogue (NT = 2).
//   grid (N / 64, S), block = NWK waves.  The block owns two adjacent 32-column tiles and the K range of
//   split blockIdx.y; its waves take the k-steps of that range round-robin.  Every wave streams its weight
//   fragments from HBM and its X fragments from L2 (lane-linear 1 KiB loads, U k-steps ahead) with no LDS and
//   no barrier in the loop; the waves' accumulators are summed once through LDS at the end.
//   Split-K across work-groups (gridDim.y > 1) is resolved inside the kernel: every block stores its
//   fp32 partial, and the block that arrives last at the column block's counter sums all partials in
//   split order (so the result does not depend on which block was last) and runs the epilogue.
//   The RMSNorm of the A operand is folded in: A holds x * gain (bf16, not normalised) and the row
//   factor r_m = rsqrt(mean(x_m^2) + eps) is applied to the accumulators; the sums of squares come
//   from the producing epilogue as per-column-block partials (deterministic, no atomics on floats).
//   EPI_SWIGLU: act = silu(r g) * (r u)                      -> A-tiled bf16 (gate/up interleaved W)
//   EPI_RESID : x += acc; partial sums of x^2; x * gain_next -> A-tiled bf16 (or the bf16 stage output)
//   EPI_QKV   : r * acc, RoPE, q -> bf16 rows, k / v -> page slot + write-back staging
//               (W_qkv tiles are ordered so that a block holds columns j and j + 64 of one head)
// =================================================================================================
enum { EPI_SWIGLU = 1, EPI_RESID = 2, EPI_QKV = 3 };


struct FusedArgs {
  int* counters;          // one per 64-column block; zero at launch, reset by the last arriver
  const float* ssq_in;    // [64][n_ssq_in] partial sums of squares of A's rows, or null (no row factor)
  int n_ssq_in;
  float inv_h, eps;
  uint16_t* act_t;        // EPI_SWIGLU
  float* x;               // EPI_RESID
  const uint16_t* gain_next;
  uint16_t* xg_t;
  float* ssq_out;
  uint16_t* hout;
  int* ctx_advance;
  int layer;              // EPI_QKV
  const float2* cs;
  const int* ctx;
  const int* table;
  uint16_t* pool;
  uint16_t* staging;
  uint16_t* q_out;
  int Hq, Hkv, max_pages;
  int64_t page_stride, layer_off;     // device pool addressing: see Dims (layer_off = layer * layer_stride)
};

template <int MT, int NWK, int U, int EPI, int MP>
__global__ __launch_bounds__(NWK * 64) void k_gemm_f(const uint4* __restrict__ Xt,
                                                     const uint4* __restrict__ Wt,
                                                     float* __restrict__ part, FusedArgs A, int M, int N,
                                                     int KT, int ksp, int64_t split_stride) {
  constexpr int NT = 2;
  // cross-wave reduction buffer: MP row tiles per pass (NWK * MP * 8 KiB), [wave][(row tile * NT + column tile) * 4 + g]
  // [lane] holds accumulator registers 4 g .. 4 g + 3 (rows 8 g + 4 (lane >> 5) + 0 .. 3 of the tile) as one 16-byte word
  static_assert(MT % MP == 0, "whole passes");
  __shared__ float4 red[NWK][MP * NT * 4][64];
  __shared__ float rs[MT * 32];
  __shared__ int s_last;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int nt0 = blockIdx.x * NT;
  const int kb0 = blockIdx.y * ksp;
  const int kb1 = min(KT, kb0 + ksp);
  const int nsteps = (kb1 - kb0 > w) ? (kb1 - kb0 - w + NWK - 1) / NWK : 0;
  const uint4* wp = Wt + ((int64_t)nt0 * KT + kb0 + w) * 64 + lane;
  const uint4* xp = Xt + ((int64_t)kb0 + w) * 64 + lane;

  f32x16 acc[NT * MT];
#pragma unroll
  for (int t = 0; t < NT * MT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  uint4 wb[U][NT], xb[U][MT];
  auto load = [&](int j, uint4* wd, uint4* xd) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wd[nt] = ld_stream(wp + ((int64_t)nt * KT + (int64_t)j * NWK) * 64);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xd[mt] = xp[((int64_t)mt * KT + (int64_t)j * NWK) * 64];
  };
#pragma unroll
  for (int r = 0; r < U; ++r)
    if (r < nsteps) load(r, wb[r], xb[r]);

  // row factors of the folded RMSNorm: GS threads per row, each sums n_ssq_in / GS partials in a
  // fixed order, then a fixed shuffle tree (all loads of a thread are in flight together)
  if (A.ssq_in != nullptr) {
    constexpr int GS = (NWK * 64) / (MT * 32);
    const int m = tid / GS, sub = tid % GS;
    const float* p = A.ssq_in + (int64_t)m * A.n_ssq_in;
    float v[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) v[t] = (sub + t * GS < A.n_ssq_in) ? p[sub + t * GS] : 0.f;
    float sacc = 0.f;
#pragma unroll
    for (int t = 0; t < 16; ++t) sacc += v[t];
    for (int t = sub + 16 * GS; t < A.n_ssq_in; t += GS) sacc += p[t];
#pragma unroll
    for (int o2 = GS / 2; o2 > 0; o2 >>= 1) sacc += __shfl_xor(sacc, o2);
    if (sub == 0) rs[m] = 1.0f / sqrtf(sacc * A.inv_h + A.eps);
  }

  for (int j0 = 0; j0 < nsteps; j0 += U) {
#pragma unroll
    for (int r = 0; r < U; ++r) {
      const int j = j0 + r;
      if (j < nsteps) {
        bf16x8 Af[MT], Bf[NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) Af[mt] = __builtin_bit_cast(bf16x8, xb[r][mt]);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) Bf[nt] = __builtin_bit_cast(bf16x8, wb[r][nt]);
        if (j + U < nsteps) load(j + U, wb[r], xb[r]);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[nt * MT + mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Af[mt], Bf[nt], acc[nt * MT + mt], 0, 0, 0);
      }
    }
  }

  // The epilogue of output element pair (row m; columns c and c + 32 of the block), c = lane & 31, in two
  // parts: `pre` requests what the epilogue reads from memory besides the sums, `epi` computes and stores.
  // A thread that owns several pairs calls `pre` for all of them first: its stores may alias its loads as
  // far as the compiler can tell, so loads left inside `epi` would each wait behind the previous pair's
  // stores -- one exposed memory latency per pair.
  struct Pre {
    float xl, xh;      // EPI_RESID: the residual stream
    float2 cs;         // EPI_QKV: RoPE factors; position and physical page of the row's new token
    int pos, phys;
  };
  float gain_lo = 1.f, gain_hi = 1.f;      // EPI_RESID: the next norm's gain of this thread's two columns
  if (EPI == EPI_RESID && A.hout == nullptr && A.gain_next != nullptr) {
    gain_lo = bf2f(A.gain_next[blockIdx.x * 64 + (lane & 31)]);
    gain_hi = bf2f(A.gain_next[blockIdx.x * 64 + (lane & 31) + 32]);
  }
  auto pre = [&](int m, int c) {
    Pre P;
    P.xl = P.xh = 0.f;
    P.cs = make_float2(0.f, 0.f);
    P.pos = P.phys = 0;
    if (m < M) {
      if (EPI == EPI_RESID) {
        const int64_t o = (int64_t)m * N + (int64_t)blockIdx.x * 64 + c;
        P.xl = A.x[o];
        P.xh = A.x[o + 32];
      } else if (EPI == EPI_QKV) {
        const int hd = blockIdx.x >> 1, j = ((blockIdx.x & 1) << 5) + c;
        if (hd < A.Hq + A.Hkv) P.cs = A.cs[m * 64 + j];
        if (hd >= A.Hq) {
          P.pos = A.ctx[m];
          P.phys = A.table[(int64_t)m * A.max_pages + (P.pos >> 4)];
        }
      }
    }
    return P;
  };
  // All 64 lanes call `epi` together (it contains wave shuffles); the 32 lanes of a half-wave share m.
  auto epi = [&](int m, int c, float lo, float hi, const Pre& P) {
    const bool ok = m < M;
    if (EPI == EPI_SWIGLU) {
      if (ok) {
        const float r = A.ssq_in ? rs[m] : 1.0f;
        const float g = lo * r, u = hi * r;
        A.act_t[a_tiled_idx(N >> 5, m, blockIdx.x * 32 + c)] = f2bf(g / (1.0f + expf(-g)) * u);
      }
    } else if (EPI == EPI_RESID) {
      const int64_t o = (int64_t)m * N + (int64_t)blockIdx.x * 64 + c;
      float xl = 0.f, xh = 0.f;
      if (ok) {
        xl = P.xl + lo;
        xh = P.xh + hi;
        A.x[o] = xl;
        A.x[o + 32] = xh;
        if (A.hout) {
          A.hout[o] = f2bf(xl);
          A.hout[o + 32] = f2bf(xh);
        } else {
          const int n = blockIdx.x * 64 + c;
          A.xg_t[a_tiled_idx(N >> 4, m, n)] = f2bf(xl * gain_lo);
          A.xg_t[a_tiled_idx(N >> 4, m, n + 32)] = f2bf(xh * gain_hi);
        }
      }
      float ss = xl * xl + xh * xh;
#pragma unroll
      for (int o2 = 16; o2 > 0; o2 >>= 1) ss += __shfl_xor(ss, o2);
      if (ok && c == 0 && A.ssq_out) A.ssq_out[(int64_t)m * gridDim.x + blockIdx.x] = ss;
    } else {
      if (ok) {
        const float r = rs[m];
        lo *= r;
        hi *= r;
        const int hd = blockIdx.x >> 1, j = ((blockIdx.x & 1) << 5) + c;
        if (hd < A.Hq) {
          uint16_t* q = A.q_out + ((int64_t)m * A.Hq + hd) * 128;
          q[j] = f2bf(lo * P.cs.x - hi * P.cs.y);
          q[j + 64] = f2bf(hi * P.cs.x + lo * P.cs.y);
        } else {
          const int kv = (hd < A.Hq + A.Hkv) ? 0 : 1;
          const int head = hd - A.Hq - kv * A.Hkv;
          if (kv == 0) {
            const float a = lo * P.cs.x - hi * P.cs.y, b2 = hi * P.cs.x + lo * P.cs.y;
            lo = a;
            hi = b2;
          }
          const int slot = P.pos & 15;
          uint16_t* sub = A.pool + (int64_t)P.phys * A.page_stride + A.layer_off + sub_block_off(A.Hkv, 128, 0, head, kv);
          const uint16_t blo = f2bf(lo), bhi = f2bf(hi);
          if (kv == 0) {
            sub[k_sub_idx(slot, j)] = blo;
            sub[k_sub_idx(slot, j + 64)] = bhi;
          } else {
            sub[v_sub_idx(slot, j)] = blo;
            sub[v_sub_idx(slot, j + 64)] = bhi;
          }
          uint16_t* st = A.staging + (((int64_t)m * 2 + kv) * A.Hkv + head) * 128;
          st[j] = blo;
          st[j + 64] = bhi;
        }
      }
    }
  };

  const bool split = gridDim.y > 1;
#pragma unroll
  for (int mt0 = 0; mt0 < MT; mt0 += MP) {
    if (mt0) __syncthreads();
#pragma unroll
    for (int mtl = 0; mtl < MP; ++mtl)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x16& a = acc[nt * MT + mt0 + mtl];
          red[w][(mtl * NT + nt) * 4 + g][lane] = make_float4(a[4 * g], a[4 * g + 1], a[4 * g + 2], a[4 * g + 3]);
        }
    __syncthreads();            // also orders the rs[] writes before their use
    // a wave sums, over the waves in order, four rows of both column tiles
    for (int combo = w; combo < MP * 4; combo += NWK) {
      const int mtl = combo >> 2, g = combo & 3;
      float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
#pragma unroll
      for (int ww = 0; ww < NWK; ++ww) {
        const float4 a = red[ww][(mtl * NT) * 4 + g][lane], c2 = red[ww][(mtl * NT + 1) * 4 + g][lane];
        v0.x += a.x; v0.y += a.y; v0.z += a.z; v0.w += a.w;
        v1.x += c2.x; v1.y += c2.y; v1.z += c2.z; v1.w += c2.w;
      }
      const float lo4[4] = {v0.x, v0.y, v0.z, v0.w}, hi4[4] = {v1.x, v1.y, v1.z, v1.w};
      const int m0 = (mt0 + mtl) * 32 + 8 * g + 4 * (lane >> 5);
      if (split) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (m0 + i < M) {
            float* out = part + (int64_t)blockIdx.y * split_stride + (int64_t)(m0 + i) * N + (int64_t)nt0 * 32 + (lane & 31);
            st_agent(out, lo4[i]);
            st_agent(out + 32, hi4[i]);
          }
      } else {
        Pre P[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) P[i] = pre(m0 + i, lane & 31);
#pragma unroll
        for (int i = 0; i < 4; ++i) epi(m0 + i, lane & 31, lo4[i], hi4[i], P[i]);
      }
    }
  }
  if (split) {
    publish_stores();                      // this block's partial has reached the coherent level ...
    __syncthreads();
    if (tid == 0) s_last = (arrive(&A.counters[blockIdx.x]) == (int)gridDim.y - 1);
    __syncthreads();                       // ... before its arrival is counted
    if (!s_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    if (tid == 0) A.counters[blockIdx.x] = 0;
    constexpr int NE = (MT * 1024) / (NWK * 64);       // output pairs per thread
    const int S = (int)gridDim.y;
    float lo[NE], hi[NE];
    Pre P[NE];
#pragma unroll
    for (int q = 0; q < NE; ++q) {
      const int e = tid + q * NWK * 64;
      lo[q] = 0.f;
      hi[q] = 0.f;
      P[q] = pre(e >> 5, e & 31);
    }
    // the loads of UD splits are in flight together; the sums run in split order (an absent split adds 0)
    constexpr int UD = (NE <= 8) ? 4 : 2;
    for (int s0 = 0; s0 < S; s0 += UD) {
      float tl[UD][NE], th[UD][NE];
#pragma unroll
      for (int u = 0; u < UD; ++u)
#pragma unroll
        for (int q = 0; q < NE; ++q) {
          const int e = tid + q * NWK * 64, m = e >> 5, c = e & 31;
          const float* p = part + (int64_t)(s0 + u) * split_stride + (int64_t)m * N + (int64_t)nt0 * 32 + c;
          const bool ok = m < M && s0 + u < S;
          tl[u][q] = ok ? ld_agent(p) : 0.f;
          th[u][q] = ok ? ld_agent(p + 32) : 0.f;
        }
#pragma unroll
      for (int u = 0; u < UD; ++u)
#pragma unroll
        for (int q = 0; q < NE; ++q) {
          lo[q] += tl[u][q];
          hi[q] += th[u][q];
        }
    }
#pragma unroll
    for (int q = 0; q < NE; ++q) {
      const int e = tid + q * NWK * 64;
      epi(e >> 5, e & 31, lo[q], hi[q], P[q]);
    }
  }
  if (EPI == EPI_RESID && A.ctx_advance != nullptr && blockIdx.x == 0 && tid < M) A.ctx_advance[tid] += 1;
}

// first kernel of a step: x = hidden_in, sums of squares, x * gain -> A-tiled bf16, RoPE table
//   grid (b), block 256.  ssq_out[i][0] = sum of squares of row i, [1..nb) = 0.
__global__ __launch_bounds__(256) void k_first(int h, const uint16_t* __restrict__ hin, float* __restrict__ x,
                                               const uint16_t* __restrict__ gain, uint16_t* __restrict__ xg_t,
                                               float* __restrict__ ssq_out, int nb, const int* __restrict__ ctx,
                                               float2* __restrict__ cs, double base) {
  __shared__ float sh[4];
  const int i = blockIdx.x;
  const int KT = h >> 4;
  float ss = 0.f;
  for (int j0 = threadIdx.x * 8; j0 < h; j0 += 256 * 8) {
    float v[8], gv[8];
    unpack8(*(const uint4*)(hin + (int64_t)i * h + j0), v);
    unpack8(*(const uint4*)(gain + j0), gv);
    *(float4*)(x + (int64_t)i * h + j0) = make_float4(v[0], v[1], v[2], v[3]);
    *(float4*)(x + (int64_t)i * h + j0 + 4) = make_float4(v[4], v[5], v[6], v[7]);
#pragma unroll
    for (int e = 0; e < 8; ++e) { ss += v[e] * v[e]; v[e] *= gv[e]; }
    *(uint4*)(xg_t + a_tiled_idx(KT, i, j0)) = pack8(v);
  }
  ss = block_sum256(ss, sh);
  for (int t = threadIdx.x; t < nb; t += 256) ssq_out[(int64_t)i * nb + t] = (t == 0) ? ss : 0.f;
  if (threadIdx.x < 64) {
    const int j = threadIdx.x;
    const double ang = (double)ctx[i] * pow(base, -2.0 * (double)j / 128.0);
    cs[i * 64 + j] = make_float2((float)cos(ang), (float)sin(ang));
  }
}

// =================================================================================================
// RoPE + KV append + write-back staging; also reduces the split-K partials of the QKV GEMM
//   grid (b, Hq + 2 Hkv), block 64: thread j rotates the pair (j, j + 64)
// =================================================================================================
__global__ __launch_bounds__(64) void k_rope_append(Dims D, int layer, const float* part, int n_split,
                                                    int64_t split_stride, const float2* cs,
                                                    const int* ctx, const int* table, uint16_t* pool,
                                                    uint16_t* staging, uint16_t* q_out) {
  const int i = blockIdx.x, hd = blockIdx.y, j = threadIdx.x;
  // the tiled W_qkv orders the four 32-column tiles of a head as (0, 2, 1, 3): element j of the
  // head is GEMM output column j (j < 32), j + 32 (32 <= j < 64), j - 32 (64 <= j < 96), j (j >= 96)
  const float* row = part + (int64_t)i * D.Nqkv + (int64_t)hd * 128;
  const int c_lo = (j < 32) ? j : j + 32, c_hi = (j < 32) ? j + 32 : j + 64;
  float lo = 0.f, hi = 0.f;
  for (int s = 0; s < n_split; ++s) {
    lo += row[s * split_stride + c_lo];
    hi += row[s * split_stride + c_hi];
  }
  const int pos = ctx[i];
  if (hd < D.Hq) {
    float2 c = cs[i * 64 + j];
    uint16_t* q = q_out + ((int64_t)i * D.Hq + hd) * 128;
    q[j] = f2bf(lo * c.x - hi * c.y);
    q[j + 64] = f2bf(hi * c.x + lo * c.y);
    return;
  }
  const int kv = (hd < D.Hq + D.Hkv) ? 0 : 1;
  const int head = hd - D.Hq - kv * D.Hkv;
  if (kv == 0) {
    float2 c = cs[i * 64 + j];
    float a = lo * c.x - hi * c.y, b2 = hi * c.x + lo * c.y;
    lo = a;
    hi = b2;
  }
  const int phys = table[(int64_t)i * D.max_pages + (pos >> 4)];
  const int slot = pos & 15;
  uint16_t* sub = pool + (int64_t)phys * D.page_stride + (int64_t)layer * D.layer_stride + sub_block_off(D.Hkv, 128, 0, head, kv);
  const uint16_t blo = f2bf(lo), bhi = f2bf(hi);
  if (kv == 0) {
    sub[k_sub_idx(slot, j)] = blo;
    sub[k_sub_idx(slot, j + 64)] = bhi;
  } else {
    sub[v_sub_idx(slot, j)] = blo;
    sub[v_sub_idx(slot, j + 64)] = bhi;
  }
  uint16_t* st = staging + (((int64_t)i * 2 + kv) * D.Hkv + head) * 128;   // [b][2][Hkv][128]
  st[j] = blo;
  st[j + 64] = bhi;
}

// =================================================================================================
// GQA paged decode attention, split-K over the context
//   A wave owns a run of consecutive pages of one (sequence, kv head) and keeps an online-softmax
//   state for the G query heads of the group (padded to the 16 columns of the MFMA tile).
//   S^T[tok][head] = K[tok][:] . Q[head][:]      mfma_f32_16x16x32_bf16   (A = K page, B = Q)
//   O^T[d][head]  += V^T[d][tok] . P^T[tok][head] mfma_f32_16x16x16_bf16   (A = V page, B = P)
//   The S^T accumulator layout (lane: column = head, 4 consecutive tokens) is exactly the B-operand
//   layout of the second product, so P never leaves its registers.
// =================================================================================================
// chunk j of a sequence covers pages [j*CP, min(npages, (j+1)*CP)): the boundaries do not depend on
// the sequence's length, so the block-table entries can be requested before the length has arrived
__device__ inline void chunk_range(int n_tok, int CP, int chunk, int& nch, int& p0, int& p1) {
  const int npages = (n_tok + 15) >> 4;
  nch = (npages + CP - 1) / CP;
  p0 = chunk * CP;
  p1 = min(npages, p0 + CP);
}

constexpr int kORow = 132;   // padded LDS row of the cross-wave merge

// Three waves per SIMD: the body needs 145 registers, and left to itself the compiler takes 181.
template <int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(3, 3))) void k_attn(
    Dims D, int layer, const uint16_t* __restrict__ q, const uint16_t* __restrict__ pool,
    const int* __restrict__ table, const int* __restrict__ ctx, float* __restrict__ part_o,
    float* __restrict__ part_ml, int CP, int NCH, int* __restrict__ counters, uint16_t* __restrict__ out_t,
    const int* __restrict__ order) {
  extern __shared__ float so[];                 // [NW][G][kORow], later [G][kORow] merged
  __shared__ float sm[NW][16], sl[NW][16];
  __shared__ int s_last;
  // work-groups are dispatched in grid order: `order` lists the sequences longest first, so that the
  // long ones start early and the kernel's tail consists of short ones
  // Work-groups go to the 8 XCDs round-robin in grid order; with the KV head taken from blockIdx.y alone every XCD
  // would read one fixed 8 KiB slot (K and V of its head) of each page's 64 KiB layer block for the whole launch.  Wave times differ
  // between slots and between XCDs (cycle counters: up to 40 %), and a slow slot that stays on a slow XCD sets the
  // launch time; rotating the head by the sequence index gives every XCD all slots (-6 % on a one-layer stage,
  // whose pages are 64 KiB apart; -1 % with eight layers per page).
  const int chunk = blockIdx.x, c = (blockIdx.y + blockIdx.z) % gridDim.y, i = order[blockIdx.z];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, n = lane & 15, g = lane >> 4;
  const int G = D.G;
  // issue the three independent first loads together: length, this wave's page ids, Q
  int my_page = 0;
  {
    const int pidx = chunk * CP + w + NW * lane;          // this wave's pages: p0 + w, p0 + w + NW, ...
    if (NW * lane + w < CP && pidx < D.max_pages) my_page = table[(int64_t)i * D.max_pages + pidx];
  }
  const int n_tok = ctx[i] + 1;
  int nch, p0, p1;
  chunk_range(n_tok, CP, chunk, nch, p0, p1);
  if (chunk >= nch) return;

  // Q fragments: B operand, lane (n, g) holds Q[head n][kk*32 + 8g .. +8]
  bf16x8 qf[4];
  {
    const uint16_t* qrow = q + ((int64_t)i * D.Hq + c * G + (n < G ? n : 0)) * 128 + g * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 v = (n < G) ? *(const uint4*)(qrow + kk * 32) : make_uint4(0, 0, 0, 0);
      qf[kk] = __builtin_bit_cast(bf16x8, v);
    }
  }
  // at most 64 pages per wave: the host keeps CP <= 64 * NW
  const int span = p1 - p0;
  const int npw = (span > w) ? ((span - w + NW - 1) / NW) : 0;
  const int64_t sub_off = (int64_t)layer * D.layer_stride + sub_block_off(D.Hkv, 128, 0, c, 0);
  const float scale_log2 = 1.4426950408889634f / sqrtf(128.0f);

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 oacc[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // two register buffers: the next page is requested before the current one is consumed.  Every K / V line is used
  // exactly once per launch, so the loads are marked non-temporal: as ordinary loads, which claim an L2 line each,
  // the same kernel streamed 10 % slower (256 sequences x 2048 tokens, 8 KV heads: 386 -> 349 us per launch).
  uint4 kf[2][4], vf[2][4];
  auto load_page = [&](int t, uint4* kd, uint4* vd) {
    const int phys = __builtin_amdgcn_readfirstlane(__shfl(my_page, t));
    const uint4* base = (const uint4*)(pool + (int64_t)phys * D.page_stride + sub_off) + lane;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kd[kk] = ld_stream(base + kk * 64);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) vd[jj] = ld_stream(base + 256 + jj * 64);
  };
  if (npw > 0) load_page(0, kf[0], vf[0]);
  for (int t0 = 0; t0 < npw; t0 += 2) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int t = t0 + r;
      if (t < npw) {
        if (t + 1 < npw) load_page(t + 1, kf[r ^ 1], vf[r ^ 1]);
        f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[r][kk]), qf[kk],
                                                         sacc, 0, 0, 0);
        const int tok0 = ((p0 + w + NW * t) << 4) + 4 * g;
        float s[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) s[e] = (tok0 + e < n_tok) ? sacc[e] * scale_log2 : -INFINITY;
        float mloc = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float m_new = fmaxf(m_run, mloc);
        const float alpha = exp2f(m_run - m_new);
        float p[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) p[e] = exp2f(s[e] - m_new);
        float lsum = (p[0] + p[1]) + (p[2] + p[3]);
        lsum += __shfl_xor(lsum, 16);
        lsum += __shfl_xor(lsum, 32);
        l_run = l_run * alpha + lsum;
        m_run = m_new;
        const uint2 pp = make_uint2(pack2(p[0], p[1]), pack2(p[2], p[3]));
        const s16x4 pf = __builtin_bit_cast(s16x4, pp);
        // slots past the sequence's last token hold whatever the page held before: their weight is
        // 0, but 0 * NaN is NaN, so the V operand of the last (partial) page is masked as well
        uint32_t vm0 = 0xffffffffu, vm1 = 0xffffffffu;
        if (tok0 + 3 >= n_tok) {
          const int valid = n_tok - tok0;                       // tokens tok0 .. tok0+3 of this lane
          vm0 = valid >= 2 ? 0xffffffffu : (valid == 1 ? 0x0000ffffu : 0u);
          vm1 = valid >= 4 ? 0xffffffffu : (valid == 3 ? 0x0000ffffu : 0u);
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const s16x4 v0 = __builtin_bit_cast(s16x4, make_uint2(vf[r][jj].x & vm0, vf[r][jj].y & vm1));
          const s16x4 v1 = __builtin_bit_cast(s16x4, make_uint2(vf[r][jj].z & vm0, vf[r][jj].w & vm1));
          oacc[2 * jj] = oacc[2 * jj] * alpha;
          oacc[2 * jj + 1] = oacc[2 * jj + 1] * alpha;
          oacc[2 * jj] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v0, pf, oacc[2 * jj], 0, 0, 0);
          oacc[2 * jj + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v1, pf, oacc[2 * jj + 1], 0, 0, 0);
        }
      }
    }
  }

  // ---- merge the NW waves of the block through LDS -------------------------------------------------
  if (g == 0) { sm[w][n] = m_run; sl[w][n] = l_run; }
  __syncthreads();
  float m_blk = sm[0][n];
#pragma unroll
  for (int ww = 1; ww < NW; ++ww) m_blk = fmaxf(m_blk, sm[ww][n]);
  float l_blk = 0.f;
#pragma unroll
  for (int ww = 0; ww < NW; ++ww) l_blk += sl[ww][n] * exp2f(sm[ww][n] - m_blk);
  {
    const float f = exp2f(m_run - m_blk);          // 0 for a wave that had no page
    if (n < G) {
      float* dst = so + ((int64_t)w * G + n) * kORow + 4 * g;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        f32x4 v = oacc[dt] * f;
        *(float4*)(dst + dt * 16) = make_float4(v[0], v[1], v[2], v[3]);
      }
    }
  }
  __syncthreads();
  // thread e8 < G*16 owns 8 consecutive output dimensions of one query head
  const int KTo = D.Hq * 128 / 16;
  const int nn8 = tid >> 4, dd8 = (tid & 15) * 8;
  const bool owner = tid < G * 16;
  float o8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float m8 = 0.f, l8 = 1.f;
  if (owner) {
    m8 = sm[0][nn8];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) m8 = fmaxf(m8, sm[ww][nn8]);
    l8 = 0.f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) l8 += sl[ww][nn8] * exp2f(sm[ww][nn8] - m8);
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
      const float* src = so + ((int64_t)ww * G + nn8) * kORow + dd8;
      const float4 a = *(const float4*)src, b2 = *(const float4*)(src + 4);
      o8[0] += a.x; o8[1] += a.y; o8[2] += a.z; o8[3] += a.w;
      o8[4] += b2.x; o8[5] += b2.y; o8[6] += b2.z; o8[7] += b2.w;
    }
  }
  if (nch == 1) {          // the block saw the whole context: normalise and write the A-tiled bf16 row
    if (owner) {
      const float inv = 1.0f / l8;
#pragma unroll
      for (int e = 0; e < 8; ++e) o8[e] *= inv;
      *(uint4*)(out_t + a_tiled_idx(KTo, i, (c * G + nn8) * 128 + dd8)) = pack8(o8);
    }
    return;
  }
  // several chunks: publish this block's (m, l, o); the block that arrives last at the
  // (sequence, kv head) counter merges all chunks, in chunk order
  if (owner) {
    float* dst = part_o + (((int64_t)i * D.Hq + c * G + nn8) * NCH + chunk) * 128 + dd8;
#pragma unroll
    for (int e = 0; e < 8; e += 2) st_agent2(dst + e, o8[e], o8[e + 1]);
    if (dd8 == 0) st_agent2(part_ml + (((int64_t)i * D.Hq + c * G + nn8) * NCH + chunk) * 2, m8, l8);
  }
  publish_stores();
  __syncthreads();
  if (tid == 0) s_last = (arrive(&counters[i * D.Hkv + c]) == nch - 1);
  __syncthreads();
  if (!s_last) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  if (tid == 0) counters[i * D.Hkv + c] = 0;
  if (owner) {
    const float* ml = part_ml + ((int64_t)i * D.Hq + c * G + nn8) * NCH * 2;
    const float* po = part_o + ((int64_t)i * D.Hq + c * G + nn8) * NCH * 128 + dd8;
    float m_tot = -INFINITY;
    for (int j = 0; j < nch; ++j) m_tot = fmaxf(m_tot, ld_agent(ml + 2 * j));
    float l = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < nch; ++j) {
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = ld_agent(po + (int64_t)j * 128 + e);
      const float fj = exp2f(ld_agent(ml + 2 * j) - m_tot);
      l += ld_agent(ml + 2 * j + 1) * fj;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] += v[e] * fj;
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] *= inv;
    *(uint4*)(out_t + a_tiled_idx(KTo, i, (c * G + nn8) * 128 + dd8)) = pack8(o);
  }
}

// The same attention with a wave, not a work-group, as the worker: wave (blockIdx.x * NW + w) takes item (chunk, KV
// head, sequence) of that number and streams all of the chunk's pages (up to 256: four registers of page ids) by
// itself; the NW waves of a work-group share nothing and never meet at a barrier.  In k_attn the waves of an item
// drift apart while they stream and the faster ones wait at the merge for the slowest: a copy of k_attn without
// its merge ran 332 us where k_attn runs 348 (256 sequences x 2048 tokens, 8 KV heads), and the loss grows as the
// items shrink (66 / 33 pages per item: +48 / +100 us with the merge, +3 / +7 us without).  A chunk that is the whole
// context is normalised and written by its wave; several chunks are merged by the wave that arrives last at the
// (sequence, KV head) counter, as in k_attn.  For launches with enough items to fill the chip (the host decides).
template <int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(3, 3))) void k_attn_w(
    Dims D, int layer, const uint16_t* __restrict__ q, const uint16_t* __restrict__ pool,
    const int* __restrict__ table, const int* __restrict__ ctx, float* __restrict__ part_o,
    float* __restrict__ part_ml, int CP, int NCH, int* __restrict__ counters, uint16_t* __restrict__ out_t,
    const int* __restrict__ order, int n_items) {
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, n = lane & 15, g = lane >> 4;
  const int G = D.G, Hkv = D.Hkv;
  const int j = blockIdx.x * NW + w;
  if (j >= n_items) return;
  // item j of a (chunks, heads, sequences) grid; the head is rotated by the sequence as in k_attn
  const int chunk = j % NCH, yz = j / NCH, y = yz % Hkv, z = yz / Hkv;
  const int c = (y + z) % Hkv, i = order[z];
  // length, the first 256 page ids (lane l holds pages p0 + l, + 64, + 128, + 192 of the chunk) and Q are requested
  // together
  int mp[4];
  auto load_ids = [&](int first) {                // page ids of the chunk's pages first .. first + 255
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int off = first + lane + 64 * r, pidx = chunk * CP + off;
      mp[r] = (off < CP && pidx < D.max_pages) ? table[(int64_t)i * D.max_pages + pidx] : 0;
    }
  };
  load_ids(0);
  const int n_tok = ctx[i] + 1;
  int nch, p0, p1;
  chunk_range(n_tok, CP, chunk, nch, p0, p1);
  if (chunk >= nch) return;                       // a sequence shorter than the longest has fewer chunks
  const int np = p1 - p0;                         // >= 1

  bf16x8 qf[4];                                   // B operand, lane (n, g) holds Q[head n][kk*32 + 8g .. +8]
  {
    const uint16_t* qrow = q + ((int64_t)i * D.Hq + c * G + (n < G ? n : 0)) * 128 + g * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 v = (n < G) ? *(const uint4*)(qrow + kk * 32) : make_uint4(0, 0, 0, 0);
      qf[kk] = __builtin_bit_cast(bf16x8, v);
    }
  }
  const int64_t sub_off = (int64_t)layer * D.layer_stride + sub_block_off(Hkv, 128, 0, c, 0);
  const float scale_log2 = 1.4426950408889634f / sqrtf(128.0f);
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 oacc[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint4 kf[2][4], vf[2][4];
  auto load_page = [&](int t, uint4* kd, uint4* vd) {
    const int r = t >> 6;
    const int ids = r == 0 ? mp[0] : r == 1 ? mp[1] : r == 2 ? mp[2] : mp[3];
    const int phys = __builtin_amdgcn_readfirstlane(__shfl(ids, t & 63));
    const uint4* base = (const uint4*)(pool + (int64_t)phys * D.page_stride + sub_off) + lane;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kd[kk] = ld_stream(base + kk * 64);      // used once: see k_attn
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) vd[jj] = ld_stream(base + 256 + jj * 64);
  };
  auto consume_page = [&](int t, const uint4* kq, const uint4* vq) {
    f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kq[kk]), qf[kk], sacc, 0, 0, 0);
    const int tok0 = ((p0 + t) << 4) + 4 * g;
    float s[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) s[e] = (tok0 + e < n_tok) ? sacc[e] * scale_log2 : -INFINITY;
    float mloc = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    const float m_new = fmaxf(m_run, mloc);
    const float alpha = exp2f(m_run - m_new);
    float p[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) p[e] = exp2f(s[e] - m_new);
    float lsum = (p[0] + p[1]) + (p[2] + p[3]);
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    l_run = l_run * alpha + lsum;
    m_run = m_new;
    const uint2 pp = make_uint2(pack2(p[0], p[1]), pack2(p[2], p[3]));
    const s16x4 pf = __builtin_bit_cast(s16x4, pp);
    // the V operand of the last (partial) page is masked: see k_attn
    uint32_t vm0 = 0xffffffffu, vm1 = 0xffffffffu;
    if (tok0 + 3 >= n_tok) {
      const int valid = n_tok - tok0;
      vm0 = valid >= 2 ? 0xffffffffu : (valid == 1 ? 0x0000ffffu : 0u);
      vm1 = valid >= 4 ? 0xffffffffu : (valid == 3 ? 0x0000ffffu : 0u);
    }
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const s16x4 v0 = __builtin_bit_cast(s16x4, make_uint2(vq[jj].x & vm0, vq[jj].y & vm1));
      const s16x4 v1 = __builtin_bit_cast(s16x4, make_uint2(vq[jj].z & vm0, vq[jj].w & vm1));
      oacc[2 * jj] = oacc[2 * jj] * alpha;
      oacc[2 * jj + 1] = oacc[2 * jj + 1] * alpha;
      oacc[2 * jj] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v0, pf, oacc[2 * jj], 0, 0, 0);
      oacc[2 * jj + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v1, pf, oacc[2 * jj + 1], 0, 0, 0);
    }
  };
  // two buffers, one page requested ahead; no branch between a request and the wait for the older page in the
  // steady part (the compiler would otherwise wait for both).  The page ids in registers reach 256 pages; a longer
  // chunk goes window by window (one exposed load of ids and one of a first page per 256 pages).
  for (int first = 0; first < np; first += 256) {
    if (first) load_ids(first);
    const int nw = min(256, np - first);
    load_page(0, kf[0], vf[0]);
    int t = 0;
    for (; t + 2 < nw; t += 2) {
      load_page(t + 1, kf[1], vf[1]);
      consume_page(first + t, kf[0], vf[0]);
      load_page(t + 2, kf[0], vf[0]);
      consume_page(first + t + 1, kf[1], vf[1]);
    }
    if (t + 1 < nw) {
      load_page(t + 1, kf[1], vf[1]);
      consume_page(first + t, kf[0], vf[0]);
      consume_page(first + t + 1, kf[1], vf[1]);
    } else {
      consume_page(first + t, kf[0], vf[0]);
    }
  }

  // lane (n, g) holds, of query head n, output dimensions 16 dt + 4 g .. + 3 (dt = 0..7) and the head's (m, l)
  const int KTo = D.Hq * 128 / 16;
  const int head = c * G + n;
  if (nch == 1) {
    if (n < G) {
      const float inv = 1.0f / l_run;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const f32x4 v = oacc[dt] * inv;
        *(uint2*)(out_t + a_tiled_idx(KTo, i, head * 128 + dt * 16 + 4 * g)) = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
      }
    }
    return;
  }
  // several chunks: publish (m, l, o); the wave that arrives last merges them in chunk order
  if (n < G) {
    float* dst = part_o + (((int64_t)i * D.Hq + head) * NCH + chunk) * 128 + 4 * g;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      st_agent2(dst + dt * 16, oacc[dt][0], oacc[dt][1]);
      st_agent2(dst + dt * 16 + 2, oacc[dt][2], oacc[dt][3]);
    }
    if (g == 0) st_agent2(part_ml + (((int64_t)i * D.Hq + head) * NCH + chunk) * 2, m_run, l_run);
  }
  publish_stores();
  int old = 0;
  if (lane == 0) old = arrive(&counters[i * Hkv + c]);
  old = __builtin_amdgcn_readfirstlane(old);
  if (old != nch - 1) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  if (lane == 0) counters[i * Hkv + c] = 0;
  if (n < G) {
    const float* ml = part_ml + ((int64_t)i * D.Hq + head) * NCH * 2;
    const float* po = part_o + ((int64_t)i * D.Hq + head) * NCH * 128 + 4 * g;
    float m_tot = -INFINITY;
    for (int jc = 0; jc < nch; ++jc) m_tot = fmaxf(m_tot, ld_agent(ml + 2 * jc));
    float l = 0.f;
    f32x4 o[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int jc = 0; jc < nch; ++jc) {
      f32x4 v[8];
#pragma unroll
      for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int e = 0; e < 4; ++e) v[dt][e] = ld_agent(po + (int64_t)jc * 128 + dt * 16 + e);
      const float fj = exp2f(ld_agent(ml + 2 * jc) - m_tot);
      l += ld_agent(ml + 2 * jc + 1) * fj;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) o[dt] += v[dt] * fj;
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      const f32x4 v = o[dt] * inv;
      *(uint2*)(out_t + a_tiled_idx(KTo, i, head * 128 + dt * 16 + 4 * g)) = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
    }
  }
}

// =================================================================================================
// Causal attention of a prefill chunk: R rows = R consecutive new tokens of ONE sequence, row r at
// position pos0 + r, whose K,V are already in the sequence's pages.
//   grid (row tiles of 16, longest first; query heads), block NW waves.  The 16 columns of the MFMA tiles are
//   16 query rows of one head (in the decode kernel they are the heads of a group); the waves take the pages
//   of the tile's visible context round-robin and merge once through LDS, exactly as in the decode kernel.
//   Column n sees tokens <= pos0 + r0 + n.  At most 64 * NW pages (the host checks).
// =================================================================================================
template <int NW>
__global__ __launch_bounds__(NW * 64, 2) void k_attn_prefill(Dims D, int layer, const uint16_t* __restrict__ q,
                                                          const uint16_t* __restrict__ pool,
                                                          const int* __restrict__ table, int pos0, int R,
                                                          uint16_t* __restrict__ out_t) {
  __shared__ float so[NW][16][kORow];
  __shared__ float sm[NW][16], sl[NW][16];
  const int tile = (int)gridDim.x - 1 - (int)blockIdx.x, hq = blockIdx.y, c = hq / D.G;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, n = lane & 15, g = lane >> 4;
  const int r0 = tile * 16;
  const int row = min(r0 + n, R - 1);                     // rows past the chunk repeat its last row (not written)
  const int n_vis = pos0 + row + 1;                       // tokens this column sees
  const int n_total = pos0 + R;                           // tokens the pages hold
  const int npages = (pos0 + min(r0 + 15, R - 1)) / 16 + 1;
  int my_page = 0;
  {
    const int pidx = w + NW * lane;                       // this wave's pages: w, w + NW, ...
    if (pidx < npages) my_page = table[pidx];
  }
  bf16x8 qf[4];
  {
    const uint16_t* qrow = q + ((int64_t)row * D.Hq + hq) * 128 + g * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, *(const uint4*)(qrow + kk * 32));
  }
  const int npw = (npages > w) ? ((npages - w + NW - 1) / NW) : 0;
  const int64_t sub_off = (int64_t)layer * D.layer_stride + sub_block_off(D.Hkv, 128, 0, c, 0);
  const float scale_log2 = 1.4426950408889634f / sqrtf(128.0f);

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 oacc[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // The softmax bookkeeping of an update (maximum and sum across the wave, the rescale of 32 accumulator
  // registers) costs more vector instructions than the scores themselves, so an update covers TWO pages
  // (32 tokens): the kernel is bound by that arithmetic, not by memory.  Groups of two pages are
  // double-buffered; a missing second page (odd count) re-reads the wave's first page and is masked out.
  uint4 kf[2][2][4], vf[2][2][4];
  auto load_page = [&](int t, uint4* kd, uint4* vd) {
    const int phys = __builtin_amdgcn_readfirstlane(__shfl(my_page, t < npw ? t : 0));
    const uint4* base = (const uint4*)(pool + (int64_t)phys * D.page_stride + sub_off) + lane;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kd[kk] = base[kk * 64];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) vd[jj] = base[256 + jj * 64];
  };
  const int ngr = (npw + 1) / 2;
  if (ngr > 0) {
    load_page(0, kf[0][0], vf[0][0]);
    load_page(1, kf[0][1], vf[0][1]);
  }
  for (int g0 = 0; g0 < ngr; g0 += 2) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int gi = g0 + r;
      if (gi < ngr) {
        if (gi + 1 < ngr) {
          load_page(2 * gi + 2, kf[r ^ 1][0], vf[r ^ 1][0]);
          load_page(2 * gi + 3, kf[r ^ 1][1], vf[r ^ 1][1]);
        }
        f32x4 sacc[2];
        float sv[2][4];
        int tok0[2];
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          sacc[p] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            sacc[p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[r][p][kk]), qf[kk],
                                                              sacc[p], 0, 0, 0);
          const int t = 2 * gi + p;
          tok0[p] = ((w + NW * t) << 4) + 4 * g;
          const bool have = t < npw;                     // wave-uniform: the second page of the last group
#pragma unroll
          for (int e = 0; e < 4; ++e)
            sv[p][e] = (have && tok0[p] + e < n_vis) ? sacc[p][e] * scale_log2 : -INFINITY;
        }
        float mloc = fmaxf(fmaxf(fmaxf(sv[0][0], sv[0][1]), fmaxf(sv[0][2], sv[0][3])),
                           fmaxf(fmaxf(sv[1][0], sv[1][1]), fmaxf(sv[1][2], sv[1][3])));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float m_new = fmaxf(m_run, mloc);
        // a column may see nothing of this wave's pages so far: keep the exponents finite
        const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f(m_run - m_ref);
        float pr[2][4];
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
          for (int e = 0; e < 4; ++e) pr[p][e] = exp2f(sv[p][e] - m_ref);
        float lsum = ((pr[0][0] + pr[0][1]) + (pr[0][2] + pr[0][3])) + ((pr[1][0] + pr[1][1]) + (pr[1][2] + pr[1][3]));
        lsum += __shfl_xor(lsum, 16);
        lsum += __shfl_xor(lsum, 32);
        l_run = l_run * alpha + lsum;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) oacc[dt] = oacc[dt] * alpha;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          const uint2 pp = make_uint2(pack2(pr[p][0], pr[p][1]), pack2(pr[p][2], pr[p][3]));
          const s16x4 pf = __builtin_bit_cast(s16x4, pp);
          // slots past the last appended token hold whatever the page held before (0 * NaN is NaN)
          uint32_t vm0 = 0xffffffffu, vm1 = 0xffffffffu;
          if (2 * gi + p >= npw) {
            vm0 = vm1 = 0u;                              // the stand-in for a missing second page: V = 0
          } else if (tok0[p] + 3 >= n_total) {
            const int valid = n_total - tok0[p];
            vm0 = valid >= 2 ? 0xffffffffu : (valid == 1 ? 0x0000ffffu : 0u);
            vm1 = valid >= 4 ? 0xffffffffu : (valid == 3 ? 0x0000ffffu : 0u);
          }
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const s16x4 v0 = __builtin_bit_cast(s16x4, make_uint2(vf[r][p][jj].x & vm0, vf[r][p][jj].y & vm1));
            const s16x4 v1 = __builtin_bit_cast(s16x4, make_uint2(vf[r][p][jj].z & vm0, vf[r][p][jj].w & vm1));
            oacc[2 * jj] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v0, pf, oacc[2 * jj], 0, 0, 0);
            oacc[2 * jj + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(v1, pf, oacc[2 * jj + 1], 0, 0, 0);
          }
        }
      }
    }
  }

  // ---- merge the NW waves through LDS (wave 0 always holds page 0, which every column sees) ---------
  if (g == 0) { sm[w][n] = m_run; sl[w][n] = l_run; }
  __syncthreads();
  float m_blk = sm[0][n];
#pragma unroll
  for (int ww = 1; ww < NW; ++ww) m_blk = fmaxf(m_blk, sm[ww][n]);
  {
    const float f = exp2f(m_run - m_blk);          // 0 for a wave that saw nothing of this column
    float* dst = &so[w][n][4 * g];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      f32x4 v = oacc[dt] * f;
      *(float4*)(dst + dt * 16) = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
  __syncthreads();
  // thread (column nn8, 8 consecutive output dimensions): 16 columns x 16 groups = 256 threads
  const int KTo = D.Hq * 128 / 16;
  for (int e8 = tid; e8 < 256; e8 += NW * 64) {
    const int nn8 = e8 >> 4, dd8 = (e8 & 15) * 8;
    if (r0 + nn8 >= R) continue;
    float m8 = sm[0][nn8];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) m8 = fmaxf(m8, sm[ww][nn8]);
    float l8 = 0.f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) l8 += sl[ww][nn8] * exp2f(sm[ww][nn8] - m8);
    float o8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
      const float* src = &so[ww][nn8][dd8];
      const float4 a = *(const float4*)src, b2 = *(const float4*)(src + 4);
      o8[0] += a.x; o8[1] += a.y; o8[2] += a.z; o8[3] += a.w;
      o8[4] += b2.x; o8[5] += b2.y; o8[6] += b2.z; o8[7] += b2.w;
    }
    const float inv = 1.0f / l8;
#pragma unroll
    for (int e = 0; e < 8; ++e) o8[e] *= inv;
    *(uint4*)(out_t + a_tiled_idx(KTo, r0 + nn8, hq * 128 + dd8)) = pack8(o8);
  }
}

// =================================================================================================
// SwiGLU over the split-K partials of the gate/up GEMM -> A-tiled bf16 input of the down GEMM
// =================================================================================================
__global__ __launch_bounds__(256) void k_swiglu(int b, int F, const float* part, int n_split,
                                                int64_t split_stride, uint16_t* act_t) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int F8 = F >> 3;
  if (idx >= (int64_t)b * F8) return;
  const int i = (int)(idx / F8), f0 = (int)(idx - (int64_t)i * F8) * 8;
  const int col = (f0 >> 5) * 64 + (f0 & 31);          // gate columns; the up columns follow at +32
  const float* p = part + (int64_t)i * 2 * F + col;
  float gt[8] = {0, 0, 0, 0, 0, 0, 0, 0}, up[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int s = 0; s < n_split; ++s) {
    const float* ps = p + s * split_stride;
    float4 a = *(const float4*)ps, b2 = *(const float4*)(ps + 4);
    float4 c = *(const float4*)(ps + 32), d2 = *(const float4*)(ps + 36);
    gt[0] += a.x; gt[1] += a.y; gt[2] += a.z; gt[3] += a.w;
    gt[4] += b2.x; gt[5] += b2.y; gt[6] += b2.z; gt[7] += b2.w;
    up[0] += c.x; up[1] += c.y; up[2] += c.z; up[3] += c.w;
    up[4] += d2.x; up[5] += d2.y; up[6] += d2.z; up[7] += d2.w;
  }
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = gt[e] / (1.0f + expf(-gt[e])) * up[e];
  *(uint4*)(act_t + a_tiled_idx(F >> 4, i, f0)) = pack8(v);
}

}  // namespace

// ---- launchers -------------------------------------------------------------------------------------
void resid_norm(hipStream_t s, int b, int h, float eps, const uint16_t* hin, const float* part,
                int n_split, int64_t split_stride, float* x, const uint16_t* gain, uint16_t* xn_t,
                uint16_t* hout) {
  hipLaunchKernelGGL(k_resid_norm, dim3(b), dim3(256), 0, s, h, eps, hin, part, n_split, split_stride,
                     x, gain, xn_t, hout);
}

template <int WN>
static void gemm_wn(hipStream_t s, const uint16_t* Xt, const uint16_t* Wt, float* part, int M, int K,
                    int N, int n_split) {
  const int KT = K / 16;
  const int ksp = (KT + n_split - 1) / n_split;
  const int MT = (M + 31) / 32;
  const int64_t stride = (int64_t)MT * 32 * N;
  dim3 grid(N / (32 * WN), n_split), block(WN * 64);
  const uint4* X4 = (const uint4*)Xt;
  const uint4* W4 = (const uint4*)Wt;
#define PMX_GEMM_CASE(mt)                                                                         \
  hipLaunchKernelGGL((k_gemm<mt, WN>), grid, block, 0, s, X4, W4, part, M, N, KT, ksp, stride)
  if (MT <= 1) PMX_GEMM_CASE(1);
  else if (MT <= 2) PMX_GEMM_CASE(2);
  else if (MT <= 4) PMX_GEMM_CASE(4);
  else PMX_GEMM_CASE(8);
#undef PMX_GEMM_CASE
}

// 0 = not asked yet, 1 = granted, 2 = refused: more than 64 KiB of dynamic LDS must be allowed once per device
// and kernel
template <int R, int RH, bool WNT>
static bool ring_allowed(int lds) {
  static std::atomic<int> state[64];
  int dev = 0;
  (void)hipGetDevice(&dev);
  dev = std::min(std::max(dev, 0), 63);
  int st = state[dev].load(std::memory_order_acquire);
  if (st == 0) {
    st = hipFuncSetAttribute((const void*)k_gemm_l5<R, RH, WNT>, hipFuncAttributeMaxDynamicSharedMemorySize, lds) ==
                 hipSuccess ? 1 : 2;
    if (st == 2) (void)hipGetLastError();
    state[dev].store(st, std::memory_order_release);
  }
  return st == 1;
}

// The X operand must be readable up to the next multiple of 256 rows (128 when M <= 128); rows >= M are not stored.
static void gemm_large(hipStream_t s, const uint16_t* Xt, const uint16_t* Wt, float* part, int M, int K, int N,
                       int n_split, uint16_t* act_t) {
  const int KT = K / 16;
  int ksp = 0;
  const int S = large_gemm_splits(KT, n_split, &ksp);
  const int MTall = (M + 31) / 32;
  const int64_t stride = (int64_t)MTall * 32 * N;
  if (S > 1) act_t = nullptr;       // the fused SwiGLU epilogue needs the whole K range in one work-group
  // the ring kernel's slots hold two k-steps; odd k ranges (or the tuning switch) take the 4-wave tile
  static const bool four_waves = getenv("PIPEMAX_GEMM_L1") != nullptr;
  const bool even = KT % 2 == 0 && (S == 1 || ksp % 2 == 0);
  constexpr int R2 = 4, kLds2 = R2 * 2048 * 16;       // 256-row blocks: 4 slots of 32 KiB
  constexpr int R1 = 3, kLds1 = R1 * 1536 * 16;       // 128-row block: 3 slots of 24 KiB, two work-groups per CU
  // One row block: every weight line is used once, and the large matrices are requested non-temporal (256 rows of the
  // 70B shape: gate/up 235 -> 226 us, down unchanged; QKV and O, whose 134-168 MB were 2-3 % slower that way, are
  // not; on a box whose GEMMs ran 20 % slower than usual the gain was 13 % on gate/up and 23 % on down).
  static const bool no_wnt_env = getenv("PIPEMAX_GEMM_NO_WNT") != nullptr;
  const bool no_wnt = no_wnt_env || (int64_t)K * N * 2 < ((int64_t)256 << 20);
  if (even && !four_waves && ring_allowed<R2, 2, false>(kLds2) && ring_allowed<R1, 1, false>(kLds1) &&
      ring_allowed<R2, 2, true>(kLds2) && ring_allowed<R1, 1, true>(kLds1)) {
    // blocks of 256 rows along grid.z; a last block of at most 128 rows takes the 128-row tile
    const int rem = M % 256;
    const int tall = (rem == 0 || rem > 128) ? (M + 255) / 256 : M / 256;
    const int n_x = N / 256;
    if (tall > 1 && n_x % 8 == 0) {      // XCD-aware tile order (see the kernel)
      int G = 1;
      for (int c = 8; c >= 1; --c)
        if ((n_x / 8) % c == 0) { G = c; break; }
      hipLaunchKernelGGL((k_gemm_l5<R2, 2, false>), dim3(n_x * tall, S, 1), dim3(512), kLds2, s, (const uint4*)Xt,
                         (const uint4*)Wt, part, M, N, KT, ksp, stride, act_t, tall, G);
    } else if (tall == 1 && !no_wnt)      // one row block: the weights are read once
      hipLaunchKernelGGL((k_gemm_l5<R2, 2, true>), dim3(n_x, S, 1), dim3(512), kLds2, s, (const uint4*)Xt,
                         (const uint4*)Wt, part, M, N, KT, ksp, stride, act_t, 0, 0);
    else if (tall)
      hipLaunchKernelGGL((k_gemm_l5<R2, 2, false>), dim3(n_x, S, tall), dim3(512), kLds2, s, (const uint4*)Xt,
                         (const uint4*)Wt, part, M, N, KT, ksp, stride, act_t, 0, 0);
    if (tall * 256 < M) {
      const uint4* Xr = (const uint4*)Xt + (int64_t)tall * 8 * KT * 64;
      float* pr = part + (int64_t)tall * 256 * N;
      // the A-tiled output of these rows starts at row tile tall * 8 of the next GEMM's operand
      uint16_t* ar = act_t ? act_t + (int64_t)tall * 8 * (N >> 5) * 512 : nullptr;
      if (tall == 0 && !no_wnt)
        hipLaunchKernelGGL((k_gemm_l5<R1, 1, true>), dim3(N / 256, S, 1), dim3(256), kLds1, s, Xr, (const uint4*)Wt, pr,
                           M - tall * 256, N, KT, ksp, stride, ar, 0, 0);
      else
        hipLaunchKernelGGL((k_gemm_l5<R1, 1, false>), dim3(N / 256, S, 1), dim3(256), kLds1, s, Xr, (const uint4*)Wt, pr,
                           M - tall * 256, N, KT, ksp, stride, ar, 0, 0);
    }
    return;
  }
  const int full = M / 256, rem = M - full * 256;
  dim3 block(256);
  if (full)      // whole blocks of 256 rows: one launch, row blocks along grid.z
    hipLaunchKernelGGL((k_gemm_l<8, 4>), dim3(N / 256, S, full), block, 0, s, (const uint4*)Xt, (const uint4*)Wt,
                       part, full * 256, N, KT, ksp, stride, act_t);
  if (rem) {     // the remaining rows with the smallest tile count that covers them
    const uint4* Xr = (const uint4*)Xt + (int64_t)full * 8 * KT * 64;
    float* pr = part + (int64_t)full * 256 * N;
    uint16_t* ar = act_t ? act_t + (int64_t)full * 8 * (N >> 5) * 512 : nullptr;
    dim3 grid(N / 256, S);
    if (rem <= 128)
      hipLaunchKernelGGL((k_gemm_l<4, 4>), grid, block, 0, s, Xr, (const uint4*)Wt, pr, rem, N, KT, ksp, stride, ar);
    else
      hipLaunchKernelGGL((k_gemm_l<8, 4>), grid, block, 0, s, Xr, (const uint4*)Wt, pr, rem, N, KT, ksp, stride, ar);
  }
}

void gemm(hipStream_t s, const uint16_t* Xt, const uint16_t* Wt, float* part, int M, int K, int N,
          int n_split, int wn, uint16_t* swiglu_act_t) {
  if (wn == 0) { gemm_large(s, Xt, Wt, part, M, K, N, n_split, swiglu_act_t); return; }
  if (wn == 8) gemm_wn<8>(s, Xt, Wt, part, M, K, N, n_split);
  else gemm_wn<4>(s, Xt, Wt, part, M, K, N, n_split);
}

void rope_append(hipStream_t s, const Dims& D, int layer, int b, const float* part, int n_split,
                 int64_t split_stride, const float2* cs, const int* ctx, const int* table,
                 uint16_t* pool, uint16_t* staging, uint16_t* q_out) {
  hipLaunchKernelGGL(k_rope_append, dim3(b, D.Hq + 2 * D.Hkv), dim3(64), 0, s, D, layer, part, n_split,
                     split_stride, cs, ctx, table, pool, staging, q_out);
}

void attention_prefill(hipStream_t s, const Dims& D, int layer, int rows, int pos0, const uint16_t* q,
                       const uint16_t* pool, const int* table, uint16_t* out_t) {
  constexpr int NW = kAttnWaves;
  hipLaunchKernelGGL((k_attn_prefill<NW>), dim3((rows + 15) / 16, D.Hq), dim3(NW * 64), 0, s, D, layer, q, pool,
                     table, pos0, rows, out_t);
}

void attention(hipStream_t s, const Dims& D, int layer, int b, const uint16_t* q, const uint16_t* pool,
               const int* table, const int* ctx, float* part_o, float* part_ml, int chunk_pages,
               int max_chunks, int* counters, uint16_t* out_t, const int* order, hipEvent_t ev_start,
               hipEvent_t ev_stop, bool per_wave) {
  constexpr int NW = kAttnWaves;
  const size_t lds = (size_t)NW * D.G * kORow * sizeof(float);
  const int n_items = max_chunks * D.Hkv * b;
  if (chunk_pages > 64 * NW) per_wave = true;      // beyond the reach of a work-group's page ids: the wave kernel takes any length
  if (per_wave) {
    const unsigned grid = (unsigned)((n_items + NW - 1) / NW);
    if (ev_start && ev_stop)
      hipExtLaunchKernelGGL((k_attn_w<NW>), dim3(grid), dim3(NW * 64), 0u, s, ev_start, ev_stop, 0u, D, layer, q, pool,
                            table, ctx, part_o, part_ml, chunk_pages, max_chunks, counters, out_t, order, n_items);
    else
      hipLaunchKernelGGL((k_attn_w<NW>), dim3(grid), dim3(NW * 64), 0, s, D, layer, q, pool, table, ctx, part_o,
                         part_ml, chunk_pages, max_chunks, counters, out_t, order, n_items);
    return;
  }
  if (ev_start && ev_stop)      // the events take the start and stop times of this dispatch itself
    hipExtLaunchKernelGGL((k_attn<NW>), dim3(max_chunks, D.Hkv, b), dim3(NW * 64), (uint32_t)lds, s, ev_start, ev_stop,
                          0u, D, layer, q, pool, table, ctx, part_o, part_ml, chunk_pages, max_chunks, counters, out_t,
                          order);
  else
    hipLaunchKernelGGL((k_attn<NW>), dim3(max_chunks, D.Hkv, b), dim3(NW * 64), lds, s, D, layer, q, pool, table,
                       ctx, part_o, part_ml, chunk_pages, max_chunks, counters, out_t, order);
}

void first(hipStream_t s, int b, int h, const uint16_t* hin, float* x, const uint16_t* gain, uint16_t* xg_t,
           float* ssq_out, int nb, const int* ctx, float2* cs, float rope_base) {
  hipLaunchKernelGGL(k_first, dim3(b), dim3(256), 0, s, h, hin, x, gain, xg_t, ssq_out, nb, ctx, cs,
                     (double)rope_base);
}

int compute_units() {      // of the current device (cached per device)
  static std::atomic<int> cus[64];
  int dev = 0;
  (void)hipGetDevice(&dev);
  dev = std::min(std::max(dev, 0), 63);
  int n = cus[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
      (void)hipGetLastError();
      n = 256;
    }
    cus[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

template <int NWK, int EPI>
static void gemm_fused_t(hipStream_t s, const uint16_t* Xt, const uint16_t* Wt, float* part, const FusedArgs& A,
                         int M, int K, int N, int n_split) {
  const int KT = K / 16;
  const int ksp = (KT + n_split - 1) / n_split;
  const int S = (KT + ksp - 1) / ksp;
  const int MT = (M + 31) / 32;
  const int64_t stride = (int64_t)MT * 32 * N;
  dim3 grid(N / 64, S), block(NWK * 64);
  if (MT <= 1)
    hipLaunchKernelGGL((k_gemm_f<1, NWK, 4, EPI, 1>), grid, block, 0, s, (const uint4*)Xt, (const uint4*)Wt, part, A, M,
                       N, KT, ksp, stride);
  else if (MT <= 2) {   // two k-steps in flight measured 1-4 % faster than four, six or eight (fewer registers)
    // Both row tiles in one reduction pass keep all eight waves busy in it (-0.5 .. -1.3 us per launch), but 128 KiB
    // of LDS leave room for one work-group per compute unit: only where the grid does not ask for a second one.
    if (NWK == 4 || (int)(grid.x * grid.y) <= compute_units())
      hipLaunchKernelGGL((k_gemm_f<2, NWK, 2, EPI, 2>), grid, block, 0, s, (const uint4*)Xt, (const uint4*)Wt, part, A,
                         M, N, KT, ksp, stride);
    else
      hipLaunchKernelGGL((k_gemm_f<2, NWK, 2, EPI, 1>), grid, block, 0, s, (const uint4*)Xt, (const uint4*)Wt, part, A,
                         M, N, KT, ksp, stride);
  } else     // up to 128 rows: 8 accumulator tiles per wave, two k-steps in flight as well
    hipLaunchKernelGGL((k_gemm_f<4, NWK, 2, EPI, 2>), grid, block, 0, s, (const uint4*)Xt, (const uint4*)Wt, part, A, M,
                       N, KT, ksp, stride);
}

static void gemm_fused(hipStream_t s, int epi, const uint16_t* Xt, const uint16_t* Wt, float* part,
                       const FusedArgs& A, int M, int K, int N, int n_split, int nwk) {
  if (epi == EPI_SWIGLU) {
    if (nwk == 8) gemm_fused_t<8, EPI_SWIGLU>(s, Xt, Wt, part, A, M, K, N, 1);
    else gemm_fused_t<4, EPI_SWIGLU>(s, Xt, Wt, part, A, M, K, N, 1);
  } else if (epi == EPI_RESID) {
    if (nwk == 8) gemm_fused_t<8, EPI_RESID>(s, Xt, Wt, part, A, M, K, N, n_split);
    else gemm_fused_t<4, EPI_RESID>(s, Xt, Wt, part, A, M, K, N, n_split);
  } else {
    if (nwk == 8) gemm_fused_t<8, EPI_QKV>(s, Xt, Wt, part, A, M, K, N, n_split);
    else gemm_fused_t<4, EPI_QKV>(s, Xt, Wt, part, A, M, K, N, n_split);
  }
}

void gemm_qkv_rope_append(hipStream_t s, const Dims& D, int layer, int b, const uint16_t* xg_t, const uint16_t* Wt,
                          float* part, int* counters, const float* ssq_in, int n_ssq_in, const float2* cs,
                          const int* ctx, const int* table, uint16_t* pool, uint16_t* staging, uint16_t* q_out,
                          int n_split, int nwk) {
  FusedArgs A{};
  A.counters = counters; A.ssq_in = ssq_in; A.n_ssq_in = n_ssq_in; A.inv_h = 1.0f / (float)D.h; A.eps = D.eps;
  A.layer = layer; A.cs = cs; A.ctx = ctx; A.table = table; A.pool = pool; A.staging = staging; A.q_out = q_out;
  A.Hq = D.Hq; A.Hkv = D.Hkv; A.max_pages = D.max_pages; A.page_stride = D.page_stride;
  A.layer_off = (int64_t)layer * D.layer_stride;
  gemm_fused(s, EPI_QKV, xg_t, Wt, part, A, b, D.h, D.Nqkv, n_split, nwk);
}

void gemm_resid(hipStream_t s, int b, int K, int N, const uint16_t* Xt, const uint16_t* Wt, float* part,
                int* counters, float* x, const uint16_t* gain_next, uint16_t* xg_t, float* ssq_out,
                uint16_t* hout, int* ctx_advance, int n_split, int nwk) {
  FusedArgs A{};
  A.counters = counters; A.x = x; A.gain_next = gain_next; A.xg_t = xg_t; A.ssq_out = ssq_out; A.hout = hout;
  A.ctx_advance = ctx_advance;
  gemm_fused(s, EPI_RESID, Xt, Wt, part, A, b, K, N, n_split, nwk);
}

void gemm_swiglu(hipStream_t s, int b, int K, int F, float eps, const uint16_t* xg_t, const uint16_t* Wt,
                 const float* ssq_in, int n_ssq_in, uint16_t* act_t, int nwk) {
  FusedArgs A{};
  A.ssq_in = ssq_in; A.n_ssq_in = n_ssq_in; A.inv_h = 1.0f / (float)K; A.eps = eps; A.act_t = act_t;
  gemm_fused(s, EPI_SWIGLU, xg_t, Wt, nullptr, A, b, K, 2 * F, 1, nwk);
}

void swiglu(hipStream_t s, int b, int F, const float* part, int n_split, int64_t split_stride,
            uint16_t* act_t) {
  hipLaunchKernelGGL(k_swiglu, dim3(cdiv((int64_t)b * (F / 8), 256)), dim3(256), 0, s, b, F, part,
                     n_split, split_stride, act_t);
}

}  // namespace mfma
}  // namespace pmx

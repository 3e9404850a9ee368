// Shape-generic kernels of the stage decode step (any hidden / head_dim % 32 == 0 / ffn; element
// type float or bf16).  They serve the fp32 configuration and shapes the matrix-core kernels do
// not cover; activations are kept in fp32, only stored K,V and weights are in the element type.
#include <algorithm>

#include "kernels.hpp"

namespace pmx {

namespace {

__device__ inline float ldf(const float* p) { return *p; }
__device__ inline float ldf(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }
__device__ inline void stf(float* p, float v) { *p = v; }
__device__ inline void stf(uint16_t* p, float v) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7fffffffu) > 0x7f800000u) { *p = 0x7fc0; return; }
  u += 0x7fffu + ((u >> 16) & 1u);
  *p = (uint16_t)(u >> 16);
}

__device__ inline float block_sum(float v, float* sh) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += sh[i];
  return t;
}
__device__ inline float block_max(float v, float* sh) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  float t = -INFINITY;
  for (int i = 0; i < nw; ++i) t = fmaxf(t, sh[i]);
  return t;
}

// ---- shared small kernels ---------------------------------------------------------------------
__global__ void k_rope_table(const int* ctx, float2* cs, int b, int half, int d, double base) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= b * half) return;
  int i = idx / half, j = idx - i * half;
  double theta = pow(base, -2.0 * (double)j / (double)d);
  double ang = (double)ctx[i] * theta;
  cs[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

__global__ void k_advance_ctx(int* ctx, int b) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < b) ctx[i] += 1;
}

__global__ __launch_bounds__(256) void k_probe_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// ---- generic engine ------------------------------------------------------------------------------
template <typename T>
__global__ void k_load_hidden(const T* in, float* x, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) x[i] = ldf(in + i);
}
template <typename T>
__global__ void k_store_hidden(const float* x, T* out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) stf(out + i, x[i]);
}

template <typename T>
__global__ void k_rmsnorm(const float* x, const T* gain, float* xn, int h, float eps) {
  __shared__ float sh[16];
  const float* row = x + (int64_t)blockIdx.x * h;
  float ss = 0.f;
  for (int j = threadIdx.x; j < h; j += blockDim.x) ss += row[j] * row[j];
  ss = block_sum(ss, sh);
  float r = 1.0f / sqrtf(ss / (float)h + eps);
  for (int j = threadIdx.x; j < h; j += blockDim.x)
    xn[(int64_t)blockIdx.x * h + j] = row[j] * r * ldf(gain + j);
}

// one thread per output element; a block covers 256 columns of one row
template <typename T>
__global__ void k_gemm(const float* A, const T* W, float* C, int M, int K, int N, int accumulate) {
  int n = blockIdx.x * blockDim.x + threadIdx.x;
  int m = blockIdx.y;
  if (n >= N || m >= M) return;
  const float* a = A + (int64_t)m * K;
  float acc = 0.f;
  for (int k = 0; k < K; ++k) acc = fmaf(a[k], ldf(W + (int64_t)k * N + n), acc);
  float* c = C + (int64_t)m * N + n;
  *c = accumulate ? (*c + acc) : acc;
}

// grid (b, Hq + 2 Hkv), block d/2 threads: one rotation pair (or two v elements) per thread
template <typename T>
__global__ void k_rope_append(Dims D, int layer, const float* qkv, const float2* cs, const int* ctx,
                              const int* table, T* pool, T* staging, float* q_out) {
  int i = blockIdx.x, hd = blockIdx.y, j = threadIdx.x, half = D.d / 2;
  const float* row = qkv + (int64_t)i * D.Nqkv + (int64_t)hd * D.d;
  float lo = row[j], hi = row[j + half];
  int pos = ctx[i];
  if (hd < D.Hq) {
    float2 c = cs[i * half + j];
    float* q = q_out + ((int64_t)i * D.Hq + hd) * D.d;
    q[j] = lo * c.x - hi * c.y;
    q[j + half] = hi * c.x + lo * c.y;
    return;
  }
  int kv = (hd < D.Hq + D.Hkv) ? 0 : 1;
  int head = hd - D.Hq - kv * D.Hkv;
  if (kv == 0) {
    float2 c = cs[i * half + j];
    float a = lo * c.x - hi * c.y, b2 = hi * c.x + lo * c.y;
    lo = a;
    hi = b2;
  }
  int phys = table[(int64_t)i * D.max_pages + pos / kPageTokens];
  int slot = pos % kPageTokens;
  T* sub = pool + (int64_t)phys * D.page_stride + (int64_t)layer * D.layer_stride + sub_block_off(D.Hkv, D.d, 0, head, kv);
  if (kv == 0) {
    stf(sub + k_sub_idx(slot, j), lo);
    stf(sub + k_sub_idx(slot, j + half), hi);
  } else {
    stf(sub + v_sub_idx(slot, j), lo);
    stf(sub + v_sub_idx(slot, j + half), hi);
  }
  T* st = staging + (((int64_t)i * 2 + kv) * D.Hkv + head) * D.d;   // [b][2][Hkv][d]
  stf(st + j, lo);
  stf(st + j + half, hi);
}

// grid (b, Hq), block 128: scores -> softmax -> weighted sum, all in fp32
template <typename T>
__global__ void k_attention(Dims D, int layer, const float* q, const T* pool, const int* table,
                            const int* ctx, float* scores, float* out) {
  extern __shared__ float qs[];            // d floats
  __shared__ float sh[16];
  int i = blockIdx.x, u = blockIdx.y, c = u / D.G;
  int n_tok = ctx[i] + 1;
  const float* qr = q + ((int64_t)i * D.Hq + u) * D.d;
  for (int e = threadIdx.x; e < D.d; e += blockDim.x) qs[e] = qr[e];
  __syncthreads();
  float* sc = scores + ((int64_t)i * D.Hq + u) * D.max_ctx_pad;
  const int* trow = table + (int64_t)i * D.max_pages;
  float scale = 1.0f / sqrtf((float)D.d);
  float mx = -INFINITY;
  for (int t = threadIdx.x; t < n_tok; t += blockDim.x) {
    const T* sub = pool + (int64_t)trow[t / kPageTokens] * D.page_stride + (int64_t)layer * D.layer_stride +
                   sub_block_off(D.Hkv, D.d, 0, c, 0);
    int slot = t % kPageTokens;
    float s = 0.f;
    for (int e = 0; e < D.d; ++e) s = fmaf(qs[e], ldf(sub + k_sub_idx(slot, e)), s);
    s *= scale;
    sc[t] = s;
    mx = fmaxf(mx, s);
  }
  mx = block_max(mx, sh);
  float sum = 0.f;
  for (int t = threadIdx.x; t < n_tok; t += blockDim.x) {
    float p = expf(sc[t] - mx);
    sc[t] = p;
    sum += p;
  }
  sum = block_sum(sum, sh);     // also orders the sc[] writes before the reads below
  float inv = 1.0f / sum;
  for (int e = threadIdx.x; e < D.d; e += blockDim.x) {
    float o = 0.f;
    for (int t = 0; t < n_tok; ++t) {
      const T* sub = pool + (int64_t)trow[t / kPageTokens] * D.page_stride + (int64_t)layer * D.layer_stride +
                     sub_block_off(D.Hkv, D.d, 0, c, 1);
      o = fmaf(sc[t], ldf(sub + v_sub_idx(t % kPageTokens, e)), o);
    }
    out[((int64_t)i * D.Hq + u) * D.d + e] = o * inv;
  }
}

__global__ void k_swiglu_generic(const float* gu, float* act, int b, int F) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)b * F) return;
  int i = idx / F, f = idx - (int64_t)i * F;
  float g = gu[(int64_t)i * 2 * F + f], u = gu[(int64_t)i * 2 * F + F + f];
  act[idx] = g / (1.0f + expf(-g)) * u;
}

inline unsigned cdiv(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

}  // namespace

void launch_rope_table(hipStream_t s, const int* ctx, float2* cs, int b, int d, float base) {
  int n = b * (d / 2);
  hipLaunchKernelGGL(k_rope_table, dim3(cdiv(n, 256)), dim3(256), 0, s, ctx, cs, b, d / 2, d,
                     (double)base);
}
void launch_probe_copy(hipStream_t s, void* dst, const void* src, size_t bytes) {
  const size_t n = bytes / 16;
  const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 256 * 32);
  if (n == 0) return;
  hipLaunchKernelGGL(k_probe_copy, dim3(blocks), dim3(256), 0, s, (uint4*)dst, (const uint4*)src, n);
}
void launch_advance_ctx(hipStream_t s, int* ctx, int b) {
  hipLaunchKernelGGL(k_advance_ctx, dim3(cdiv(b, 256)), dim3(256), 0, s, ctx, b);
}
void launch_swiglu_generic(hipStream_t s, const float* gu, float* act, int b, int F) {
  hipLaunchKernelGGL(k_swiglu_generic, dim3(cdiv((int64_t)b * F, 256)), dim3(256), 0, s, gu, act, b, F);
}

template <typename T>
void Generic<T>::load_hidden(hipStream_t s, const T* in, float* x, int64_t n) {
  hipLaunchKernelGGL(k_load_hidden<T>, dim3(cdiv(n, 256)), dim3(256), 0, s, in, x, n);
}
template <typename T>
void Generic<T>::store_hidden(hipStream_t s, const float* x, T* out, int64_t n) {
  hipLaunchKernelGGL(k_store_hidden<T>, dim3(cdiv(n, 256)), dim3(256), 0, s, x, out, n);
}
template <typename T>
void Generic<T>::rmsnorm(hipStream_t s, const float* x, const T* gain, float* xn, int b, int h,
                         float eps) {
  hipLaunchKernelGGL(k_rmsnorm<T>, dim3(b), dim3(256), 0, s, x, gain, xn, h, eps);
}
template <typename T>
void Generic<T>::gemm(hipStream_t s, const float* A, const T* W, float* C, int M, int K, int N,
                      int accumulate) {
  hipLaunchKernelGGL(k_gemm<T>, dim3(cdiv(N, 256), M), dim3(256), 0, s, A, W, C, M, K, N, accumulate);
}
template <typename T>
void Generic<T>::rope_append(hipStream_t s, const Dims& D, int layer, int b, const float* qkv,
                             const float2* cs, const int* ctx, const int* table, T* pool, T* staging,
                             float* q_out) {
  hipLaunchKernelGGL(k_rope_append<T>, dim3(b, D.Hq + 2 * D.Hkv), dim3(D.d / 2), 0, s, D, layer, qkv,
                     cs, ctx, table, pool, staging, q_out);
}
template <typename T>
void Generic<T>::attention(hipStream_t s, const Dims& D, int layer, int b, const float* q,
                           const T* pool, const int* table, const int* ctx, float* scores, float* out) {
  hipLaunchKernelGGL(k_attention<T>, dim3(b, D.Hq), dim3(128), D.d * sizeof(float), s, D, layer, q,
                     pool, table, ctx, scores, out);
}

template struct Generic<float>;
template struct Generic<uint16_t>;

}  // namespace pmx

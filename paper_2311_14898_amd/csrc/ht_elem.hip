// Small HBM-bound kernels: ReLU derivative mask (Sec. 2.3), softmax
// cross-entropy and its gradient (the downstream task of Alg. 1),
// SGD step (Alg. 1), zero fill.
#include <algorithm>

#include "ht_internal.h"

namespace {

__global__ void k_relu_mask(const float* __restrict__ dh, int64_t ld_dh, const float* __restrict__ ref,
                            int64_t ld_ref, float* __restrict__ dz, int64_t ld_dz, int64_t rows, int cols4) {
  // one thread per float4 of the padded row
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int vec_per_row = cols4 >> 2;
  if (i >= rows * vec_per_row) return;
  const int64_t r = i / vec_per_row;
  const int c = (int)(i % vec_per_row) * 4;
  const float4 g = *reinterpret_cast<const float4*>(dh + r * ld_dh + c);
  const float4 z = *reinterpret_cast<const float4*>(ref + r * ld_ref + c);
  float4 o;
  o.x = z.x > 0.f ? g.x : 0.f;
  o.y = z.y > 0.f ? g.y : 0.f;
  o.z = z.z > 0.f ? g.z : 0.f;
  o.w = z.w > 0.f ? g.w : 0.f;
  *reinterpret_cast<float4*>(dz + r * ld_dz + c) = o;
}

__global__ void k_count_labelled(const int32_t* __restrict__ labels, int64_t V, unsigned long long* __restrict__ T) {
  const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  unsigned long long c = (v < V && labels[v] >= 0) ? 1ull : 0ull;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_down(c, o, 64);
  if ((threadIdx.x & 63) == 0 && c) atomicAdd(T, c);
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// One wave per vertex, classes across lanes.  loss_v[v] = lse - x[y] (0 if unlabelled).
__global__ void __launch_bounds__(256) k_softmax_ce(const float* __restrict__ logits, int64_t ld,
                                                    const int32_t* __restrict__ labels, int64_t V, int C,
                                                    const unsigned long long* __restrict__ Tp,
                                                    float* __restrict__ grad, int64_t ld_g,
                                                    float* __restrict__ loss_v) {
  const int lane = threadIdx.x & 63;
  // (a bounded grid that strides: a launch holds fewer than 2^32 threads, 64 V can be more)
  for (int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); v < V; v += (int64_t)gridDim.x * 4) {
    const int32_t y = labels[v];
    const float* x = logits + v * ld;
    float* g = grad + v * ld_g;
    if (y < 0) {
      for (int c = lane; c < C; c += 64) g[c] = 0.f;
      if (lane == 0) loss_v[v] = 0.f;
      continue;
    }
    const float invT = 1.f / (float)(*Tp);
    float m = -INFINITY;
    for (int c = lane; c < C; c += 64) m = fmaxf(m, x[c]);
    m = wave_max(m);
    float z = 0.f;
    for (int c = lane; c < C; c += 64) z += expf(x[c] - m);
    z = wave_sum(z);
    const float lse = m + logf(z);
    for (int c = lane; c < C; c += 64) g[c] = (expf(x[c] - lse) - (c == y ? 1.f : 0.f)) * invT;
    if (lane == 0) loss_v[v] = lse - x[y];
  }
}

// Fixed-order sum of n floats in fp64: 256-thread blocks of 4096 elements, then one block.
__global__ void __launch_bounds__(256) k_sum_stage(const float* __restrict__ in_f, const double* __restrict__ in_d,
                                                   int64_t n, double* __restrict__ out) {
  __shared__ double sh[256];
  const int64_t base = (int64_t)blockIdx.x * 4096;
  double s = 0.0;
  for (int i = 0; i < 16; ++i) {
    const int64_t idx = base + (int64_t)i * 256 + threadIdx.x;
    if (idx < n) s += in_f ? (double)in_f[idx] : in_d[idx];
  }
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = sh[0];
}

__global__ void k_finish_loss(const double* __restrict__ sum, const unsigned long long* __restrict__ Tp,
                              float* __restrict__ loss) {
  const unsigned long long T = *Tp;
  *loss = T > 0 ? (float)(*sum / (double)T) : 0.f;
}

__global__ void k_sgd(float* __restrict__ W, const float* __restrict__ dW, int64_t n, float lr) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) W[i] = W[i] - lr * dW[i];
}

// n16 16-byte words from p16 (16-byte aligned), then the words of the ragged ends; a bounded grid
// that strides, so the launch also fits a HIP graph node at any size
__global__ void k_zero(uint4* __restrict__ p16, int64_t n16, uint32_t* __restrict__ head, int n_head,
                       uint32_t* __restrict__ tail, int n_tail) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (int64_t i = t; i < n16; i += stride) p16[i] = make_uint4(0u, 0u, 0u, 0u);
  if (t < n_head) head[t] = 0u;
  if (t < n_tail) tail[t] = 0u;
}

}  // namespace

int ht_relu_mask(ht_ctx* ctx, hipStream_t st, const float* dh, int64_t ld_dh, const float* ref, int64_t ld_ref,
                 float* dz, int64_t ld_dz, int64_t rows, int32_t cols) {
  if (rows <= 0 || cols <= 0) return HT_OK;
  const int cols4 = (cols + 3) & ~3;
  const int64_t n = rows * (cols4 >> 2);
  // one thread per 16-byte vector: a launch of 2^32 threads or more would silently run only a part
  if (n >= ((int64_t)1 << 32) - 256) return ht_set_err(ctx, HT_ESHAPE, "ReLU mask: %lld rows x %d columns in one chunk is too large", (long long)rows, cols);
  k_relu_mask<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(dh, ld_dh, ref, ld_ref, dz, ld_dz, rows, cols4);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

// scratch slot 2: per-vertex losses, stage sums, labelled count
int ht_softmax_ce(ht_ctx* ctx, hipStream_t st, const float* logits, int64_t ld, const int32_t* labels, int64_t V,
                  int32_t C, float* grad, int64_t ld_g, float* loss_dev) {
  if (V <= 0 || C <= 0) return ht_set_err(ctx, HT_EINVAL, "loss: empty input");
  const int64_t nb1 = (V + 4095) / 4096;
  const int64_t nb2 = (nb1 + 4095) / 4096;
  const size_t bytes = 16 + (size_t)V * 4 + 16 + (size_t)(nb1 + nb2 + 2) * 8;
  char* p = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_LOSS, bytes, (void**)&p));
  unsigned long long* T = (unsigned long long*)p;
  double* st1 = (double*)(p + 16);
  double* st2 = st1 + nb1;
  double* st3 = st2 + nb2;
  float* loss_v = (float*)(st3 + 2);
  HT_TRY(ht_fill_zero(ctx, st, T, 16));
  k_count_labelled<<<(unsigned)((V + 255) / 256), 256, 0, st>>>(labels, V, T);
  HT_LAUNCH_CHECK(ctx);
  k_softmax_ce<<<(unsigned)std::min<int64_t>((V + 3) / 4, 1 << 22), 256, 0, st>>>(logits, ld, labels, V, C, T, grad, ld_g, loss_v);
  HT_LAUNCH_CHECK(ctx);
  k_sum_stage<<<(unsigned)nb1, 256, 0, st>>>(loss_v, nullptr, V, st1);
  HT_LAUNCH_CHECK(ctx);
  const double* fin = st1;
  if (nb1 > 1) {
    k_sum_stage<<<(unsigned)nb2, 256, 0, st>>>(nullptr, st1, nb1, st2);
    HT_LAUNCH_CHECK(ctx);
    fin = st2;
    if (nb2 > 1) {
      if (nb2 > 4096) return ht_set_err(ctx, HT_ESHAPE, "loss: too many vertices for the 3-stage sum");
      k_sum_stage<<<1, 256, 0, st>>>(nullptr, st2, nb2, st3);
      HT_LAUNCH_CHECK(ctx);
      fin = st3;
    }
  }
  k_finish_loss<<<1, 1, 0, st>>>(fin, T, loss_dev);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

int ht_sgd(ht_ctx* ctx, hipStream_t st, float* W, const float* dW, int64_t n, float lr) {
  if (n <= 0) return HT_OK;
  k_sgd<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(W, dW, n, lr);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

int ht_fill_zero(ht_ctx* ctx, hipStream_t st, void* p, size_t bytes) {
  if (bytes == 0) return HT_OK;
  if (bytes & 3) return ht_set_err(ctx, HT_EINVAL, "fill: size must be a multiple of 4");
  if ((uintptr_t)p & 3) return ht_set_err(ctx, HT_EINVAL, "fill: pointer must be 4-byte aligned");
  const int64_t n = (int64_t)(bytes >> 2);
  uint32_t* w = (uint32_t*)p;
  int n_head = (int)((16 - ((uintptr_t)p & 15)) & 15) >> 2;   // words before the first 16-byte boundary
  if (n_head > n) n_head = (int)n;
  const int64_t n16 = (n - n_head) >> 2;
  const int n_tail = (int)(n - n_head - 4 * n16);
  int64_t blocks = (n16 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks < 1) blocks = 1;
  k_zero<<<(unsigned)blocks, 256, 0, st>>>((uint4*)(w + n_head), n16, w, n_head, w + n_head + 4 * n16, n_tail);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

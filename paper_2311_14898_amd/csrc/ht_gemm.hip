// Dense transform of the update stage (Eq. 2: linear + ReLU) and its gradient
// GEMMs (Sec. 2.3: grad W = a^T (ReLU'(aW) * grad h'), grad a = grad z W^T) on
// the fp32 matrix cores (v_mfma_f32_32x32x2_f32), LDS-tiled for 64-wide waves.
//
//   NN: C[M x N] = A[M x K] Bp        M = chunk rows (tall), K, N = layer widths
//   TN: C[K x N] = A[M x K]^T B[M x N] reduction over the tall M, cut into
//       slices whose partial tiles are added in slice order (no atomics).
// The small operand W is first packed into a zero-padded tile-aligned copy.
#include "ht_internal.h"

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BK = 16;        // reduction depth of one LDS stage
constexpr int BM = 128;       // rows of A per block (NN) / output rows per block (TN)
constexpr int LDA_S = BK + 1; // LDS pitch of the row-major A tile (NN): odd, conflict-free column reads

__device__ __forceinline__ float4 ld4g(const float* p) { return *reinterpret_cast<const float4*>(p); }

// Pack W[K x N] (row-major, dense) into Bp[Kp x Np] zero-padded; transpose = 1 packs W^T.
__global__ void k_pack_b(const float* __restrict__ W, int K, int N, int transpose, float* __restrict__ Bp, int Kp,
                         int Np) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)Kp * Np) return;
  const int r = (int)(i / Np), c = (int)(i % Np);
  float v = 0.f;
  if (!transpose) {
    if (r < K && c < N) v = W[(int64_t)r * N + c];
  } else {  // Bp[r][c] = W[c][r], W is [N' x K'] = [c-range x r-range]
    if (r < N && c < K) v = W[(int64_t)c * N + r];
  }
  Bp[i] = v;
}

// C = A Bp (+ReLU).  A [M x K] pitch lda (columns >= K are never used as data),
// Bp [Kp x Np] padded.  Block: 256 threads = WM x WN waves, wave tile (TI*32) x (TJ*32).
template <int BN, int WM, int WN, int TI, int TJ>
__global__ void __launch_bounds__(256) k_gemm_nn(const float* __restrict__ A, int64_t lda,
                                                 const float* __restrict__ Bp, int Np, float* __restrict__ C,
                                                 int64_t ldc, int64_t M, int K, int N, int relu) {
  static_assert(WM * WN == 4 && WM * TI * 32 == BM && WN * TJ * 32 == BN, "tile shape");
  __shared__ float As[BM * LDA_S];
  __shared__ float Bs[BK * (BN + 4)];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, half = lane >> 5;
  const int64_t m0 = (int64_t)blockIdx.x * BM;
  const int n0 = blockIdx.y * BN;

  v16f acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // The tiles of step k0 + BK are fetched into registers while the matrix cores work on step k0.
  constexpr int NA = BM * 4 / 256, NB = BK * BN / 4 / 256;
  static_assert(NA * 256 == BM * 4 && NB * 256 == BK * BN / 4, "tile loads must divide among 256 threads");
  float4 ra[NA], rb[NB];
  // interior blocks (all BM rows exist) take their full K-steps without any bounds test
  const bool interior = m0 + BM <= M;
  auto fetch = [&](int k0) {
    if (interior && k0 + BK <= K) {
#pragma unroll
      for (int u = 0; u < NA; ++u) {
        const int f = tid + u * 256;
        const int row = f >> 2, kv = (f & 3) * 4;
        ra[u] = ld4g(A + (m0 + row) * lda + k0 + kv);
      }
    } else {
#pragma unroll
      for (int u = 0; u < NA; ++u) {
        const int f = tid + u * 256;
        const int row = f >> 2, kv = (f & 3) * 4;
        const int64_t gm = m0 + row;
        const int gk = k0 + kv;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gm < M && gk < K) {
          v = ld4g(A + gm * lda + gk);
          if (gk + 1 >= K) v.y = 0.f;
          if (gk + 2 >= K) v.z = 0.f;
          if (gk + 3 >= K) v.w = 0.f;
        }
        ra[u] = v;
      }
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int f = tid + u * 256;
      const int kr = f / (BN / 4), nv = (f % (BN / 4)) * 4;
      rb[u] = ld4g(Bp + (int64_t)(k0 + kr) * Np + n0 + nv);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int u = 0; u < NA; ++u) {
      const int f = tid + u * 256;
      const int row = f >> 2, kv = (f & 3) * 4;
      float* d = As + row * LDA_S + kv;
      d[0] = ra[u].x; d[1] = ra[u].y; d[2] = ra[u].z; d[3] = ra[u].w;
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int f = tid + u * 256;
      const int kr = f / (BN / 4), nv = (f % (BN / 4)) * 4;
      *reinterpret_cast<float4*>(Bs + kr * (BN + 4) + nv) = rb[u];
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < K; k0 += BK) {
    stash();
    __syncthreads();
    if (k0 + BK < K) fetch(k0 + BK);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float af[TI], bf[TJ];
#pragma unroll
      for (int i = 0; i < TI; ++i) af[i] = As[(wm * TI * 32 + i * 32 + l32) * LDA_S + kk + half];
#pragma unroll
      for (int j = 0; j < TJ; ++j) bf[j] = Bs[(kk + half) * (BN + 4) + wn * TJ * 32 + j * 32 + l32];
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
  // D layout of the 32x32 tile: lane holds column l32, rows (e/4)*8 + half*4 + e%4
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
      const int gc = n0 + wn * TJ * 32 + j * 32 + l32;
      if (gc >= N) continue;
      float* cp = C + (m0 + wm * TI * 32 + i * 32 + half * 4) * ldc + gc;
      if (interior && relu < 2) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float v = acc[i][j][e];
          if (relu) v = v > 0.f ? v : 0.f;
          cp[((e >> 2) * 8 + (e & 3)) * ldc] = v;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int64_t gr = m0 + wm * TI * 32 + i * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
          if (gr < M) {
            float v = acc[i][j][e];
            if (relu & 1) v = v > 0.f ? v : 0.f;
            if (relu & 2) v += C[gr * ldc + gc];
            C[gr * ldc + gc] = v;
          }
        }
      }
    }
}

// Partial tile of C[K x N] = A[M x K]^T B[M x N] over the M-slice blockIdx.z.
// P[slice][K x N] dense.  Block tile: BM output rows (k) x BN output columns.
template <int BN, int WM, int WN, int TI, int TJ>
__global__ void __launch_bounds__(256) k_gemm_tn(const float* __restrict__ A, int64_t lda,
                                                 const float* __restrict__ B, int64_t ldb, float* __restrict__ P,
                                                 int64_t M, int K, int N, int64_t slice_rows) {
  static_assert(WM * WN == 4 && WM * TI * 32 == BM && WN * TJ * 32 == BN, "tile shape");
  __shared__ float As[BK * (BM + 4)];
  __shared__ float Bs[BK * (BN + 4)];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, half = lane >> 5;
  const int kc0 = blockIdx.x * BM;  // first output row (a column of A)
  const int n0 = blockIdx.y * BN;
  const int64_t ms = (int64_t)blockIdx.z * slice_rows;
  const int64_t me = (ms + slice_rows) < M ? (ms + slice_rows) : M;

  v16f acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  constexpr int NA = BK * BM / 4 / 256, NB = BK * BN / 4 / 256;
  static_assert(NA * 256 == BK * BM / 4 && NB * 256 == BK * BN / 4, "tile loads must divide among 256 threads");
  float4 ra[NA], rb[NB];
  // tiles that lie inside both operands are fetched without bounds tests
  const bool full_a = kc0 + BM <= K, full_b = n0 + BN <= N;
  auto fetch = [&](int64_t mm0) {
    const bool full_m = mm0 + BK <= me;
    if (full_m && full_a) {
#pragma unroll
      for (int u = 0; u < NA; ++u) {
        const int f = tid + u * 256;
        const int mr = f / (BM / 4), cv = (f % (BM / 4)) * 4;
        ra[u] = ld4g(A + (mm0 + mr) * lda + kc0 + cv);
      }
    } else {
#pragma unroll
      for (int u = 0; u < NA; ++u) {
        const int f = tid + u * 256;
        const int mr = f / (BM / 4), cv = (f % (BM / 4)) * 4;
        const int64_t gm = mm0 + mr;
        const int gk = kc0 + cv;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gm < me && gk < K) {
          v = ld4g(A + gm * lda + gk);
          if (gk + 1 >= K) v.y = 0.f;
          if (gk + 2 >= K) v.z = 0.f;
          if (gk + 3 >= K) v.w = 0.f;
        }
        ra[u] = v;
      }
    }
    if (full_m && full_b) {
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int f = tid + u * 256;
        const int mr = f / (BN / 4), cv = (f % (BN / 4)) * 4;
        rb[u] = ld4g(B + (mm0 + mr) * ldb + n0 + cv);
      }
    } else {
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int f = tid + u * 256;
        const int mr = f / (BN / 4), cv = (f % (BN / 4)) * 4;
        const int64_t gm = mm0 + mr;
        const int gn = n0 + cv;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gm < me && gn < N) {
          v = ld4g(B + gm * ldb + gn);
          if (gn + 1 >= N) v.y = 0.f;
          if (gn + 2 >= N) v.z = 0.f;
          if (gn + 3 >= N) v.w = 0.f;
        }
        rb[u] = v;
      }
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int u = 0; u < NA; ++u) {
      const int f = tid + u * 256;
      const int mr = f / (BM / 4), cv = (f % (BM / 4)) * 4;
      *reinterpret_cast<float4*>(As + mr * (BM + 4) + cv) = ra[u];
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int f = tid + u * 256;
      const int mr = f / (BN / 4), cv = (f % (BN / 4)) * 4;
      *reinterpret_cast<float4*>(Bs + mr * (BN + 4) + cv) = rb[u];
    }
  };
  if (ms < me) fetch(ms);
  for (int64_t mm0 = ms; mm0 < me; mm0 += BK) {
    stash();
    __syncthreads();
    if (mm0 + BK < me) fetch(mm0 + BK);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float af[TI], bf[TJ];
#pragma unroll
      for (int i = 0; i < TI; ++i) af[i] = As[(kk + half) * (BM + 4) + wm * TI * 32 + i * 32 + l32];
#pragma unroll
      for (int j = 0; j < TJ; ++j) bf[j] = Bs[(kk + half) * (BN + 4) + wn * TJ * 32 + j * 32 + l32];
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
  float* Ps = P + (int64_t)blockIdx.z * K * N;
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
      const int gc = n0 + wn * TJ * 32 + j * 32 + l32;
      if (gc >= N) continue;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int gr = kc0 + wm * TI * 32 + i * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
        if (gr < K) Ps[(int64_t)gr * N + gc] = acc[i][j][e];
      }
    }
}

// C[i] (+)= sum over slices, slice order
__global__ void k_reduce_slices(const float* __restrict__ P, int64_t n, int slices, int accumulate,
                                float* __restrict__ C) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = accumulate ? C[i] : 0.f;
  for (int k = 0; k < slices; ++k) s += P[(int64_t)k * n + i];
  C[i] = s;
}

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

int gemm_nn_packed(ht_ctx* ctx, hipStream_t st, const float* A, int64_t lda, const float* Bp, int Np, float* C,
                   int64_t ldc, int64_t M, int K, int N, int relu) {
  if (M <= 0 || N <= 0) return HT_OK;
  const unsigned gx = (unsigned)((M + BM - 1) / BM);
  if (N > 64) {
    dim3 grid(gx, (unsigned)((N + 127) / 128));
    k_gemm_nn<128, 2, 2, 2, 2><<<grid, 256, 0, st>>>(A, lda, Bp, Np, C, ldc, M, K, N, relu);
  } else {
    dim3 grid(gx, 1);
    k_gemm_nn<64, 4, 1, 1, 2><<<grid, 256, 0, st>>>(A, lda, Bp, Np, C, ldc, M, K, N, relu);
  }
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

}  // namespace

// scratch slots: 0 = packed W, 1 = TN partial tiles
// Bp = the zero-padded, tile-aligned copy of W [K x N] that the NN kernels read ([round_up(K, 16) x round_up(N, 128)], in
// the context's scratch); *Np its row pitch.
int ht_pack_w(ht_ctx* ctx, hipStream_t st, const float* W, int32_t K, int32_t N, float** Bp, int* Np) {
  const int Kp = round_up(K, BK), Npp = round_up(N, 128);
  HT_TRY(ht_scratch(ctx, HT_S_PACKW, (size_t)Kp * Npp * 4, (void**)Bp));
  k_pack_b<<<(unsigned)(((int64_t)Kp * Npp + 255) / 256), 256, 0, st>>>(W, K, N, 0, *Bp, Kp, Npp);
  HT_LAUNCH_CHECK(ctx);
  *Np = Npp;
  return HT_OK;
}

int ht_gemm_nn(ht_ctx* ctx, hipStream_t st, const float* A, int64_t lda, const float* B, float* C, int64_t ldc,
               int64_t M, int32_t K, int32_t N, int relu) {
  if (lda & 3) return ht_set_err(ctx, HT_ESHAPE, "gemm: row pitch must be a multiple of 4");
  const int Kp = round_up(K, BK), Np = round_up(N, 128);
  float* Bp = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_PACKW, (size_t)Kp * Np * 4, (void**)&Bp));
  k_pack_b<<<(unsigned)(((int64_t)Kp * Np + 255) / 256), 256, 0, st>>>(B, K, N, 0, Bp, Kp, Np);
  HT_LAUNCH_CHECK(ctx);
  return gemm_nn_packed(ctx, st, A, lda, Bp, Np, C, ldc, M, K, N, relu);
}

int ht_gemm_nt(ht_ctx* ctx, hipStream_t st, const float* A, int64_t lda, const float* B, float* C, int64_t ldc,
               int64_t M, int32_t N, int32_t K, int accumulate) {
  // C[M x K] = A[M x N] (B[K x N])^T : reduction over N, output width K
  if (lda & 3) return ht_set_err(ctx, HT_ESHAPE, "gemm: row pitch must be a multiple of 4");
  const int Rp = round_up(N, BK), Cp = round_up(K, 128);
  float* Bp = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_PACKW, (size_t)Rp * Cp * 4, (void**)&Bp));
  // Bp[n][k] = B[k][n]
  k_pack_b<<<(unsigned)(((int64_t)Rp * Cp + 255) / 256), 256, 0, st>>>(B, K, N, 1, Bp, Rp, Cp);
  HT_LAUNCH_CHECK(ctx);
  return gemm_nn_packed(ctx, st, A, lda, Bp, Cp, C, ldc, M, N, K, accumulate ? 2 : 0);
}

int ht_gemm_tn(ht_ctx* ctx, hipStream_t st, const float* A, int64_t lda, const float* B, int64_t ldb, float* C,
               int64_t M, int32_t K, int32_t N, int accumulate) {
  if ((lda & 3) || (ldb & 3)) return ht_set_err(ctx, HT_ESHAPE, "gemm: row pitch must be a multiple of 4");
  if (K <= 0 || N <= 0) return HT_OK;
  const int64_t kn = (int64_t)K * N;
  if (M <= 0) {
    if (!accumulate) HT_TRY(ht_fill_zero(ctx, st, C, (size_t)kn * 4));
    return HT_OK;
  }
  const int bn = N > 64 ? 128 : 64;
  const int tiles = ((K + BM - 1) / BM) * ((N + bn - 1) / bn);
  int64_t slices = (1024 + tiles - 1) / tiles;
  const int64_t max_slices = (M + 255) / 256;
  if (slices > max_slices) slices = max_slices;
  if (slices < 1) slices = 1;
  int64_t slice_rows = (M + slices - 1) / slices;
  slice_rows = (slice_rows + BK - 1) / BK * BK;
  slices = (M + slice_rows - 1) / slice_rows;
  float* P = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_TNPART, (size_t)(slices * kn) * 4, (void**)&P));
  dim3 grid((unsigned)((K + BM - 1) / BM), (unsigned)((N + bn - 1) / bn), (unsigned)slices);
  if (bn == 128)
    k_gemm_tn<128, 2, 2, 2, 2><<<grid, 256, 0, st>>>(A, lda, B, ldb, P, M, K, N, slice_rows);
  else
    k_gemm_tn<64, 4, 1, 1, 2><<<grid, 256, 0, st>>>(A, lda, B, ldb, P, M, K, N, slice_rows);
  HT_LAUNCH_CHECK(ctx);
  k_reduce_slices<<<(unsigned)((kn + 255) / 256), 256, 0, st>>>(P, kn, (int)slices, accumulate, C);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

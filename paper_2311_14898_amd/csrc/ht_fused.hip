// Aggregate and update in one kernel (Eq. 2: AGGREGATE, then the linear transform and ReLU), for layers that keep no
// aggregate (Sec. 4.2, pure recomputation): a^l of a block of destination rows is built in LDS and consumed there by
// the matrix cores, so it never reaches HBM.  A workgroup owns 32 destination rows of a chunk.  Phase 1: each of the 8 waves
// aggregates 4 of them over their whole in-edge lists (full-width rows across the lanes as float4, fp32 FMAs in edge
// order, no cut rows and no partial sums) and writes s_v * sum into the LDS tile.  Phase 2: the tile [32 x K] times the
// packed W [K x N] on v_mfma_f32_32x32x2_f32, a wave per 32-column block, the activation in the epilogue.
// An A/B variant (HT_FUSE_UPDATE=1): one workgroup per CU fits beside the 78 KB tile of a 602-wide layer, which starves a
// gather that lives on many waves in flight; the separate kernels are faster and stay the default.
#include "ht_internal.h"

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }

struct FusedArgs {
  const int64_t* rowptr;   // [V+1] entry offsets of every destination's list (global)
  const int32_t* idx;      // per entry: source row (global id)
  const float* w_edge;     // per-entry weights (nullable)
  const float* ew;         // weight table indexed by source (used when w_edge is null)
  const float* src;        // layer input [V x src_ld]
  int64_t src_ld;
  const float* post;       // s_v per destination (global)
  const float* Bp;         // packed W [Kp x Np], zero-padded
  int32_t Np;
  float* out;              // H_out
  int64_t out_ld;
  int64_t dst0, ndst;      // the chunk's destination range
  int32_t K, N, pitch, relu;
};

template <int VPL>
__global__ void __launch_bounds__(512) k_agg_update(FusedArgs a) {
  extern __shared__ float tile[];   // [32][pitch], pitch odd: conflict-free column reads in phase 2
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t r0 = (int64_t)blockIdx.x * 32;
  const int K = a.K, pitch = a.pitch;
  // ---- phase 1: aggregate
  for (int rr = wave; rr < 32; rr += 8) {
    const int64_t row = r0 + rr;
    float4 acc[VPL];
#pragma unroll
    for (int j = 0; j < VPL; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row < a.ndst) {
      const int64_t v = a.dst0 + row;
      const int64_t e0 = a.rowptr[v], e1 = a.rowptr[v + 1];
      for (int64_t base = e0; base < e1; base += 64) {
        const int n_here = (e1 - base) < 64 ? (int)(e1 - base) : 64;
        int32_t my_idx = 0;
        float my_w = 0.f;
        if (lane < n_here) {
          my_idx = a.idx[base + lane];
          my_w = a.w_edge ? a.w_edge[base + lane] : a.ew[my_idx];
        }
        for (int k = 0; k < n_here; k += 4) {   // four row reads in flight
          int32_t c[4];
          float w[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int kk = k + u, kc = kk < n_here ? kk : n_here - 1;   // past the end: the last entry again, weight 0
            c[u] = __builtin_amdgcn_readlane(my_idx, kc);
            w[u] = kk < n_here ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_w), kc)) : 0.f;
          }
#pragma unroll
          for (int j = 0; j < VPL; ++j) {
            const int c4 = (j * 64 + lane) * 4;
            if (c4 < K) {
              float4 x[4];
#pragma unroll
              for (int u = 0; u < 4; ++u) x[u] = ld4(a.src + (int64_t)c[u] * a.src_ld + c4);
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                acc[j].x = fmaf(w[u], x[u].x, acc[j].x);
                acc[j].y = fmaf(w[u], x[u].y, acc[j].y);
                acc[j].z = fmaf(w[u], x[u].z, acc[j].z);
                acc[j].w = fmaf(w[u], x[u].w, acc[j].w);
              }
            }
          }
        }
      }
    }
    const float post = row < a.ndst ? a.post[a.dst0 + row] : 0.f;
    float* t = tile + rr * pitch;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int c4 = (j * 64 + lane) * 4;
      if (c4 < pitch - 1) {            // columns K .. pitch-2 are pad: zero (the row's pad floats in HBM are not data)
        t[c4 + 0] = c4 + 0 < K ? post * acc[j].x : 0.f;
        t[c4 + 1] = c4 + 1 < K ? post * acc[j].y : 0.f;
        t[c4 + 2] = c4 + 2 < K ? post * acc[j].z : 0.f;
        t[c4 + 3] = c4 + 3 < K ? post * acc[j].w : 0.f;
      }
    }
  }
  __syncthreads();
  // ---- phase 2: transform on the matrix cores; D layout of a 32x32 tile: lane holds column l32, rows (e/4)*8 + half*4 + e%4
  const int l32 = lane & 31, half = lane >> 5;
  const int K2 = (K + 1) & ~1;
  for (int n0 = wave * 32; n0 < a.N; n0 += 256) {
    v16f acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    const float* bp = a.Bp + n0 + l32;
    const float* ap = tile + l32 * pitch + half;
    const int64_t np = a.Np;
    int k = 0;
    for (; k + 8 <= K2; k += 8) {   // four operand pairs in flight
      const float a0 = ap[k], a1 = ap[k + 2], a2 = ap[k + 4], a3 = ap[k + 6];
      const float b0 = bp[(k + half) * np], b1 = bp[(k + 2 + half) * np], b2 = bp[(k + 4 + half) * np], b3 = bp[(k + 6 + half) * np];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a2, b2, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a3, b3, acc, 0, 0, 0);
    }
    for (; k < K2; k += 2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[k], bp[(k + half) * np], acc, 0, 0, 0);
    const int gc = n0 + l32;
    if (gc < a.N) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t row = r0 + (e / 4) * 8 + half * 4 + (e % 4);
        if (row < a.ndst) {
          float v = acc[e];
          if (a.relu) v = v > 0.f ? v : 0.f;
          a.out[(a.dst0 + row) * a.out_ld + gc] = v;
        }
      }
    }
  }
}

}  // namespace

int ht_pack_w(ht_ctx* ctx, hipStream_t st, const float* W, int32_t K, int32_t N, float** Bp, int* Np);

// H_out[dst0 .. dst1) = act((A_hat H_in)[rows] W) for one chunk, the aggregate kept in LDS.  H_in in HBM, read in place.
int ht_agg_update_fused(ht_ctx* ctx, hipStream_t st, const ht_graph* g, const ChunkMeta& c, const float* H_in, int64_t in_ld,
                        int32_t d_in, const float* W, int32_t d_out, int relu, float* H_out, int64_t out_ld) {
  const int64_t ndst = c.dst1 - c.dst0;
  if (ndst <= 0) return HT_OK;
  if (in_ld & 3) return ht_set_err(ctx, HT_ESHAPE, "fused layer step: row pitch must be a multiple of 4");
  if (d_in > 1024) return ht_set_err(ctx, HT_ESHAPE, "fused layer step: d_in = %d is wider than the 1024 columns its LDS tile holds", d_in);
  FusedArgs a{};
  a.rowptr = g->merged ? g->uindptr.p : g->indptr.p;
  a.idx = g->merged ? g->ucol.p : g->col.p;
  a.w_edge = g->merged ? g->uw_fwd.p : nullptr;
  a.ew = g->s.p;
  a.src = H_in;
  a.src_ld = in_ld;
  a.post = g->s.p;
  float* Bp = nullptr;
  int Np = 0;
  HT_TRY(ht_pack_w(ctx, st, W, d_in, d_out, &Bp, &Np));
  a.Bp = Bp;
  a.Np = Np;
  a.out = H_out;
  a.out_ld = out_ld;
  a.dst0 = c.dst0;
  a.ndst = ndst;
  a.K = d_in;
  a.N = d_out;
  a.pitch = ((d_in + 3) & ~3) + 1;
  a.relu = relu;
  const size_t sh = (size_t)32 * a.pitch * sizeof(float);
  const unsigned nb = (unsigned)((ndst + 31) / 32);
  const int vpl = (((d_in + 3) >> 2) + 63) / 64;
  // the dynamic LDS limit of each instantiation is raised once per process (the call is not free)
#define HT_FUSED_LAUNCH(V)                                                                                                \
  do {                                                                                                                    \
    static bool raised = false;                                                                                           \
    if (!raised) {                                                                                                        \
      HT_HIP(ctx, hipFuncSetAttribute((const void*)k_agg_update<V>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)); \
      raised = true;                                                                                                      \
    }                                                                                                                     \
    k_agg_update<V><<<nb, 512, sh, st>>>(a);                                                                              \
  } while (0)
  if (vpl <= 1) HT_FUSED_LAUNCH(1);
  else if (vpl == 2) HT_FUSED_LAUNCH(2);
  else if (vpl == 3) HT_FUSED_LAUNCH(3);
  else HT_FUSED_LAUNCH(4);
#undef HT_FUSED_LAUNCH
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

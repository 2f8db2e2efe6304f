// Aggregation (Eq. 2's AGGREGATE and its backward, Sec. 4.1) and the row
// gather / scatter kernels of the in-place neighbour buffer (Alg. 2,
// Alg. 3).
//
// Aggregation: a wave owns one work item (at most HT_SEG edges of one row).
// Features run across lanes as float4; for narrow rows a wave splits into
// lane groups that take interleaved edges and are summed in a fixed order.
// No atomics: a row cut into several items is finished by a second kernel
// that adds the partial sums in item order, so results are bit-reproducible.
#include "ht_internal.h"

namespace {

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ float4 fma4(float w, float4 v, float4 a) {
  a.x = fmaf(w, v.x, a.x);
  a.y = fmaf(w, v.y, a.y);
  a.z = fmaf(w, v.z, a.z);
  a.w = fmaf(w, v.w, a.w);
  return a;
}
__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ __forceinline__ float4 mul4(float s, float4 a) { return make_float4(s * a.x, s * a.y, s * a.z, s * a.w); }
__device__ __forceinline__ float4 shfl_xor4(float4 v, int o) {
  return make_float4(__shfl_xor(v.x, o, 64), __shfl_xor(v.y, o, 64), __shfl_xor(v.z, o, 64), __shfl_xor(v.w, o, 64));
}

// Final write of one output row's float4 column `c4` (in floats).
__device__ __forceinline__ void write_out(const SpmmArgs& a, int32_t r, int c4, float4 v) {
  const float post = a.post ? a.post[a.post_idx ? a.post_idx[r] : r] : 1.f;
  uint32_t orow = a.out_idx ? (uint32_t)a.out_idx[r] : (uint32_t)r;
  const bool fresh = (orow & 0x80000000u) != 0u;
  orow &= 0x7FFFFFFFu;
  float* p = a.out + (int64_t)orow * a.out_ld + c4;
  v = mul4(post, v);
  if (a.accumulate && !fresh) v = add4(ld4(p), v);
  if (a.relu) v = make_float4(v.x > 0.f ? v.x : 0.f, v.y > 0.f ? v.y : 0.f, v.z > 0.f ? v.z : 0.f, v.w > 0.f ? v.w : 0.f);
  st4(p, v);
}

template <int LPR, int VPL>
__global__ void __launch_bounds__(256) k_spmm_items(SpmmArgs a) {
  constexpr int G = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= a.n_items) return;
  const int32_t r = a.it_row[t];
  const int64_t e0 = a.it_e0[t];
  const int32_t len = a.it_len[t];
  const int32_t part = a.it_part[t];
  const int sub = lane / LPR, ll = lane % LPR;
  const int d4 = (a.d + 3) & ~3;

  float4 acc[VPL];
  bool colok[VPL];
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    colok[j] = (j * LPR + ll) * 4 < d4;
  }
  for (int32_t base = 0; base < len; base += 64) {
    const int32_t n_here = (len - base) < 64 ? (len - base) : 64;
    int32_t my_idx = 0;
    float my_w = 0.f;
    if (lane < n_here) {
      my_idx = a.idx[e0 + base + lane];
      my_w = a.w_edge ? a.w_edge[e0 + base + lane] : (a.ew ? a.ew[my_idx] : 1.f);
    }
    for (int32_t k = 0; k < n_here; k += G) {
      int32_t c;
      float w;
      if (G == 1) {
        c = __builtin_amdgcn_readlane(my_idx, k);
        w = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_w), k));
      } else {
        const int kk = k + sub;           // lanes past the end carry weight 0 and row 0
        c = __shfl(my_idx, kk & 63, 64);
        w = __shfl(my_w, kk & 63, 64);
        if (kk >= n_here) { c = 0; w = 0.f; }
      }
      const float* row = a.src + (int64_t)c * a.src_ld;
#pragma unroll
      for (int j = 0; j < VPL; ++j)
        if (colok[j]) acc[j] = fma4(w, ld4(row + (j * LPR + ll) * 4), acc[j]);
    }
  }
  if (G > 1) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1)
#pragma unroll
      for (int j = 0; j < VPL; ++j) acc[j] = add4(acc[j], shfl_xor4(acc[j], o));
    if (sub != 0) return;
  }
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    if (!colok[j]) continue;
    const int c4 = (j * LPR + ll) * 4;
    if (part >= 0)
      st4(a.partial + (int64_t)part * a.out_ld + c4, acc[j]);
    else
      write_out(a, r, c4, acc[j]);
  }
}

// Rows cut into several items: add their partial sums in item order.  One
// block per row; each wave adds a contiguous quarter of the partial sums, the
// four results are added in wave order.
__global__ void __launch_bounds__(256) k_spmm_fix(SpmmArgs a) {
  __shared__ float4 sh[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t f = blockIdx.x;
  const int32_t r = a.fx_row[f];
  const int32_t p0 = a.fx_part0[f];
  const int32_t ns = a.fx_nseg[f];
  const int d4 = (a.d + 3) & ~3;
  const int32_t per = (ns + 3) >> 2;
  const int32_t k0 = wave * per, k1 = (k0 + per) < ns ? (k0 + per) : ns;
  for (int cb = 0; cb < d4; cb += 256) {
    const int c4 = cb + lane * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c4 < d4) {
      const float* p = a.partial + (int64_t)p0 * a.out_ld + c4;
      int32_t k = k0;
      for (; k + 4 <= k1; k += 4) {
        const float4 v0 = ld4(p + (int64_t)(k + 0) * a.out_ld);
        const float4 v1 = ld4(p + (int64_t)(k + 1) * a.out_ld);
        const float4 v2 = ld4(p + (int64_t)(k + 2) * a.out_ld);
        const float4 v3 = ld4(p + (int64_t)(k + 3) * a.out_ld);
        acc = add4(add4(add4(add4(acc, v0), v1), v2), v3);
      }
      for (; k < k1; ++k) acc = add4(acc, ld4(p + (int64_t)k * a.out_ld));
    }
    sh[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && c4 < d4) {
      float4 t = add4(add4(add4(sh[0][lane], sh[1][lane]), sh[2][lane]), sh[3][lane]);
      write_out(a, r, c4, t);
    }
    __syncthreads();
  }
}

// Feature-slab variant.  The 8 XCDs each have their own L2; workgroups go to
// XCDs round-robin by id, so workgroup b runs on XCD b % 8.  Giving every XCD a
// fixed slab of the feature columns makes its L2 hold 8x more distinct source
// rows than full-width rows would.  A wave owns one item and one slab; lanes
// are (edge slot, float4 of the slab); `eps` edges are read per step.
template <int U, bool UNI>
__global__ void __launch_bounds__(256) k_spmm_slab(SpmmArgs a, int S, int nvs, int eps, int64_t grp_per_part, int slab0) {
  // the wave index is the same in all 64 lanes: saying so keeps the item's fields and the loop control in scalar registers
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int xcd = blockIdx.x & 7;
  const int slab = slab0 + xcd % S;
  // The 8/S XCDs that share a slab split the (source-ordered) item list into contiguous parts
  // (grp_per_part > 0), so their L2s hold different source rows; or interleave it (grp_per_part = 0).
  const int64_t i = blockIdx.x >> 3;
  if (grp_per_part > 0 && i >= grp_per_part) return;
  const int64_t grp = grp_per_part > 0 ? (int64_t)(xcd / S) * grp_per_part + i : i * (8 / S) + xcd / S;
  const int64_t t = grp * 4 + wave;
  if (t >= a.n_items) return;
  const int nvec = (a.d + 3) >> 2;
  const int v0 = slab * nvs;
  const int nv_here = (nvec - v0) < nvs ? (nvec - v0) : nvs;
  if (nv_here <= 0) return;
  const int32_t r = a.it_row[t];
  const int64_t e0 = a.it_e0[t];
  const int32_t len = a.it_len[t];
  const int32_t part = a.it_part[t];
  const int es = lane / nvs, vec = lane - es * nvs;
  const bool active = es < eps && vec < nv_here;
  const int coff = (v0 + vec) * 4;
  const float* srcc = a.src + coff;

  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int32_t base = 0; base < len; base += 64) {
    const int32_t n_here = (len - base) < 64 ? (len - base) : 64;
    int32_t my_idx = 0;
    float my_w = 0.f;
    if (lane < n_here) {
      my_idx = a.idx[e0 + base + lane];
      my_w = a.w_edge ? a.w_edge[e0 + base + lane] : (a.ew ? a.ew[my_idx] : 1.f);
    }
    if (UNI) {
      // one edge per step for the whole wave: the index and weight are wave-uniform
      for (int32_t k = 0; k < n_here; k += U) {
        int32_t c[U];
        float w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int kk = k + u;
          const int kc = kk < n_here ? kk : (n_here - 1);
          c[u] = __builtin_amdgcn_readlane(my_idx, kc);
          w[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_w), kc));
          if (kk >= n_here) w[u] = 0.f;
        }
        if (active) {
          float4 v[U];
#pragma unroll
          for (int u = 0; u < U; ++u) v[u] = ld4(srcc + (int64_t)c[u] * a.src_ld);
#pragma unroll
          for (int u = 0; u < U; ++u) acc = fma4(w[u], v[u], acc);
        }
      }
    } else {
      for (int32_t k = 0; k < n_here; k += U * eps) {
        int32_t c[U];
        float w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int kk = k + u * eps + es;
          const int kc = kk < n_here ? kk : (n_here - 1);   // past the end: re-read the last edge with weight 0
          c[u] = __shfl(my_idx, kc, 64);
          w[u] = __shfl(my_w, kc, 64);
          if (kk >= n_here) w[u] = 0.f;
        }
        if (active) {
          float4 v[U];
#pragma unroll
          for (int u = 0; u < U; ++u) v[u] = ld4(srcc + (int64_t)c[u] * a.src_ld);
#pragma unroll
          for (int u = 0; u < U; ++u) acc = fma4(w[u], v[u], acc);
        }
      }
    }
  }
  // add the edge slots in slot order; slot 0 holds the result
  float4 tot = acc;
  for (int q = 1; q < eps; ++q) {
    const int from = (lane + q * nvs) & 63;
    float4 o = make_float4(__shfl(acc.x, from, 64), __shfl(acc.y, from, 64), __shfl(acc.z, from, 64), __shfl(acc.w, from, 64));
    tot = add4(tot, o);
  }
  if (es != 0 || vec >= nv_here) return;
  if (part >= 0)
    st4(a.partial + (int64_t)part * a.out_ld + coff, tot);
  else
    write_out(a, r, coff, tot);
}

template <int LPR, int VPL>
int launch_items(ht_ctx* ctx, hipStream_t st, const SpmmArgs& a) {
  const unsigned blocks = (unsigned)((a.n_items + 3) / 4);
  k_spmm_items<LPR, VPL><<<blocks, 256, 0, st>>>(a);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

// dst[dst_idx[k]] = scale[src_idx[k]] * src[src_idx[k]]; a lane group per row,
// grid-stride over rows so the launch can be kept small (see ht_gather_rows).
template <int ADD>
__global__ void __launch_bounds__(256) k_rows(const float* __restrict__ src, int64_t src_ld,
                                              const int32_t* __restrict__ src_idx, float* __restrict__ dst,
                                              int64_t dst_ld, const int32_t* __restrict__ dst_idx, int64_t n_rows,
                                              int d4, int lpr, const float* __restrict__ scale) {
  const int tid = threadIdx.x;
  const int rows_per_block = 256 / lpr;
  const int ll = tid % lpr;
  for (int64_t k = (int64_t)blockIdx.x * rows_per_block + tid / lpr; k < n_rows;
       k += (int64_t)gridDim.x * rows_per_block) {
    const int64_t si = src_idx ? (int64_t)src_idx[k] : k;
    const int64_t di = dst_idx ? (int64_t)(dst_idx[k] & 0x7FFFFFFF) : k;
    const float sc = scale ? scale[si] : 1.f;
    const float* sp = src + si * src_ld;
    float* dp = dst + di * dst_ld;
    for (int c4 = ll * 4; c4 < d4; c4 += lpr * 4) {
      float4 v = ld4(sp + c4);
      if (scale) v = mul4(sc, v);
      if (ADD) v = add4(ld4(dp + c4), v);
      st4(dp + c4, v);
    }
  }
}

// Contiguous copy of n16 16-byte words with a small fixed grid: four loads in
// flight per lane, grid-stride.  Used for rows that cross the host link, where a
// few dozen waves saturate the link and a device-filling launch would only
// crowd out the compute kernels running beside it.
__global__ void __launch_bounds__(256) k_copy16(const float4* __restrict__ src, float4* __restrict__ dst, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const float4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a;
    dst[i + stride] = b;
    dst[i + 2 * stride] = c;
    dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

int lanes_for(int nvec) { return nvec <= 8 ? 8 : nvec <= 16 ? 16 : nvec <= 32 ? 32 : 64; }

// Grid of a row kernel: one lane group per row, at most `cap` blocks (k_rows strides over the rest).  A launch of
// 2^32 threads or more is not rejected, its excess is silently dropped, so the grid is bounded whatever n_rows is.
constexpr int64_t HT_ROW_GRID_MAX = 1 << 20;
constexpr int64_t row_blocks(int64_t n_rows, int rows_per_block, int64_t cap) {
  const int64_t want = (n_rows + rows_per_block - 1) / rows_per_block;
  const int64_t lim = (cap > 0 && cap < HT_ROW_GRID_MAX) ? cap : HT_ROW_GRID_MAX;
  return want < lim ? want : lim;
}
static_assert(row_blocks(1ll << 26, 4, 0) * 256 < (1ll << 32), "a row launch must stay below 2^32 threads");
static_assert(row_blocks(111'000'000ll, 4, 0) == HT_ROW_GRID_MAX && row_blocks(int64_t(1) << 40, 1, 0) == HT_ROW_GRID_MAX, "");
static_assert(row_blocks(1000, 4, 64) == 64 && row_blocks(100, 4, 64) == 25 && row_blocks(5, 4, 0) == 2, "");

}  // namespace

int ht_spmm_launch(ht_ctx* ctx, hipStream_t st, const SpmmArgs& a0) {
  if (a0.n_items <= 0) return HT_OK;
  if ((a0.src_ld & 3) || (a0.out_ld & 3)) return ht_set_err(ctx, HT_ESHAPE, "aggregation: row pitch must be a multiple of 4");
  // wide rows go in column blocks of 1024 floats
  for (int c0 = 0; c0 < a0.d; c0 += 1024) {
    SpmmArgs a = a0;
    a.src = a0.src + c0;
    a.out = a0.out + c0;
    a.partial = a0.partial ? a0.partial + c0 : nullptr;
    a.d = (a0.d - c0) < 1024 ? (a0.d - c0) : 1024;
    const int nvec = (a.d + 3) / 4;
    int rc = HT_OK;
    if (a.tm && a.t_items) a.tm->begin(a.t_items);
    if (ctx->agg_variant == 0) {
      // Slabs cost one pass over the item's indices each, so short rows get fewer:
      // measured best on 256-wide rows is 4 slabs for ~500-edge items and 1 for ~80-edge items.
      int S = nvec >= 32 ? 4 : nvec >= 16 ? 2 : 1;
      const int64_t avg_len = a.n_edges / (a.n_items > 0 ? a.n_items : 1);
      if (avg_len < 96) S = 1;
      else if (avg_len < 192 && S > 2) S = 2;
      if (a.max_slabs > 0) S = a.max_slabs;                // experiments: force a slab count
      while (S > 1 && nvec / S < 1) S /= 2;
      int P = ctx->agg_phases;
      while (P > 1 && nvec / (S * P) < 1) P /= 2;
      while (S < 8 && (nvec + S * P - 1) / (S * P) > 64) S *= 2;   // a slab must fit the 64 lanes of a wave
      int nvs = (nvec + S * P - 1) / (S * P);
      // rows that start on 128-byte lines: slabs in whole lines, so no line is fetched by two XCDs
      if (ctx->slab_align && (a.src_ld & 31) == 0 && ((uintptr_t)a.src & 127) == 0 && nvs > 8 && ((nvs + 7) & ~7) <= 64) nvs = (nvs + 7) & ~7;
      const int eps = 64 / nvs;
      if (S < 1 || (S & (S - 1)) || S > 8 || nvs < 1 || nvs > 64 || eps < 1)
        return ht_set_err(ctx, HT_ESHAPE, "aggregation: bad slab shape S=%d nvs=%d", S, nvs);
      const int64_t groups = (a.n_items + 3) / 4;
      const int parts = 8 / S;
      const int64_t gpp = (groups + parts - 1) / parts;   // item groups per XCD of a slab
      const int64_t rows8 = ctx->xcd_contig ? gpp : (groups + parts - 1) / parts;
      for (int p = 0; p < P; ++p) {
        const unsigned nb = (unsigned)(rows8 * 8);
        const int64_t gp = ctx->xcd_contig ? gpp : 0;
        const bool uni = eps == 1 && ctx->agg_uniform;
        if (ctx->agg_unroll == 8) {
          if (uni) k_spmm_slab<8, true><<<nb, 256, 0, st>>>(a, S, nvs, eps, gp, p * S);
          else k_spmm_slab<8, false><<<nb, 256, 0, st>>>(a, S, nvs, eps, gp, p * S);
        } else {
          if (uni) k_spmm_slab<4, true><<<nb, 256, 0, st>>>(a, S, nvs, eps, gp, p * S);
          else k_spmm_slab<4, false><<<nb, 256, 0, st>>>(a, S, nvs, eps, gp, p * S);
        }
        HT_LAUNCH_CHECK(ctx);
      }
    } else if (nvec <= 8) rc = launch_items<8, 1>(ctx, st, a);
    else if (nvec <= 16) rc = launch_items<16, 1>(ctx, st, a);
    else if (nvec <= 32) rc = launch_items<32, 1>(ctx, st, a);
    else if (nvec <= 64) rc = launch_items<64, 1>(ctx, st, a);
    else if (nvec <= 128) rc = launch_items<64, 2>(ctx, st, a);
    else if (nvec <= 192) rc = launch_items<64, 3>(ctx, st, a);
    else rc = launch_items<64, 4>(ctx, st, a);
    if (a.tm && a.t_items) a.tm->end();
    if (rc != HT_OK) return rc;
    if (a.n_fix > 0) {
      if (a.tm && a.t_fix) a.tm->begin(a.t_fix);
      k_spmm_fix<<<(unsigned)a.n_fix, 256, 0, st>>>(a);
      if (a.tm && a.t_fix) a.tm->end();
      HT_LAUNCH_CHECK(ctx);
    }
  }
  return HT_OK;
}

int ht_spmm_fix_launch(ht_ctx* ctx, hipStream_t st, const SpmmArgs& a) {
  if (a.n_fix <= 0) return HT_OK;
  if (a.out_ld & 3) return ht_set_err(ctx, HT_ESHAPE, "aggregation: row pitch must be a multiple of 4");
  k_spmm_fix<<<(unsigned)a.n_fix, 256, 0, st>>>(a);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

int ht_gather_rows(ht_ctx* ctx, hipStream_t st, const float* src, int64_t src_ld, const int32_t* src_idx, float* dst,
                   int64_t dst_ld, const int32_t* dst_idx, int64_t n_rows, int32_t d, const float* scale,
                   int max_blocks) {
  if (n_rows <= 0) return HT_OK;
  const int d4 = (d + 3) & ~3;
  const int lpr = lanes_for(d4 / 4);
  const int rpb = 256 / lpr;
  const int64_t blocks = row_blocks(n_rows, rpb, max_blocks);
  k_rows<0><<<(unsigned)blocks, 256, 0, st>>>(src, src_ld, src_idx, dst, dst_ld, dst_idx, n_rows, d4, lpr, scale);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

int ht_add_rows(ht_ctx* ctx, hipStream_t st, const float* src, int64_t src_ld, const int32_t* src_idx, float* dst,
                int64_t dst_ld, const int32_t* dst_idx, int64_t n_rows, int32_t d) {
  if (n_rows <= 0) return HT_OK;
  const int d4 = (d + 3) & ~3;
  const int lpr = lanes_for(d4 / 4);
  const int rpb = 256 / lpr;
  k_rows<1><<<(unsigned)row_blocks(n_rows, rpb, 0), 256, 0, st>>>(src, src_ld, src_idx, dst, dst_ld, dst_idx, n_rows,
                                                                d4, lpr, nullptr);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

int ht_copy_link(ht_ctx* ctx, hipStream_t st, void* dst, const void* src, size_t bytes, int blocks) {
  if (bytes == 0) return HT_OK;
  if ((bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15))
    return ht_set_err(ctx, HT_ESHAPE, "link copy: pointers and size must be multiples of 16 bytes");
  const int64_t n16 = (int64_t)(bytes >> 4);
  int64_t nb = (n16 + 255) / 256;
  if (nb > blocks) nb = blocks;
  k_copy16<<<(unsigned)nb, 256, 0, st>>>((const float4*)src, (float4*)dst, n16);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

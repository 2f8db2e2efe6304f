// GAT layer (Eq. 3), one attention head, forward and backward over the chunks
// of a partitioned graph.  The layer's tensors H_in, H_out, dH_out, dH_in may live
// in HBM or in pinned host memory; the parameterised rows t = H W of all vertices
// always stay in HBM for the duration of a call, so neighbour rows never cross the
// host link: a host-resident tensor is only ever read or written in contiguous row
// ranges (V rows per pass instead of the sum of |N_j|), through staging pairs on
// side streams.
//
//   t = H W ;  p_v = a_dst . t_v ;  q_u = a_src . t_u
//   edge (u -> v):  y = p_v + q_u ;  x = LeakyReLU(y) ;  alpha = softmax over in(v)
//   z_v = sum alpha_e t_u ;  h'_v = act(z_v)
//
// A chunk holds every in-edge of its destinations (Sec. 4.1), so the neighbour
// softmax is complete inside a chunk.  Nothing of size O(E) survives a call: the
// backward pass recomputes t, p, q and the coefficients (Sec. 4.2: for models
// with edge computation recomputation is cheaper than caching O(|E|) data).
// Per chunk, edge coefficients live in a scratch array of the chunk's size.
//
// Backward.  With dz = dh' * act'(z) and S_v = dz_v . z_v  (= sum_e alpha_e dalpha_e):
//   dalpha_e = dz_v . t_u ;  dy_e = alpha_e (dalpha_e - S_v) f_e ,  f_e = LeakyReLU'(y_e)
//   dp_v = sum_{e in in(v)} dy_e  = dz_v . (sum_e alpha_e f_e t_u) - S_v sum_e alpha_e f_e
//                                     (pass over destinations, an aggregation of rows of t)
//   dq_u = sum_{e in out(u)} dy_e = t_u . (sum_e alpha_e f_e dz_v) - sum_e alpha_e f_e S_v
//   dt_u = sum_{e in out(u)} alpha_e dz_v
//                                     (pass over sources, two aggregations of the same rows of dz)
//   dt_v += dp_v a_dst + dq_v a_src ;  da_dst = sum_v dp_v t_v ;  da_src = sum_v dq_v t_v
//   dW = H^T dt ;  dH = dt W^T
// Both passes are pulls over the work items built at partition time; rows cut
// into several items are finished in a fixed order, so results are bit-reproducible.
// Merged duplicate edges: an entry of multiplicity k stands for k equal edges,
// its coefficient is k times the single edge's.
#include <algorithm>
#include <chrono>
#include <vector>

#include "ht_internal.h"

namespace {

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ float lrelu(float y, float slope) { return y > 0.f ? y : slope * y; }
// coefficient of one entry; the same expression in every kernel, so the forward, the
// destination pass and the source pass of a chunk see identical values
__device__ __forceinline__ float coef(float y, float slope, float m, float zinv, float mult) {
  const float x = lrelu(y, slope);
  return mult * expf(x - m) * zinv;
}

// p[v] = a_dst . T[v], q[v] = a_src . T[v]; a wave per vertex
__global__ void __launch_bounds__(256) k_gat_pq(const float* __restrict__ T, int64_t ld, int d, const float* __restrict__ a_dst,
                                                const float* __restrict__ a_src, int64_t V, float* __restrict__ p,
                                                float* __restrict__ q) {
  const int lane = threadIdx.x & 63;
  for (int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); v < V; v += (int64_t)gridDim.x * 4) {
    float sp = 0.f, sq = 0.f;
    for (int c = lane; c < d; c += 64) {
      const float t = T[v * ld + c];
      sp = fmaf(a_dst[c], t, sp);
      sq = fmaf(a_src[c], t, sq);
    }
    sp = wave_sum(sp);
    sq = wave_sum(sq);
    if (lane == 0) {
      p[v] = sp;
      q[v] = sq;
    }
  }
}

// Neighbour softmax of the rows of one chunk in three steps over the work items (a wave per
// item, so a hub row is shared by many waves):
//   1. per item: the scores x_e (kept in w[]), their maximum m_i and s_i = sum mult_e exp(x_e - m_i);
//   2. per row cut into several items: m_v = max m_i, Z_v = sum s_i exp(m_i - m_v), in a fixed order;
//   3. per item: w_e = mult_e exp(x_e - m_v) / Z_v.
__global__ void __launch_bounds__(256) k_gat_scores(const int32_t* __restrict__ it_row, const int64_t* __restrict__ it_e0,
                                                    const int32_t* __restrict__ it_len, const int32_t* __restrict__ it_part,
                                                    int64_t n_items, const int32_t* __restrict__ col,
                                                    const float* __restrict__ mult, const float* __restrict__ p_chunk,
                                                    const float* __restrict__ q, float slope, float* __restrict__ w,
                                                    float* __restrict__ m_chunk, float* __restrict__ zinv_chunk,
                                                    float* __restrict__ part_m, float* __restrict__ part_s) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t t = (int64_t)blockIdx.x * 4 + wave;
  if (t >= n_items) return;
  const int32_t r = it_row[t], len = it_len[t], part = it_part[t];
  const int64_t e0 = it_e0[t];
  const float pv = p_chunk[r];
  float m = -3.0e38f;
  for (int32_t k = lane; k < len; k += 64) {
    const float x = lrelu(pv + q[col[e0 + k]], slope);
    w[e0 + k] = x;
    m = fmaxf(m, x);
  }
  m = wave_max(m);
  float s = 0.f;
  for (int32_t k = lane; k < len; k += 64) s += (mult ? mult[e0 + k] : 1.f) * expf(w[e0 + k] - m);
  s = wave_sum(s);
  if (lane == 0) {
    if (part >= 0) {
      part_m[part] = m;
      part_s[part] = s;
    } else {
      m_chunk[r] = m;
      zinv_chunk[r] = s > 0.f ? 1.f / s : 0.f;
    }
  }
}

__global__ void __launch_bounds__(256) k_gat_rowstats(const int32_t* __restrict__ fx_row, const int32_t* __restrict__ fx_part0,
                                                      const int32_t* __restrict__ fx_nseg, int64_t n_fix,
                                                      const float* __restrict__ part_m, const float* __restrict__ part_s,
                                                      float* __restrict__ m_chunk, float* __restrict__ zinv_chunk) {
  // a wave per cut row; lanes take the row's items 64 apart, lane sums are added in lane order
  const int lane = threadIdx.x & 63;
  const int64_t f = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (f >= n_fix) return;
  const int32_t p0 = fx_part0[f], ns = fx_nseg[f];
  float m = -3.0e38f;
  for (int32_t k = lane; k < ns; k += 64) m = fmaxf(m, part_m[p0 + k]);
  m = wave_max(m);
  float s = 0.f;
  for (int32_t k = lane; k < ns; k += 64) s += part_s[p0 + k] * expf(part_m[p0 + k] - m);
  s = wave_sum(s);
  if (lane == 0) {
    m_chunk[fx_row[f]] = m;
    zinv_chunk[fx_row[f]] = s > 0.f ? 1.f / s : 0.f;
  }
}

// wf / r_chunk / part_r (backward pass only, nullable): wf_e = w_e f_e with f_e = LeakyReLU'(y_e), the
// weights of the destination pass, and their sum per item (per row when the row is one item).
__global__ void __launch_bounds__(256) k_gat_coefs(const int32_t* __restrict__ it_row, const int64_t* __restrict__ it_e0,
                                                   const int32_t* __restrict__ it_len, const int32_t* __restrict__ it_part,
                                                   int64_t n_items, const float* __restrict__ mult,
                                                   const float* __restrict__ m_chunk, const float* __restrict__ zinv_chunk,
                                                   float slope, float* __restrict__ w, float* __restrict__ wf,
                                                   float* __restrict__ r_chunk, float* __restrict__ part_r) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t t = (int64_t)blockIdx.x * 4 + wave;
  if (t >= n_items) return;
  const int32_t r = it_row[t], len = it_len[t];
  const int64_t e0 = it_e0[t];
  const float m = m_chunk[r], zinv = zinv_chunk[r];
  float rs = 0.f;
  for (int32_t k = lane; k < len; k += 64) {
    const float x = w[e0 + k];       // the score LeakyReLU(y_e): same sign as y_e
    const float c = (mult ? mult[e0 + k] : 1.f) * expf(x - m) * zinv;
    w[e0 + k] = c;
    if (wf) {
      const float cf = c * (x > 0.f ? 1.f : slope);
      wf[e0 + k] = cf;
      rs += cf;
    }
  }
  if (wf) {
    rs = wave_sum(rs);
    if (lane == 0) {
      const int32_t part = it_part[t];
      if (part >= 0) part_r[part] = rs;
      else r_chunk[r] = rs;
    }
  }
}

// dp_v = dz_v . Q_v - S_v r_v; a wave per row of the chunk
__global__ void __launch_bounds__(256) k_gat_dp(const float* __restrict__ dz, const float* __restrict__ Q, int64_t ld, int d,
                                                const float* __restrict__ S, const float* __restrict__ r_chunk, int64_t rows,
                                                float* __restrict__ dp_chunk) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  float s = 0.f;
  for (int c = lane; c < d; c += 64) s = fmaf(dz[r * ld + c], Q[r * ld + c], s);
  s = wave_sum(s);
  if (lane == 0) dp_chunk[r] = s - S[r] * r_chunk[r];
}

// dz = dh * [h > 0] (or dh), pad columns zero, S_v = dz_v . h_v, and d4[row] = (p_v, m_v, 1/Z_v, S_v) (p, m, zinv
// point at the chunk's first destination); a wave per row of the chunk
__global__ void __launch_bounds__(256) k_gat_dz(const float* __restrict__ dh, int64_t ld_dh, const float* __restrict__ h,
                                                int64_t ld_h, int relu, int64_t rows, int d, float* __restrict__ dz,
                                                int64_t ld_dz, float* __restrict__ S, const float* __restrict__ p,
                                                const float* __restrict__ m, const float* __restrict__ zinv,
                                                float* __restrict__ d4) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  float s = 0.f;
  for (int c = lane; c < (int)ld_dz; c += 64) {
    float g = 0.f;
    if (c < d) {
      const float hv = h[r * ld_h + c];
      g = dh[r * ld_dh + c];
      if (relu && !(hv > 0.f)) g = 0.f;
      s = fmaf(g, hv, s);
    }
    dz[r * ld_dz + c] = g;
  }
  s = wave_sum(s);
  if (lane == 0) {
    S[r] = s;
    // what the source pass needs of a destination, in one 16-byte read per entry instead of four 4-byte ones
    st4(d4 + r * 4, make_float4(p[r], m[r], zinv[r], s));
  }
}

struct GatPass {
  // items of the source pass (rows = local sources of the chunk)
  const int32_t* it_row; const int64_t* it_e0; const int32_t* it_len; const int32_t* it_part; int64_t n_items;
  const int32_t* idx;        // per entry: local destination = row of `mat` to read
  const float* mult;         // multiplicity per entry (nullable: 1)
  const float* mat;          // rows gathered per entry: dz of the chunk
  int64_t mat_ld;
  const float* own;          // the item's own row: t
  int64_t own_ld;
  const int32_t* own_idx;    // row r -> row of `own`
  int d;
  const float* p; const float* q;        // per vertex
  const float* m; const float* zinv;     // per vertex: the coefficients are recomputed from them
  const float* S;            // per row of the chunk
  const float* d4;           // per row of the chunk: (p_v, m_v, 1/Z_v, S_v)
  int64_t dst0;              // first destination of the chunk
  float slope;
  // outputs
  float* out; int64_t out_ld; const int32_t* out_idx;   // dt rows (accumulated), scalar in column sc_col
  float* partial;            // [n_part x out_ld] partial rows of cut items
  int sc_col;
};

// per-row sums of rows cut into several items: a wave per row adds the item sums (lanes 64 apart, then lane order)
__global__ void __launch_bounds__(256) k_gat_fix_scalar(const int32_t* __restrict__ fx_row, const int32_t* __restrict__ fx_part0,
                                                        const int32_t* __restrict__ fx_nseg, int64_t n_fix,
                                                        const float* __restrict__ spart, float* __restrict__ row_sum) {
  const int lane = threadIdx.x & 63;
  const int64_t f = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (f >= n_fix) return;
  const int32_t p0 = fx_part0[f], ns = fx_nseg[f];
  float s = 0.f;
  for (int32_t k = lane; k < ns; k += 64) s += spart[p0 + k];
  s = wave_sum(s);
  if (lane == 0) row_sum[fx_row[f]] = s;
}

// Source pass: for local source i (vertex u) over its entries (u -> v) of the chunk, w_e recomputed:
//   dt_u += sum_e w_e dz_v
//   dq_u += sum_e w_e f_e (dz_v . t_u - S_v) = t_u . (sum_e w_e f_e dz_v) - sum_e w_e f_e S_v
// i.e. two aggregations of the same gathered rows of dz and one dot product per item.
template <int VPL>
__global__ void __launch_bounds__(256) k_gat_src(GatPass a) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t t = (int64_t)blockIdx.x * 4 + wave;
  if (t >= a.n_items) return;
  const int32_t r = a.it_row[t];
  const int64_t e0 = a.it_e0[t];
  const int32_t len = a.it_len[t], part = a.it_part[t];
  const int32_t u_id = a.own_idx[r];
  float4 acc[VPL], G[VPL];
#pragma unroll
  for (int j = 0; j < VPL; ++j) acc[j] = G[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  const float qu = a.q[u_id];
  float csum = 0.f;
  for (int32_t base = 0; base < len; base += 64) {
    const int32_t nh = (len - base) < 64 ? (len - base) : 64;
    int32_t my_v = 0;
    float my_c = 0.f, my_cf = 0.f, my_cs = 0.f;   // w_e, w_e f_e, w_e f_e S_v of the lane's entry
    if (lane < nh) {
      my_v = a.idx[e0 + base + lane];
      const float4 dv = ld4(a.d4 + (int64_t)my_v * 4);
      const float y = dv.x + qu;
      my_c = coef(y, a.slope, dv.y, dv.z, a.mult ? a.mult[e0 + base + lane] : 1.f);
      my_cf = my_c * (y > 0.f ? 1.f : a.slope);
      my_cs = my_cf * dv.w;
    }
    csum += wave_sum(my_cs);
    for (int32_t k = 0; k < nh; k += 4) {
      int32_t c[4];
      float w[4], wf[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int kc = (k + u) < nh ? (k + u) : (nh - 1);
        c[u] = __builtin_amdgcn_readlane(my_v, kc);
        w[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_c), kc));
        wf[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_cf), kc));
        if (k + u >= nh) w[u] = wf[u] = 0.f;
      }
      float4 x[4][VPL];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
          const int cc = (j * 64 + lane) * 4;
          x[u][j] = cc < a.d ? ld4(a.mat + (int64_t)c[u] * a.mat_ld + cc) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
          acc[j].x = fmaf(w[u], x[u][j].x, acc[j].x);
          acc[j].y = fmaf(w[u], x[u][j].y, acc[j].y);
          acc[j].z = fmaf(w[u], x[u][j].z, acc[j].z);
          acc[j].w = fmaf(w[u], x[u][j].w, acc[j].w);
          G[j].x = fmaf(wf[u], x[u][j].x, G[j].x);
          G[j].y = fmaf(wf[u], x[u][j].y, G[j].y);
          G[j].z = fmaf(wf[u], x[u][j].z, G[j].z);
          G[j].w = fmaf(wf[u], x[u][j].w, G[j].w);
        }
    }
  }
  float s = 0.f;
  float* row = part >= 0 ? a.partial + (int64_t)part * a.out_ld : a.out + (int64_t)a.out_idx[r] * a.out_ld;
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    const int c = (j * 64 + lane) * 4;
    if (c >= a.d) continue;
    const float4 mine = ld4(a.own + (int64_t)u_id * a.own_ld + c);   // pads of t are zero
    s = fmaf(mine.x, G[j].x, fmaf(mine.y, G[j].y, fmaf(mine.z, G[j].z, fmaf(mine.w, G[j].w, s))));
    float4 v = acc[j];
    if (part < 0) {
      const float4 o = ld4(row + c);
      v = make_float4(o.x + v.x, o.y + v.y, o.z + v.z, o.w + v.w);
    }
    st4(row + c, v);
  }
  s = wave_sum(s);
  if (lane == 0) {
    // the scalar travels in its own float4 column block behind the data columns
    float4 sc = make_float4(s - csum, 0.f, 0.f, 0.f);
    if (part < 0) sc.x += row[a.sc_col];
    st4(row + a.sc_col, sc);
  }
}

template <int G_>
__global__ void __launch_bounds__(256) k_gat_src_g(GatPass a) {
  constexpr int NG = 64 / G_;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t t = (int64_t)blockIdx.x * 4 + wave;
  if (t >= a.n_items) return;
  const int32_t r = a.it_row[t];
  const int64_t e0 = a.it_e0[t];
  const int32_t len = a.it_len[t], part = a.it_part[t];
  const int32_t u_id = a.own_idx[r];
  const int grp = lane / G_, c4 = (lane % G_) * 4;
  const bool has = c4 < a.d;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 acc = zero, G = zero;
  const float qu = a.q[u_id];
  float csum = 0.f;
  for (int32_t base = 0; base < len; base += 64) {
    const int32_t nh = (len - base) < 64 ? (len - base) : 64;
    int32_t my_v = 0;
    float my_c = 0.f, my_cf = 0.f, my_cs = 0.f;
    if (lane < nh) {
      my_v = a.idx[e0 + base + lane];
      const float4 dv = ld4(a.d4 + (int64_t)my_v * 4);
      const float y = dv.x + qu;
      my_c = coef(y, a.slope, dv.y, dv.z, a.mult ? a.mult[e0 + base + lane] : 1.f);
      my_cf = my_c * (y > 0.f ? 1.f : a.slope);
      my_cs = my_cf * dv.w;
    }
    csum += wave_sum(my_cs);
    for (int32_t k = 0; k < nh; k += 4 * NG) {
      float4 x[4];
      float w[4], wf[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int ent = k + u * NG + grp;
        const int kc = ent < nh ? ent : (nh - 1);
        const int32_t c = __shfl(my_v, kc, 64);
        w[u] = __shfl(my_c, kc, 64);
        wf[u] = __shfl(my_cf, kc, 64);
        if (ent >= nh) w[u] = wf[u] = 0.f;
        x[u] = has ? ld4(a.mat + (int64_t)c * a.mat_ld + c4) : zero;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        acc.x = fmaf(w[u], x[u].x, acc.x);
        acc.y = fmaf(w[u], x[u].y, acc.y);
        acc.z = fmaf(w[u], x[u].z, acc.z);
        acc.w = fmaf(w[u], x[u].w, acc.w);
        G.x = fmaf(wf[u], x[u].x, G.x);
        G.y = fmaf(wf[u], x[u].y, G.y);
        G.z = fmaf(wf[u], x[u].z, G.z);
        G.w = fmaf(wf[u], x[u].w, G.w);
      }
    }
  }
#pragma unroll
  for (int o = G_; o < 64; o <<= 1) {
    acc.x += __shfl_xor(acc.x, o, 64);
    acc.y += __shfl_xor(acc.y, o, 64);
    acc.z += __shfl_xor(acc.z, o, 64);
    acc.w += __shfl_xor(acc.w, o, 64);
  }
  float s = 0.f;
  float* row = part >= 0 ? a.partial + (int64_t)part * a.out_ld : a.out + (int64_t)a.out_idx[r] * a.out_ld;
  if (has) {
    const float4 mine = ld4(a.own + (int64_t)u_id * a.own_ld + c4);
    s = fmaf(mine.x, G.x, fmaf(mine.y, G.y, fmaf(mine.z, G.z, mine.w * G.w)));
    if (grp == 0) {
      float4 v = acc;
      if (part < 0) {
        const float4 o = ld4(row + c4);
        v = make_float4(o.x + v.x, o.y + v.y, o.z + v.z, o.w + v.w);
      }
      st4(row + c4, v);
    }
  }
  s = wave_sum(s);
  if (lane == 0) {
    float4 sc = make_float4(s - csum, 0.f, 0.f, 0.f);
    if (part < 0) sc.x += row[a.sc_col];
    st4(row + a.sc_col, sc);
  }
}

// dt_v += dp_v a_dst + dq_v a_src; the pair (dp_v, dq_v) also goes to a [V x 4] matrix for da = T^T [dp dq]
__global__ void __launch_bounds__(256) k_gat_finish(float* __restrict__ dT, int64_t ld, int d, int sc_col,
                                                    const float* __restrict__ dp, const float* __restrict__ a_dst,
                                                    const float* __restrict__ a_src, int64_t V, float* __restrict__ pq4) {
  const int lane = threadIdx.x & 63;
  for (int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); v < V; v += (int64_t)gridDim.x * 4) {
    const float dpv = dp[v], dqv = dT[v * ld + sc_col];
    for (int c = lane; c < d; c += 64) dT[v * ld + c] += dpv * a_dst[c] + dqv * a_src[c];
    if (lane == 0) st4(pq4 + v * 4, make_float4(dpv, dqv, 0.f, 0.f));
  }
}

__global__ void k_gat_split(const float* __restrict__ da4, int d, float* __restrict__ da_dst, float* __restrict__ da_src) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c < d) {
    da_dst[c] = da4[c * 4 + 0];
    da_src[c] = da4[c * 4 + 1];
  }
}

struct GatWs {
  float *T, *p, *q, *m, *zinv, *S, *dp, *r, *pq4, *d4, *w, *wf;
  int64_t ld_t;
};

// Contiguous row ranges between pinned host memory and staging pairs in HBM: copies run on the
// side streams, the compute stream waits for the block it needs and frees the block it has read.
struct Link {
  ht_ctx* ctx;
  ht_stats* st;
  Timer* tm;
  hipStream_t s_c, s_in, s_out;
  hipEvent_t last_out = nullptr;
  bool used = false;
  Link(ht_ctx* c, ht_stats* s, Timer* t) : ctx(c), st(s), tm(t), s_c(c->stream), s_in(c->side[0]), s_out(c->side[1]) {}
  // A failed call must not leave side-stream work that refers to the caller's buffers.
  ~Link() {
    if (used) {
      (void)hipStreamSynchronize(s_in);
      (void)hipStreamSynchronize(s_out);
    }
  }
  int rec(hipStream_t s, hipEvent_t* out) {
    hipEvent_t e = ht_event(ctx);
    if (!e) return ht_set_err(ctx, HT_EHIP, "hipEventCreate failed");
    HT_HIP(ctx, hipEventRecord(e, s));
    *out = e;
    return HT_OK;
  }
  int wait(hipStream_t s, hipEvent_t e) {
    if (e) HT_HIP(ctx, hipStreamWaitEvent(s, e, 0));
    return HT_OK;
  }
  // the side streams start behind everything the compute stream has been given so far
  int fork() {
    hipEvent_t e = nullptr;
    HT_TRY(rec(s_c, &e));
    HT_TRY(wait(s_in, e));
    HT_TRY(wait(s_out, e));
    used = true;
    return HT_OK;
  }
  // the compute stream continues behind every store to the host
  int join() {
    HT_TRY(wait(s_c, last_out));
    hipEvent_t e = nullptr;
    HT_TRY(rec(s_in, &e));
    return wait(s_c, e);
  }
  int copy(hipStream_t s, void* dst, const void* src, size_t bytes, bool to_host) {
    if (bytes == 0) return HT_OK;
    const int id = tm->begin_on(&st->t_copy_ms, s);
    if (ctx->link_memcpy) {
      HT_HIP(ctx, hipMemcpyAsync(dst, src, bytes, to_host ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice, s));
    } else {
      void* mapped = nullptr;
      HT_HIP(ctx, hipHostGetDevicePointer(&mapped, to_host ? dst : const_cast<void*>(src), 0));
      HT_TRY(ht_copy_link(ctx, s, to_host ? mapped : dst, to_host ? src : mapped, bytes, ctx->link_blocks));
    }
    tm->end_id(id);
    (to_host ? st->bytes_d2h : st->bytes_h2d) += (int64_t)bytes;
    return HT_OK;
  }
};

inline bool on_host(const ht_tensor* t) { return t && t->loc == HT_LOC_HOST_PINNED; }

int check(ht_ctx* ctx, const ht_graph* g, const ht_gat_desc* desc, const ht_tensor* t, int32_t cols, const char* name) {
  if (!t || !t->ptr) return ht_set_err(ctx, HT_EINVAL, "%s: null tensor", name);
  if (t->rows != g->V || t->cols != cols) return ht_set_err(ctx, HT_ESHAPE, "%s: expected [%lld x %d]", name, (long long)g->V, cols);
  if (t->ld < cols || (t->ld & 3) || ((uintptr_t)t->ptr & 15)) return ht_set_err(ctx, HT_ESHAPE, "%s: bad pitch or alignment", name);
  if (t->loc != HT_LOC_DEVICE && t->loc != HT_LOC_HOST_PINNED) return ht_set_err(ctx, HT_ESHAPE, "%s: unknown location", name);
  (void)desc;
  return HT_OK;
}

int check_desc(ht_ctx* ctx, const ht_gat_desc* d) {
  if (d->d_in <= 0 || d->d_out <= 0) return ht_set_err(ctx, HT_ESHAPE, "layer widths must be positive");
  if (d->d_out > 1024) return ht_set_err(ctx, HT_ESHAPE, "GAT layer: d_out %d > 1024", d->d_out);
  if (d->act != HT_ACT_NONE && d->act != HT_ACT_RELU) return ht_set_err(ctx, HT_EINVAL, "unknown activation %d", d->act);
  if (!(d->slope >= 0.f && d->slope <= 1.f)) return ht_set_err(ctx, HT_EINVAL, "LeakyReLU slope must lie in [0, 1]");
  return HT_OK;
}

// t = H W (pad columns zero), p, q
constexpr int64_t BLOCK_HBM = (int64_t)1 << 22;    // rows per GEMM call

int prepare(ht_ctx* ctx, const ht_graph* g, const ht_gat_desc* desc, const ht_tensor* H, const float* W, const float* a_dst,
            const float* a_src, bool backward, GatWs* ws, ht_stats* st, Timer* tm, Link* lk) {
  hipStream_t s = ctx->stream;
  const int64_t V = std::max<int64_t>(g->V, 1);
  ws->ld_t = ht_row_pitch(desc->d_out, true);
  HT_TRY(ht_scratch(ctx, HT_S_TFULL, (size_t)V * ws->ld_t * 4, (void**)&ws->T));
  float* vec = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_GATV, (size_t)V * 16 * 4, (void**)&vec));
  ws->p = vec; ws->q = vec + V; ws->m = vec + 2 * V; ws->zinv = vec + 3 * V; ws->S = vec + 4 * V; ws->dp = vec + 5 * V;
  ws->r = vec + 6 * V;
  ws->pq4 = vec + 8 * V;      // 16-byte aligned whatever V is
  ws->d4 = vec + 12 * V;      // per chunk, rows of the chunk
  const size_t ne = (size_t)std::max<int64_t>(g->max_nnz, 1);
  HT_TRY(ht_scratch(ctx, HT_S_GATE, ne * 4 * (backward ? 2 : 1), (void**)&ws->w));
  ws->wf = backward ? ws->w + ne : nullptr;
  if (ws->ld_t != desc->d_out) HT_TRY(ht_fill_zero(ctx, s, ws->T, (size_t)g->V * ws->ld_t * 4));
  const bool host = on_host(H);
  const int64_t step = host ? ctx->link_block_rows : BLOCK_HBM;   // rows per staged block / per GEMM call
  float* stage[2] = {nullptr, nullptr};
  hipEvent_t ev_free[2] = {nullptr, nullptr};
  if (host) {
    const int64_t rows = std::min<int64_t>(step, V);
    HT_TRY(ht_scratch(ctx, HT_S_LINK0, (size_t)rows * H->ld * 4 * 2, (void**)&stage[0]));
    stage[1] = stage[0] + rows * H->ld;
  }
  int k = 0;
  for (int64_t r0 = 0; r0 < g->V; r0 += step, ++k) {
    const int64_t nr = std::min(step, g->V - r0);
    const float* rows = H->ptr + r0 * H->ld;
    const int b = k & 1;
    if (host) {
      hipEvent_t ev_in = nullptr;
      HT_TRY(lk->wait(lk->s_in, ev_free[b]));
      HT_TRY(lk->copy(lk->s_in, stage[b], rows, (size_t)nr * H->ld * 4, false));
      HT_TRY(lk->rec(lk->s_in, &ev_in));
      HT_TRY(lk->wait(s, ev_in));
      rows = stage[b];
    }
    tm->begin(&st->t_gemm_ms);
    HT_TRY(ht_gemm_nn(ctx, s, rows, H->ld, W, ws->T + r0 * ws->ld_t, ws->ld_t, nr, desc->d_in, desc->d_out, 0));
    tm->end();
    if (host) HT_TRY(lk->rec(s, &ev_free[b]));
    st->n_gemm += 1;
    st->gemm_flops += 2.0 * nr * desc->d_in * desc->d_out;
  }
  if (g->V > 0) {
    k_gat_pq<<<(unsigned)std::min<int64_t>((g->V + 3) / 4, 1 << 22), 256, 0, s>>>(ws->T, ws->ld_t, desc->d_out, a_dst, a_src, g->V, ws->p, ws->q);
    HT_LAUNCH_CHECK(ctx);
  }
  return HT_OK;
}

int softmax_chunk(ht_ctx* ctx, const ht_graph* g, const ChunkMeta& c, const ht_gat_desc* desc, const GatWs& ws, ht_stats* st,
                  Timer* tm, bool backward) {
  const int32_t* col = g->merged ? g->ucol.p + c.ue0 : g->col.p + c.e0;
  const float* mult = g->merged ? g->umult.p + c.ue0 : nullptr;
  const ItemSet& it = c.fwd;
  // rows without an in-edge (possible without self-loops) have no item: coefficient sums of 0
  HT_TRY(ht_fill_zero(ctx, ctx->stream, ws.zinv + c.dst0, (size_t)(c.dst1 - c.dst0) * 4));
  if (it.n_items == 0) return HT_OK;
  float* part = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_GATP, (size_t)std::max<int64_t>(g->max_fpart, 1) * 3 * 4, (void**)&part));
  float* part_s = part + std::max<int64_t>(g->max_fpart, 1);
  float* part_r = part_s + std::max<int64_t>(g->max_fpart, 1);
  if (backward) HT_TRY(ht_fill_zero(ctx, ctx->stream, ws.r + c.dst0, (size_t)(c.dst1 - c.dst0) * 4));
  const unsigned nb = (unsigned)((it.n_items + 3) / 4);
  tm->begin(&st->t_gat_softmax_ms);
  k_gat_scores<<<nb, 256, 0, ctx->stream>>>(it.row, it.e0, it.len, it.part, it.n_items, col, mult, ws.p + c.dst0, ws.q,
                                            desc->slope, ws.w, ws.m + c.dst0, ws.zinv + c.dst0, part, part_s);
  if (it.n_fix > 0)
    k_gat_rowstats<<<(unsigned)((it.n_fix + 3) / 4), 256, 0, ctx->stream>>>(it.fx_row, it.fx_part0, it.fx_nseg, it.n_fix,
                                                                               part, part_s, ws.m + c.dst0, ws.zinv + c.dst0);
  k_gat_coefs<<<nb, 256, 0, ctx->stream>>>(it.row, it.e0, it.len, it.part, it.n_items, mult, ws.m + c.dst0, ws.zinv + c.dst0,
                                           desc->slope, ws.w, backward ? ws.wf : nullptr, ws.r + c.dst0, part_r);
  if (backward && it.n_fix > 0)
    k_gat_fix_scalar<<<(unsigned)((it.n_fix + 3) / 4), 256, 0, ctx->stream>>>(it.fx_row, it.fx_part0, it.fx_nseg, it.n_fix, part_r,
                                                                             ws.r + c.dst0);
  tm->end();
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

int launch_src(ht_ctx* ctx, const GatPass& a, int nvec) {
  const unsigned nb = (unsigned)((a.n_items + 3) / 4);
  if (nvec <= 8) k_gat_src_g<8><<<nb, 256, 0, ctx->stream>>>(a);
  else if (nvec <= 16) k_gat_src_g<16><<<nb, 256, 0, ctx->stream>>>(a);
  else if (nvec <= 32) k_gat_src_g<32><<<nb, 256, 0, ctx->stream>>>(a);
  else if (nvec <= 64) k_gat_src<1><<<nb, 256, 0, ctx->stream>>>(a);
  else if (nvec <= 128) k_gat_src<2><<<nb, 256, 0, ctx->stream>>>(a);
  else k_gat_src<4><<<nb, 256, 0, ctx->stream>>>(a);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

int gat_fwd_impl(ht_ctx* ctx, const ht_graph* g, const ht_gat_desc* desc, const ht_tensor* H_in, const float* W,
                 const float* a_dst, const float* a_src, ht_tensor* H_out, ht_stats* local, Timer* tm, int layer) {
  HT_TRY(check_desc(ctx, desc));
  HT_TRY(check(ctx, g, desc, H_in, desc->d_in, "H_in"));
  HT_TRY(check(ctx, g, desc, H_out, desc->d_out, "H_out"));
  hipStream_t st = ctx->stream;
  GatWs ws{};
  Link lk(ctx, local, tm);
  const bool out_host = on_host(H_out);
  if (on_host(H_in) || out_host) HT_TRY(lk.fork());
  HT_TRY(prepare(ctx, g, desc, H_in, W, a_dst, a_src, false, &ws, local, tm, &lk));
  float* obuf[2] = {nullptr, nullptr};
  hipEvent_t ev_ofree[2] = {nullptr, nullptr};
  if (out_host) {
    const int64_t rows = std::max<int64_t>(g->max_ndst, 1);
    HT_TRY(ht_scratch(ctx, HT_S_LINK1, (size_t)rows * H_out->ld * 4 * 2, (void**)&obuf[0]));
    obuf[1] = obuf[0] + rows * H_out->ld;
  }
  int q = 0;
  for (int j = 0; j < g->n; ++j) {
    const ChunkMeta& c = g->chunks[j];
    if (c.dst1 == c.dst0) continue;
    const int b = q++ & 1;
    HT_TRY(softmax_chunk(ctx, g, c, desc, ws, local, tm, false));
    float* partial = nullptr;
    if (c.fwd.n_part > 0) HT_TRY(ht_scratch(ctx, HT_S_SPART, (size_t)g->max_fpart * H_out->ld * 4, (void**)&partial));
    SpmmArgs a{};
    a.it_row = c.fwd.row; a.it_e0 = c.fwd.e0; a.it_len = c.fwd.len; a.it_part = c.fwd.part; a.n_items = c.fwd.n_items;
    a.fx_row = c.fwd.fx_row; a.fx_part0 = c.fwd.fx_part0; a.fx_nseg = c.fwd.fx_nseg; a.n_fix = c.fwd.n_fix;
    a.n_edges = g->merged ? c.nu : c.nnz;
    a.idx = g->merged ? g->ucol.p + c.ue0 : g->col.p + c.e0;
    a.w_edge = ws.w;
    a.src = ws.T; a.src_ld = ws.ld_t; a.d = desc->d_out;
    a.out = out_host ? obuf[b] : H_out->ptr + c.dst0 * H_out->ld; a.out_ld = H_out->ld;
    a.accumulate = 0;
    a.relu = desc->act == HT_ACT_RELU;
    a.partial = partial;
    a.tm = tm;
    a.t_items = &local->t_agg_fwd_layer_ms[layer < HT_MAX_LAYERS ? layer : HT_MAX_LAYERS - 1];
    a.t_fix = &local->t_agg_fix_ms;
    if (out_host) {
      HT_TRY(lk.wait(st, ev_ofree[b]));
      // rows without an in-edge have no work item: their output is zero
      HT_TRY(ht_fill_zero(ctx, st, obuf[b], (size_t)(c.dst1 - c.dst0) * H_out->ld * 4));
    }
    HT_TRY(ht_spmm_launch(ctx, st, a));
    if (out_host) {
      hipEvent_t ev_done = nullptr;
      HT_TRY(lk.rec(st, &ev_done));
      HT_TRY(lk.wait(lk.s_out, ev_done));
      HT_TRY(lk.copy(lk.s_out, H_out->ptr + c.dst0 * H_out->ld, obuf[b], (size_t)(c.dst1 - c.dst0) * H_out->ld * 4, true));
      HT_TRY(lk.rec(lk.s_out, &ev_ofree[b]));
      lk.last_out = ev_ofree[b];
    }
    local->n_spmm_fwd += 1;
    local->n_agg_fwd_layer[layer < HT_MAX_LAYERS ? layer : HT_MAX_LAYERS - 1] += 1;
    local->edges += c.nnz;
  }
  if (lk.used) HT_TRY(lk.join());
  return HT_OK;
}

int gat_bwd_impl(ht_ctx* ctx, const ht_graph* g, const ht_gat_desc* desc, const ht_tensor* H_in, const float* W,
                 const float* a_dst, const float* a_src, const ht_tensor* H_out, const ht_tensor* dH_out,
                 ht_tensor* dH_in, float* dW, float* da_dst, float* da_src, ht_stats* local, Timer* tm,
                 bool dhin_is_zero) {
  HT_TRY(check_desc(ctx, desc));
  HT_TRY(check(ctx, g, desc, H_in, desc->d_in, "H_in"));
  HT_TRY(check(ctx, g, desc, H_out, desc->d_out, "H_out"));
  HT_TRY(check(ctx, g, desc, dH_out, desc->d_out, "dH_out"));
  if (dH_in) HT_TRY(check(ctx, g, desc, dH_in, desc->d_in, "dH_in"));
  hipStream_t st = ctx->stream;
  GatWs ws{};
  Link lk(ctx, local, tm);
  const bool hin_host = on_host(H_in), hout_host = on_host(H_out), dho_host = on_host(dH_out), dhi_host = on_host(dH_in);
  if (hin_host || hout_host || dho_host || dhi_host) HT_TRY(lk.fork());
  HT_TRY(prepare(ctx, g, desc, H_in, W, a_dst, a_src, true, &ws, local, tm, &lk));
  const int d = desc->d_out;
  const int nvec = (d + 3) / 4;
  const int sc_col = (int)ws.ld_t;              // the scalar column block sits behind the padded data columns
  const int64_t ld_dt = ws.ld_t + 4;
  const int64_t mx = std::max<int64_t>(g->max_ndst, 1);
  float *dT = nullptr, *dz = nullptr, *Q = nullptr, *da4 = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_TFULL2, (size_t)std::max<int64_t>(g->V, 1) * ld_dt * 4, (void**)&dT));
  HT_TRY(ht_scratch(ctx, HT_S_DZCHUNK, (size_t)mx * ws.ld_t * 4, (void**)&dz));
  HT_TRY(ht_scratch(ctx, HT_S_ACHUNK, (size_t)mx * ws.ld_t * 4, (void**)&Q));
  HT_TRY(ht_scratch(ctx, HT_S_MISC, (size_t)d * 16, (void**)&da4));
  HT_TRY(ht_fill_zero(ctx, st, dT, (size_t)g->V * ld_dt * 4));
  // host-resident H_out / dH_out: the rows of the next chunk are staged while this one computes
  float* hbuf[2] = {nullptr, nullptr};
  float* gbuf[2] = {nullptr, nullptr};
  hipEvent_t ev_in[2] = {nullptr, nullptr}, ev_free[2] = {nullptr, nullptr};
  if (hout_host) {
    HT_TRY(ht_scratch(ctx, HT_S_LINK1, (size_t)mx * H_out->ld * 4 * 2, (void**)&hbuf[0]));
    hbuf[1] = hbuf[0] + mx * H_out->ld;
  }
  if (dho_host) {
    HT_TRY(ht_scratch(ctx, HT_S_LINK2, (size_t)mx * dH_out->ld * 4 * 2, (void**)&gbuf[0]));
    gbuf[1] = gbuf[0] + mx * dH_out->ld;
  }
  std::vector<int> live;
  for (int j = 0; j < g->n; ++j)
    if (g->chunks[j].dst1 > g->chunks[j].dst0) live.push_back(j);
  auto stage_chunk = [&](size_t i) -> int {
    if (!(hout_host || dho_host) || i >= live.size()) return HT_OK;
    const ChunkMeta& c = g->chunks[live[i]];
    const int b = (int)(i & 1);
    const int64_t nd = c.dst1 - c.dst0;
    HT_TRY(lk.wait(lk.s_in, ev_free[b]));
    if (hout_host) HT_TRY(lk.copy(lk.s_in, hbuf[b], H_out->ptr + c.dst0 * H_out->ld, (size_t)nd * H_out->ld * 4, false));
    if (dho_host) HT_TRY(lk.copy(lk.s_in, gbuf[b], dH_out->ptr + c.dst0 * dH_out->ld, (size_t)nd * dH_out->ld * 4, false));
    return lk.rec(lk.s_in, &ev_in[b]);
  };
  HT_TRY(stage_chunk(0));
  for (size_t i = 0; i < live.size(); ++i) {
    const ChunkMeta& c = g->chunks[live[i]];
    const int64_t ndst = c.dst1 - c.dst0;
    const int b = (int)(i & 1);
    HT_TRY(stage_chunk(i + 1));
    HT_TRY(softmax_chunk(ctx, g, c, desc, ws, local, tm, true));
    if (hout_host || dho_host) HT_TRY(lk.wait(st, ev_in[b]));
    k_gat_dz<<<(unsigned)((ndst + 3) / 4), 256, 0, st>>>(dho_host ? gbuf[b] : dH_out->ptr + c.dst0 * dH_out->ld, dH_out->ld,
                                                          hout_host ? hbuf[b] : H_out->ptr + c.dst0 * H_out->ld, H_out->ld,
                                                          desc->act == HT_ACT_RELU, ndst, d, dz, ws.ld_t, ws.S, ws.p + c.dst0,
                                                          ws.m + c.dst0, ws.zinv + c.dst0, ws.d4);
    HT_LAUNCH_CHECK(ctx);
    if (hout_host || dho_host) HT_TRY(lk.rec(st, &ev_free[b]));   // the staged rows have been consumed
    GatPass a{};
    a.d = d; a.p = ws.p; a.q = ws.q; a.m = ws.m; a.zinv = ws.zinv; a.S = ws.S; a.d4 = ws.d4; a.dst0 = c.dst0; a.slope = desc->slope;
    // destination pass: Q_v = sum_e w_e f_e t_u through the aggregation kernel, then dp_v = dz_v . Q_v - S_v r_v
    tm->begin(&local->t_gat_dst_ms);
    {
      float* fpart = nullptr;
      if (c.fwd.n_part > 0) HT_TRY(ht_scratch(ctx, HT_S_SPART, (size_t)g->max_fpart * ws.ld_t * 4, (void**)&fpart));
      SpmmArgs q{};
      q.it_row = c.fwd.row; q.it_e0 = c.fwd.e0; q.it_len = c.fwd.len; q.it_part = c.fwd.part; q.n_items = c.fwd.n_items;
      q.fx_row = c.fwd.fx_row; q.fx_part0 = c.fwd.fx_part0; q.fx_nseg = c.fwd.fx_nseg; q.n_fix = c.fwd.n_fix;
      q.n_edges = g->merged ? c.nu : c.nnz;
      q.idx = g->merged ? g->ucol.p + c.ue0 : g->col.p + c.e0;
      q.w_edge = ws.wf;
      q.src = ws.T; q.src_ld = ws.ld_t; q.d = d;
      q.out = Q; q.out_ld = ws.ld_t;
      q.accumulate = 0;
      q.partial = fpart;
      HT_TRY(ht_fill_zero(ctx, st, Q, (size_t)ndst * ws.ld_t * 4));     // rows without an in-edge have no item
      HT_TRY(ht_spmm_launch(ctx, st, q));
      k_gat_dp<<<(unsigned)((ndst + 3) / 4), 256, 0, st>>>(dz, Q, ws.ld_t, d, ws.S, ws.r + c.dst0, ndst, ws.dp + c.dst0);
      HT_LAUNCH_CHECK(ctx);
    }
    tm->end();
    // source pass
    float* partial = nullptr;
    if (c.bwd.n_part > 0) HT_TRY(ht_scratch(ctx, HT_S_SPART, (size_t)g->max_bpart * ld_dt * 4, (void**)&partial));
    a.it_row = c.bwd.row; a.it_e0 = c.bwd.e0; a.it_len = c.bwd.len; a.it_part = c.bwd.part; a.n_items = c.bwd.n_items;
    a.idx = g->merged ? g->usdst.p + c.ue0 : g->sdst.p + c.e0;
    a.mult = g->merged ? g->umult_bwd.p + c.ue0 : nullptr;
    a.mat = dz; a.mat_ld = ws.ld_t;
    a.own = ws.T; a.own_ld = ws.ld_t; a.own_idx = g->nbr.p + c.nbr_off;
    a.out = dT; a.out_ld = ld_dt; a.out_idx = g->nbr.p + c.nbr_off;
    a.partial = partial; a.sc_col = sc_col;
    tm->begin(&local->t_gat_src_ms);
    if (a.n_items > 0) HT_TRY(launch_src(ctx, a, nvec));
    if (c.bwd.n_fix > 0) {
      SpmmArgs f{};
      f.fx_row = c.bwd.fx_row; f.fx_part0 = c.bwd.fx_part0; f.fx_nseg = c.bwd.fx_nseg; f.n_fix = c.bwd.n_fix;
      f.d = sc_col + 4;
      f.out = dT; f.out_ld = ld_dt; f.out_idx = g->nbr.p + c.nbr_off;
      f.accumulate = 1;
      f.partial = partial;
      HT_TRY(ht_spmm_fix_launch(ctx, st, f));
    }
    tm->end();
    local->n_spmm_bwd += 2;
    local->edges += 2 * c.nnz;
  }
  if (g->V > 0) {
    k_gat_finish<<<(unsigned)std::min<int64_t>((g->V + 3) / 4, 1 << 22), 256, 0, st>>>(dT, ld_dt, d, sc_col, ws.dp, a_dst, a_src, g->V, ws.pq4);
    HT_LAUNCH_CHECK(ctx);
  }
  // da = T^T [dp dq 0 0]; dW = H^T dt; dH += dt W^T, in row blocks; host-resident H_in / dH_in blocks go
  // through staging pairs (dH_in: in, add, out; straight out when it is known to hold zeros)
  const int64_t step = (hin_host || dhi_host) ? ctx->link_block_rows : BLOCK_HBM;
  const int64_t brows = std::min<int64_t>(step, std::max<int64_t>(g->V, 1));
  float* sH[2] = {nullptr, nullptr};
  float* sD[2] = {nullptr, nullptr};
  hipEvent_t ev_bfree[2] = {nullptr, nullptr}, ev_dout[2] = {nullptr, nullptr};
  if (hin_host) {
    HT_TRY(ht_scratch(ctx, HT_S_LINK0, (size_t)brows * H_in->ld * 4 * 2, (void**)&sH[0]));
    sH[1] = sH[0] + brows * H_in->ld;
  }
  if (dhi_host) {
    // (the chunk loop is over: its staging pair is free)
    HT_TRY(ht_scratch(ctx, HT_S_LINK1, (size_t)brows * dH_in->ld * 4 * 2, (void**)&sD[0]));
    sD[1] = sD[0] + brows * dH_in->ld;
  }
  // the staging memory was used by the earlier phases: copies into it start behind their last reader
  if (lk.used) HT_TRY(lk.fork());
  bool first = true;
  int k = 0;
  for (int64_t r0 = 0; r0 < g->V; r0 += step, ++k) {
    const int64_t nr = std::min(step, g->V - r0);
    const int b = k & 1;
    const float* h_rows = H_in->ptr + r0 * H_in->ld;
    float* dh_rows = dH_in ? dH_in->ptr + r0 * dH_in->ld : nullptr;
    const bool dh_add = !(dhi_host && dhin_is_zero);
    if (hin_host || dhi_host) {
      hipEvent_t ev_bin = nullptr;
      HT_TRY(lk.wait(lk.s_in, ev_bfree[b]));
      HT_TRY(lk.wait(lk.s_in, ev_dout[b]));
      if (hin_host) {
        HT_TRY(lk.copy(lk.s_in, sH[b], h_rows, (size_t)nr * H_in->ld * 4, false));
        h_rows = sH[b];
      }
      if (dhi_host) {
        if (dh_add) HT_TRY(lk.copy(lk.s_in, sD[b], dh_rows, (size_t)nr * dH_in->ld * 4, false));
        else HT_TRY(lk.wait(st, ev_dout[b]));      // the compute stream overwrites the block
        dh_rows = sD[b];
      }
      HT_TRY(lk.rec(lk.s_in, &ev_bin));
      HT_TRY(lk.wait(st, ev_bin));
    }
    tm->begin(&local->t_gemm_ms);
    HT_TRY(ht_gemm_tn(ctx, st, ws.T + r0 * ws.ld_t, ws.ld_t, ws.pq4 + r0 * 4, 4, da4, nr, d, 4, first ? 0 : 1));
    HT_TRY(ht_gemm_tn(ctx, st, h_rows, H_in->ld, dT + r0 * ld_dt, ld_dt, dW, nr, desc->d_in, d, first ? 0 : 1));
    if (dH_in)
      HT_TRY(ht_gemm_nt(ctx, st, dT + r0 * ld_dt, ld_dt, W, dh_rows, dH_in->ld, nr, d, desc->d_in, dh_add ? 1 : 0));
    tm->end();
    if (hin_host || dhi_host) HT_TRY(lk.rec(st, &ev_bfree[b]));
    if (dhi_host) {
      HT_TRY(lk.wait(lk.s_out, ev_bfree[b]));
      HT_TRY(lk.copy(lk.s_out, dH_in->ptr + r0 * dH_in->ld, sD[b], (size_t)nr * dH_in->ld * 4, true));
      HT_TRY(lk.rec(lk.s_out, &ev_dout[b]));
      lk.last_out = ev_dout[b];
    }
    local->n_gemm += 3;
    local->gemm_flops += 4.0 * nr * desc->d_in * d;
    first = false;
  }
  if (first) {
    HT_TRY(ht_fill_zero(ctx, st, dW, (size_t)desc->d_in * d * 4));
    HT_TRY(ht_fill_zero(ctx, st, da4, (size_t)d * 16));
  }
  k_gat_split<<<(unsigned)((d + 255) / 256), 256, 0, st>>>(da4, d, da_dst, da_src);
  HT_LAUNCH_CHECK(ctx);
  if (lk.used) HT_TRY(lk.join());
  return HT_OK;
}

}  // namespace

extern "C" {

int ht_gat_layer_fwd(ht_ctx* ctx, const ht_graph* g, const ht_gat_desc* desc, const ht_tensor* H_in, const float* W,
                     const float* a_dst, const float* a_src, ht_tensor* H_out, ht_stats* stats) {
  if (!ctx) return HT_EINVAL;
  if (!g || !desc || !H_in || !H_out || !W || !a_dst || !a_src) return ht_set_err(ctx, HT_EINVAL, "ht_gat_layer_fwd: null argument");
  if (g->ctx != ctx) return ht_set_err(ctx, HT_ESTATE, "graph belongs to another context");
  HT_HIP(ctx, hipSetDevice(ctx->device));
  auto t0 = std::chrono::steady_clock::now();
  ht_stats local{};
  Timer tm(ctx, ctx->stream, stats != nullptr);
  int rc = gat_fwd_impl(ctx, g, desc, H_in, W, a_dst, a_src, H_out, &local, &tm, 0);
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (rc == HT_OK && e == hipSuccess) rc = tm.resolve();
  ctx->ev_next = 0;
  if (rc != HT_OK) return rc;
  HT_HIP(ctx, e);
  if (stats) {
    local.t_total_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    *stats = local;
  }
  return HT_OK;
}

int ht_gat_layer_bwd(ht_ctx* ctx, const ht_graph* g, const ht_gat_desc* desc, const ht_tensor* H_in, const float* W,
                     const float* a_dst, const float* a_src, const ht_tensor* H_out, const ht_tensor* dH_out,
                     ht_tensor* dH_in, float* dW, float* da_dst, float* da_src, ht_stats* stats) {
  if (!ctx) return HT_EINVAL;
  if (!g || !desc || !H_in || !H_out || !dH_out || !W || !a_dst || !a_src || !dW || !da_dst || !da_src)
    return ht_set_err(ctx, HT_EINVAL, "ht_gat_layer_bwd: null argument");
  if (g->ctx != ctx) return ht_set_err(ctx, HT_ESTATE, "graph belongs to another context");
  HT_HIP(ctx, hipSetDevice(ctx->device));
  auto t0 = std::chrono::steady_clock::now();
  ht_stats local{};
  Timer tm(ctx, ctx->stream, stats != nullptr);
  int rc = gat_bwd_impl(ctx, g, desc, H_in, W, a_dst, a_src, H_out, dH_out, dH_in, dW, da_dst, da_src, &local, &tm, false);
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (rc == HT_OK && e == hipSuccess) rc = tm.resolve();
  ctx->ev_next = 0;
  if (rc != HT_OK) return rc;
  HT_HIP(ctx, e);
  if (stats) {
    local.t_total_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    *stats = local;
  }
  return HT_OK;
}

// Alg. 1 with GAT layers: forward over the layers (only the layer outputs are kept), softmax
// cross-entropy on the labelled vertices, backward layer by layer with every layer's
// intermediates recomputed from its input, SGD step on W^l and a^l.  With res_h = HT_RES_HOST
// the layer outputs h^1..h^{L-1} and their gradients live in pinned host memory (Alg. 1 keeps
// h^l and grad h^l on the CPU); the logits h^L and their gradient stay in HBM for the loss.
int ht_gat_epoch(ht_ctx* ctx, const ht_graph* g, const ht_gat_model* model, const ht_tensor* X, const int32_t* labels,
                 float* loss_out, ht_stats* stats) {
  if (!ctx) return HT_EINVAL;
  if (!g || !model || !X || !labels || !loss_out) return ht_set_err(ctx, HT_EINVAL, "ht_gat_epoch: null argument");
  if (g->ctx != ctx) return ht_set_err(ctx, HT_ESTATE, "graph belongs to another context");
  const int L = model->n_layers;
  if (L < 1 || L > HT_MAX_LAYERS || !model->dims || !model->W || !model->a_dst || !model->a_src)
    return ht_set_err(ctx, HT_EINVAL, "ht_gat_epoch: bad model");
  for (int l = 0; l <= L; ++l)
    if (model->dims[l] <= 0) return ht_set_err(ctx, HT_ESHAPE, "ht_gat_epoch: layer widths must be positive");
  for (int l = 0; l < L; ++l)
    if (!model->W[l] || !model->a_dst[l] || !model->a_src[l]) return ht_set_err(ctx, HT_EINVAL, "ht_gat_epoch: null parameter of layer %d", l);
  HT_HIP(ctx, hipSetDevice(ctx->device));
  auto t0 = std::chrono::steady_clock::now();
  hipStream_t st = ctx->stream;
  const int64_t V = g->V;
  if (model->res_h != HT_RES_AUTO && model->res_h != HT_RES_HBM && model->res_h != HT_RES_HOST)
    return ht_set_err(ctx, HT_EINVAL, "ht_gat_epoch: unknown residency %d", model->res_h);
  const bool h_host = model->res_h == HT_RES_HOST;
  auto in_hbm = [&](int l) { return !h_host || l == L; };
  // workspace: h^1..h^L, grad h^1..grad h^L (HBM or pinned host), then dW^l, da_dst^l, da_src^l, loss
  size_t floats = 64 + 64 * (size_t)L, hfloats = 64 * (size_t)L;
  for (int l = 1; l <= L; ++l)
    (in_hbm(l) ? floats : hfloats) += 2 * ((size_t)std::max<int64_t>(V, 1) * ht_row_pitch(model->dims[l], in_hbm(l)) + 32);
  for (int l = 0; l < L; ++l) floats += (size_t)model->dims[l] * model->dims[l + 1] + 2 * (size_t)model->dims[l + 1] + 96;
  float* base = nullptr;
  float* hbase = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_GATWS, floats * 4, (void**)&base));
  if (h_host && L > 1) HT_TRY(ht_host_scratch(ctx, 2, hfloats * 4, (void**)&hbase));
  std::vector<ht_tensor> h(L + 1), gh(L + 1);
  std::vector<float*> dW(L), dad(L), das(L);
  float* cur = base;
  float* hcur = hbase;
  auto take = [&](size_t n) { float* p = cur; cur += (n + 31) & ~(size_t)31; return p; };
  auto take_host = [&](size_t n) { float* p = hcur; hcur += (n + 31) & ~(size_t)31; return p; };
  for (int l = 1; l <= L; ++l) {
    const bool dev = in_hbm(l);
    const int64_t ld = ht_row_pitch(model->dims[l], dev);
    const size_t n = (size_t)std::max<int64_t>(V, 1) * ld;
    const int loc = dev ? HT_LOC_DEVICE : HT_LOC_HOST_PINNED;
    h[l] = ht_tensor{dev ? take(n) : take_host(n), V, model->dims[l], ld, loc};
    gh[l] = ht_tensor{dev ? take(n) : take_host(n), V, model->dims[l], ld, loc};
  }
  for (int l = 0; l < L; ++l) {
    dW[l] = take((size_t)model->dims[l] * model->dims[l + 1]);
    dad[l] = take(model->dims[l + 1]);
    das[l] = take(model->dims[l + 1]);
  }
  float* loss_dev = take(4);
  ht_stats local{};
  Timer tm(ctx, st, stats != nullptr);
  auto fail = [&](int rc) {
    (void)hipStreamSynchronize(st);
    (void)hipStreamSynchronize(ctx->side[0]);
    (void)hipStreamSynchronize(ctx->side[1]);
    ctx->ev_next = 0;
    return rc;
  };
  for (int l = 0; l < L; ++l) {
    ht_gat_desc d{model->dims[l], model->dims[l + 1], l < L - 1 ? HT_ACT_RELU : HT_ACT_NONE, model->slope};
    int rc = gat_fwd_impl(ctx, g, &d, l == 0 ? X : &h[l], model->W[l], model->a_dst[l], model->a_src[l], &h[l + 1], &local, &tm, l);
    if (rc != HT_OK) return fail(rc);
  }
  {
    tm.begin(&local.t_loss_ms);
    int rc = ht_softmax_ce(ctx, st, h[L].ptr, h[L].ld, labels, V, model->dims[L], gh[L].ptr, gh[L].ld, loss_dev);
    tm.end();
    if (rc != HT_OK) return fail(rc);
  }
  for (int l = L - 1; l >= 0; --l) {
    ht_gat_desc d{model->dims[l], model->dims[l + 1], l < L - 1 ? HT_ACT_RELU : HT_ACT_NONE, model->slope};
    if (l > 0 && gh[l].loc == HT_LOC_DEVICE) {   // (a host-resident gradient is written, not added to)
      int rc = ht_fill_zero(ctx, st, gh[l].ptr, (size_t)V * gh[l].ld * 4);
      if (rc != HT_OK) return fail(rc);
    }
    int rc = gat_bwd_impl(ctx, g, &d, l == 0 ? X : &h[l], model->W[l], model->a_dst[l], model->a_src[l], &h[l + 1], &gh[l + 1],
                          l > 0 ? &gh[l] : nullptr, dW[l], dad[l], das[l], &local, &tm, true);
    if (rc != HT_OK) return fail(rc);
  }
  for (int l = 0; l < L; ++l) {
    int rc = ht_sgd(ctx, st, model->W[l], dW[l], (int64_t)model->dims[l] * model->dims[l + 1], model->lr);
    if (rc == HT_OK) rc = ht_sgd(ctx, st, model->a_dst[l], dad[l], model->dims[l + 1], model->lr);
    if (rc == HT_OK) rc = ht_sgd(ctx, st, model->a_src[l], das[l], model->dims[l + 1], model->lr);
    if (rc != HT_OK) return fail(rc);
  }
  {
    hipError_t e = hipMemcpyAsync(loss_out, loss_dev, 4, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return fail(ht_set_err(ctx, HT_EHIP, "loss copy: %s", hipGetErrorString(e)));
  }
  {
    hipError_t e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(ht_set_err(ctx, HT_EHIP, "synchronize: %s", hipGetErrorString(e)));
    int rc = tm.resolve();
    ctx->ev_next = 0;
    if (rc != HT_OK) return rc;
  }
  if (stats) {
    for (int l = 0; l < HT_MAX_LAYERS; ++l) local.t_spmm_fwd_ms += local.t_agg_fwd_layer_ms[l];
    local.t_spmm_fwd_ms += local.t_agg_fix_ms;
    local.t_total_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    *stats = local;
  }
  return HT_OK;
}

}  // extern "C"

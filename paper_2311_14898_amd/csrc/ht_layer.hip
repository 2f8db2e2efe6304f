// Per-chunk layer step, forward and backward, and the epoch built from it.
//
//   forward  (Alg. 1, Alg. 2, Eq. 2): neighbour rows reach
//            the aggregation either in place (tensor in HBM) or through the
//            in-place neighbour buffer (reused rows stay, new rows are fetched
//            from HBM or pinned host memory); aggregate; linear + ReLU; rows
//            of a^l and h^{l+1} go to their homes.
//   backward (Alg. 1, Alg. 3, Sec. 2.3, Sec. 4.2): reload
//            the checkpoint, recompute the update stage, grad W, grad a,
//            aggregate backward by source; neighbour gradients accumulate in HBM
//            while their vertex stays buffered and leave to the gradient home
//            (CPU-side add when that home is host memory).
#include <algorithm>
#include <atomic>
#include <cstring>
#include <condition_variable>
#include <mutex>
#include <thread>

#include "ht_internal.h"

struct EpochWs {
  int64_t V = 0;
  std::vector<int32_t> dims;
  int res_h = 0, res_a = 0, res_g = 0;
  bool no_ckpt = false;              // pure recomputation: no a^l for any layer
  uint32_t upd_mask = 0;             // bit l: layer l runs update-first (no a^l is kept for it)
  std::vector<ht_tensor> h, a, gh;  // h[l] = h^l (l >= 1; h[0] unused), a[l], gh[l] = grad h^l (l >= 1)
  std::vector<float*> dW;
  std::vector<size_t> dev_bytes_of;  // for freeing
  std::vector<void*> dev_ptrs;
  std::vector<void*> host_ptrs;
  float* loss_dev = nullptr;
  const float* a0_of = nullptr;      // a[0] holds A_hat X for the X at this address (nullptr: not valid)
  uint64_t a0_graph = 0;             // ... and for the graph with this serial number
  // HIP graph of one epoch's stream work (all tensors in HBM): what it was captured for, and the
  // key of the last epoch that ran eagerly to the end (its scratch sizes are what the capture needs)
  std::vector<uintptr_t> graph_key, warm_key, bad_key;   // bad_key: a capture of this key failed, it stays eager
  hipGraphExec_t graph_exec = nullptr;
};

namespace {

__global__ void k_noop() {}

int check_tensor(ht_ctx* ctx, const ht_tensor* t, int64_t rows, int32_t cols, const char* name) {
  if (!t || !t->ptr) return ht_set_err(ctx, HT_EINVAL, "%s: null tensor", name);
  if (t->rows != rows || t->cols != cols)
    return ht_set_err(ctx, HT_ESHAPE, "%s: shape [%lld x %d], expected [%lld x %d]", name, (long long)t->rows, t->cols,
                      (long long)rows, cols);
  if (t->ld < t->cols || (t->ld & 3))
    return ht_set_err(ctx, HT_ESHAPE, "%s: row pitch %lld must be >= cols and a multiple of 4", name, (long long)t->ld);
  if (t->loc != HT_LOC_DEVICE && t->loc != HT_LOC_HOST_PINNED)
    return ht_set_err(ctx, HT_ESHAPE, "%s: unknown location %d", name, t->loc);
  if ((uintptr_t)t->ptr & 15) return ht_set_err(ctx, HT_ESHAPE, "%s: base pointer must be 16-byte aligned", name);
  return HT_OK;
}

// Pointer the GPU can dereference.
int gpu_ptr(ht_ctx* ctx, const ht_tensor* t, float** out) {
  if (t->loc == HT_LOC_DEVICE) {
    *out = t->ptr;
    return HT_OK;
  }
  void* d = nullptr;
  hipError_t e = hipHostGetDevicePointer(&d, t->ptr, 0);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return ht_set_err(ctx, HT_ESHAPE, "host tensor is not page-locked / GPU-addressable: %s", hipGetErrorString(e));
  }
  *out = (float*)d;
  return HT_OK;
}

int host_threads(ht_ctx* ctx) {
  if (ctx->n_threads <= 0) {
    unsigned hc = std::thread::hardware_concurrency();
    ctx->n_threads = (int)std::min<unsigned>(hc ? hc : 4u, 16u);
  }
  return ctx->n_threads;
}

// grad[ids[k]] += rows[k] on the host cores (Alg. 3); ids are unique.
void cpu_accumulate(ht_ctx* ctx, float* grad, int64_t ld, const int32_t* ids, const float* rows, int64_t rows_ld,
                    int64_t n, int d) {
  const int nt = (int)std::min<int64_t>(host_threads(ctx), std::max<int64_t>(1, n / 256));
  auto work = [&](int64_t k0, int64_t k1) {
    for (int64_t k = k0; k < k1; ++k) {
      float* g = grad + (int64_t)ids[k] * ld;
      const float* r = rows + k * rows_ld;
      for (int c = 0; c < d; ++c) g[c] += r[c];
    }
  };
  if (nt <= 1) {
    work(0, n);
    return;
  }
  std::vector<std::thread> th;
  const int64_t per = (n + nt - 1) / nt;
  for (int t = 0; t < nt; ++t) {
    const int64_t k0 = t * per, k1 = std::min<int64_t>(n, k0 + per);
    if (k0 < k1) th.emplace_back(work, k0, k1);
  }
  for (auto& t : th) t.join();
}

// Destination rows from which the dense work of neighbouring chunks is no longer merged into one launch.
constexpr int64_t HT_DENSE_MERGE_ROWS = 32768;

struct Run {
  ht_ctx* ctx;
  const ht_graph* g;
  Timer tm;
  ht_stats* st;  // never null inside (a local one is used when the caller passes none)
  int layer = 0; // index into the per-layer statistics
  bool dhin_is_zero = false;  // the caller guarantees dH_in holds zeros (lets leaving rows be stored, not added)
  Run(ht_ctx* c, const ht_graph* gr, ht_stats* s, bool timed) : ctx(c), g(gr), tm(c, c->stream, timed), st(s) {}
};

double spmm_alg_bytes(const ChunkMeta& c, int d) {
  const double nd = (double)(c.dst1 - c.dst0);
  return 4.0 * c.nnz + 8.0 * nd + 4.0 * d * (double)c.nsrc + 4.0 * d * nd + 4.0 * ((double)c.nsrc + nd);
}

// Streams of the per-chunk pipeline: compute on the context's stream, neighbour
// gather / H2D row copies on side[0], D2H row copies on side[1], host functions
// (CPU-side gradient accumulation) on side[2].  Stages are ordered by events.
struct Pipe {
  ht_ctx* ctx;
  hipStream_t s_c, s_in, s_out, s_host;
  bool used_in = false, used_out = false, used_host = false;
  explicit Pipe(ht_ctx* c) : ctx(c), s_c(c->stream), s_in(c->side[0]), s_out(c->side[1]), s_host(c->side[2]) {}
  // A failed call must not leave side-stream work that refers to the caller's locals.
  ~Pipe() {
    if (used_in) (void)hipStreamSynchronize(s_in);
    if (used_out) (void)hipStreamSynchronize(s_out);
    if (used_host) (void)hipStreamSynchronize(s_host);
  }
  int rec(hipStream_t s, hipEvent_t* out) {
    hipEvent_t e = ht_event(ctx);
    if (!e) return ht_set_err(ctx, HT_EHIP, "hipEventCreate failed");
    HT_HIP(ctx, hipEventRecord(e, s));
    *out = e;
    return HT_OK;
  }
  int wait(hipStream_t s, hipEvent_t e) {
    if (!e) return HT_OK;
    HT_HIP(ctx, hipStreamWaitEvent(s, e, 0));
    return HT_OK;
  }
  // Link traffic and the aggregation kernels are kept apart in time: run together both slow
  // down several-fold on this GPU (measured), while the dense transforms and the host-side
  // adds overlap with link traffic at no cost.
  hipEvent_t last_in = nullptr, last_out = nullptr, quiet = nullptr;
  bool fence = false;
  int link_begin(hipStream_t s) { return fence ? wait(s, quiet) : HT_OK; }
  int link_end(hipStream_t s) {
    if (!fence) return HT_OK;
    return rec(s, s == s_in ? &last_in : &last_out);
  }
  int agg_begin() {
    if (!fence) return HT_OK;
    HT_TRY(wait(s_c, last_in));
    return wait(s_c, last_out);
  }
  int agg_end() { return fence ? rec(s_c, &quiet) : HT_OK; }
};

// Rows of N_j \ N_{j-1} from H_in (HBM or pinned host, read in place by the
// kernel) into their positions of the in-place neighbour buffer, scaled by s_u
// on the way (Alg. 2).
int gather_chunk(Run& R, int j, const ht_tensor* H_in, const float* Hin, int d, float* nbuf, hipStream_t st) {
  const ht_graph* g = R.g;
  const ChunkMeta& c = g->chunks[j];
  const int id = R.tm.begin_on(&R.st->t_gather_ms, st);
  HT_TRY(ht_gather_rows(R.ctx, st, Hin, H_in->ld, g->load.p + c.load_off, nbuf, H_in->ld, g->load_slot.p + c.load_off,
                        c.n_load, d, g->s.p, H_in->loc == HT_LOC_HOST_PINNED ? R.ctx->gather_blocks : 0));
  R.tm.end_id(id);
  R.st->rows_loaded += c.n_load;
  R.st->rows_reused += c.n_reuse;
  if (H_in->loc == HT_LOC_HOST_PINNED) R.st->bytes_h2d += (int64_t)c.n_load * d * 4;
  R.st->bytes_h2d_nodedup += (int64_t)c.nsrc * d * 4;
  return HT_OK;
}

// Aggregate of chunk j into out rows [0, ndst) (pitch out_ld) on the compute
// stream.  src/src_ld: H_in read in place, or the neighbour buffer (rows already
// scaled by s_u, indexed by buffer position).
int spmm_chunk(Run& R, int j, bool buffer, const float* src, int64_t src_ld, int d, float* out, int64_t out_ld) {
  ht_ctx* ctx = R.ctx;
  const ht_graph* g = R.g;
  const ChunkMeta& c = g->chunks[j];
  hipStream_t st = ctx->stream;
  float* partial = nullptr;
  if (c.fwd.n_part > 0) HT_TRY(ht_scratch(ctx, HT_S_SPART, (size_t)g->max_fpart * out_ld * 4, (void**)&partial));
  SpmmArgs a{};
  a.it_row = c.fwd.row; a.it_e0 = c.fwd.e0; a.it_len = c.fwd.len; a.it_part = c.fwd.part; a.n_items = c.fwd.n_items;
  a.n_edges = c.nnz;
  a.fx_row = c.fwd.fx_row; a.fx_part0 = c.fwd.fx_part0; a.fx_nseg = c.fwd.fx_nseg; a.n_fix = c.fwd.n_fix;
  if (g->merged) {
    a.idx = (buffer ? g->ucol_slot.p : g->ucol.p) + c.ue0;
    a.w_edge = (buffer ? g->umult.p : g->uw_fwd.p) + c.ue0;
    a.n_edges = c.nu;
  } else {
    a.idx = (buffer ? g->col_slot.p : g->col.p) + c.e0;
    a.ew = buffer ? nullptr : g->s.p;
  }
  a.src = src;
  a.src_ld = src_ld;
  a.d = d;
  a.out = out; a.out_ld = out_ld; a.out_idx = nullptr;
  a.post = g->s.p + c.dst0; a.post_idx = nullptr;
  a.accumulate = 0;
  a.partial = partial;
  a.max_slabs = ctx->slabs_fwd;
  const int li = R.layer < HT_MAX_LAYERS ? R.layer : HT_MAX_LAYERS - 1;
  a.tm = &R.tm;
  a.t_items = &R.st->t_agg_fwd_layer_ms[li];
  a.t_fix = &R.st->t_agg_fix_ms;
  HT_TRY(ht_spmm_launch(ctx, st, a));
  R.st->n_spmm_fwd += 1;
  R.st->n_agg_fwd_layer[li] += 1;
  R.st->edges += c.nnz;
  R.st->spmm_fwd_alg_bytes += spmm_alg_bytes(c, d);
  R.st->agg_fwd_layer_alg_bytes[li] += spmm_alg_bytes(c, d);
  return HT_OK;
}

int resolve_gather(ht_ctx* ctx, int mode, const ht_tensor* t, bool* buffer) {
  if (mode == HT_GATHER_AUTO) *buffer = t->loc != HT_LOC_DEVICE;
  else if (mode == HT_GATHER_DIRECT) {
    if (t->loc != HT_LOC_DEVICE) return ht_set_err(ctx, HT_ESHAPE, "direct gather needs the tensor in HBM");
    *buffer = false;
  } else if (mode == HT_GATHER_BUFFER) *buffer = true;
  else return ht_set_err(ctx, HT_EINVAL, "unknown gather mode %d", mode);
  return HT_OK;
}

// Contiguous row range between HBM and pinned host memory.  host_gpu is the
// GPU-usable alias of the host side (dst for D2H, src for H2D).
int copy_rows(Run& R, hipStream_t st, void* dst, const void* src, size_t bytes, hipMemcpyKind kind) {
  if (bytes == 0) return HT_OK;
  ht_ctx* ctx = R.ctx;
  const int id = R.tm.begin_on(&R.st->t_copy_ms, st);
  const int lm = ctx->link_memcpy;   // 1: both directions, 2: device to host only, 3: host to device only
  if (lm == 1 || (lm == 2 && kind == hipMemcpyDeviceToHost) || (lm == 3 && kind == hipMemcpyHostToDevice)) {
    HT_HIP(ctx, hipMemcpyAsync(dst, src, bytes, kind, st));
  } else {
    void* d = dst;
    const void* s = src;
    void* mapped = nullptr;
    if (kind == hipMemcpyDeviceToHost) {
      HT_HIP(ctx, hipHostGetDevicePointer(&mapped, dst, 0));
      d = mapped;
    } else if (kind == hipMemcpyHostToDevice) {
      HT_HIP(ctx, hipHostGetDevicePointer(&mapped, const_cast<void*>(src), 0));
      s = mapped;
    }
    HT_TRY(ht_copy_link(ctx, st, d, s, bytes, ctx->link_blocks));
  }
  R.tm.end_id(id);
  if (kind == hipMemcpyHostToDevice) R.st->bytes_h2d += (int64_t)bytes;
  if (kind == hipMemcpyDeviceToHost) R.st->bytes_d2h += (int64_t)bytes;
  return HT_OK;
}

int layer_fwd_impl(Run& R, const ht_layer_desc* desc, const ht_tensor* H_in, const float* W, ht_tensor* H_out,
                   ht_tensor* A_ckpt) {
  ht_ctx* ctx = R.ctx;
  const ht_graph* g = R.g;
  const int di = desc->d_in, dn = desc->d_out;
  HT_TRY(check_tensor(ctx, H_in, g->V, di, "H_in"));
  HT_TRY(check_tensor(ctx, H_out, g->V, dn, "H_out"));
  if (A_ckpt) HT_TRY(check_tensor(ctx, A_ckpt, g->V, di, "A_ckpt"));
  if (!W) return ht_set_err(ctx, HT_EINVAL, "W is null");
  bool buffer = false;
  HT_TRY(resolve_gather(ctx, desc->gather_mode, H_in, &buffer));
  float* Hin = nullptr;
  HT_TRY(gpu_ptr(ctx, H_in, &Hin));

  const bool a_dev = A_ckpt && A_ckpt->loc == HT_LOC_DEVICE;
  const bool a_host = A_ckpt && !a_dev;
  const bool h_dev = H_out->loc == HT_LOC_DEVICE;
  const bool staged = a_host || !h_dev;                              // some rows leave through the output stream
  const bool side_in = buffer && H_in->loc == HT_LOC_HOST_PINNED;    // gather runs beside the compute
  const int64_t a_ld = A_ckpt ? A_ckpt->ld : ht_row_pitch(di, true);
  const int64_t mx = std::max<int64_t>(g->max_ndst, 1);
  float* a_stage[2] = {nullptr, nullptr};
  float* h_stage[2] = {nullptr, nullptr};
  float* nbuf = nullptr;
  // A/B variant: no aggregate is kept and everything is in HBM: aggregate and transform in one kernel (ht_fused.hip)
  const bool fused = ctx->fuse_update && !A_ckpt && h_dev && !buffer && H_in->loc == HT_LOC_DEVICE && di <= 1024;
  if (!a_dev && !fused) {
    HT_TRY(ht_scratch(ctx, HT_S_ACHUNK, (size_t)mx * a_ld * 4 * 2, (void**)&a_stage[0]));
    a_stage[1] = a_stage[0] + mx * a_ld;
  }
  if (!h_dev) {
    HT_TRY(ht_scratch(ctx, HT_S_OCHUNK, (size_t)mx * H_out->ld * 4 * 2, (void**)&h_stage[0]));
    h_stage[1] = h_stage[0] + mx * H_out->ld;
  }
  if (buffer) HT_TRY(ht_scratch(ctx, HT_S_NBUF, (size_t)g->cache_rows * H_in->ld * 4, (void**)&nbuf));

  Pipe P(ctx);
  P.fence = (side_in || staged) && !ctx->no_link_fence;
  if (side_in) {
    hipEvent_t ev_start = nullptr;
    HT_TRY(P.rec(P.s_c, &ev_start));
    HT_TRY(P.wait(P.s_in, ev_start));
    P.used_in = true;
  }
  hipEvent_t ev_out[2] = {nullptr, nullptr};   // D2H of the staging pair b has finished
  hipEvent_t ev_agg_prev = nullptr;            // the previous chunk's aggregation has read the buffer
  // With a^l and h^{l+1} both in HBM the update stage of neighbouring chunks runs as one GEMM over their joint row
  // range (chunks are balanced by edges, and a hub chunk of a thousand rows cannot fill the matrix cores); each output
  // row is the same sum whatever range it is computed in.
  const bool merge_dense = a_dev && h_dev;
  int64_t pend0 = -1, pend1 = -1;
  auto flush_dense = [&]() -> int {
    if (pend0 < 0) return HT_OK;
    const int64_t nr = pend1 - pend0;
    R.tm.begin(&R.st->t_gemm_ms);
    HT_TRY(ht_gemm_nn(ctx, P.s_c, A_ckpt->ptr + pend0 * a_ld, a_ld, W, H_out->ptr + pend0 * H_out->ld, H_out->ld, nr, di, dn,
                      desc->act == HT_ACT_RELU));
    R.tm.end();
    R.st->n_gemm += 1;
    R.st->gemm_flops += 2.0 * nr * di * dn;
    pend0 = pend1 = -1;
    return HT_OK;
  };
  int q = 0;
  for (int j = 0; j < g->n; ++j) {
    const ChunkMeta& c = g->chunks[j];
    const int64_t ndst = c.dst1 - c.dst0;
    if (ndst == 0) continue;
    const int b = q & 1;
    ++q;
    if (buffer) {
      if (side_in) {
        HT_TRY(P.wait(P.s_in, ev_agg_prev));   // the buffer is updated in place
        HT_TRY(P.link_begin(P.s_in));
        HT_TRY(gather_chunk(R, j, H_in, Hin, di, nbuf, P.s_in));
        HT_TRY(P.link_end(P.s_in));
        hipEvent_t ev_g = nullptr;
        HT_TRY(P.rec(P.s_in, &ev_g));
        HT_TRY(P.wait(P.s_c, ev_g));
      } else {
        HT_TRY(gather_chunk(R, j, H_in, Hin, di, nbuf, P.s_c));
      }
    }
    if (fused) {
      const int li = R.layer < HT_MAX_LAYERS ? R.layer : HT_MAX_LAYERS - 1;
      R.tm.begin(&R.st->t_agg_fwd_layer_ms[li]);
      HT_TRY(ht_agg_update_fused(ctx, P.s_c, g, c, Hin, H_in->ld, di, W, dn, desc->act == HT_ACT_RELU, H_out->ptr, H_out->ld));
      R.tm.end();
      R.st->n_spmm_fwd += 1;
      R.st->n_agg_fwd_layer[li] += 1;
      R.st->edges += c.nnz;
      R.st->spmm_fwd_alg_bytes += spmm_alg_bytes(c, di);
      R.st->agg_fwd_layer_alg_bytes[li] += spmm_alg_bytes(c, di);
      R.st->n_gemm += 1;
      R.st->gemm_flops += 2.0 * ndst * di * dn;
      continue;
    }
    if (staged) HT_TRY(P.wait(P.s_c, ev_out[b]));
    float* a_dst = a_dev ? A_ckpt->ptr + c.dst0 * a_ld : a_stage[b];
    HT_TRY(P.agg_begin());
    HT_TRY(spmm_chunk(R, j, buffer, buffer ? nbuf : Hin, H_in->ld, di, a_dst, a_ld));
    HT_TRY(P.agg_end());
    if (side_in) HT_TRY(P.rec(P.s_c, &ev_agg_prev));
    if (merge_dense) {
      if (pend0 >= 0 && c.dst0 != pend1) HT_TRY(flush_dense());   // not adjacent in vertex order (reorganised schedule)
      if (pend0 < 0) pend0 = c.dst0;
      pend1 = c.dst1;
      if (pend1 - pend0 >= HT_DENSE_MERGE_ROWS) HT_TRY(flush_dense());
      continue;
    }
    float* h_dst = h_dev ? H_out->ptr + c.dst0 * H_out->ld : h_stage[b];
    R.tm.begin(&R.st->t_gemm_ms);
    HT_TRY(ht_gemm_nn(ctx, P.s_c, a_dst, a_ld, W, h_dst, H_out->ld, ndst, di, dn, desc->act == HT_ACT_RELU));
    R.tm.end();
    R.st->n_gemm += 1;
    R.st->gemm_flops += 2.0 * ndst * di * dn;
    if (staged) {
      hipEvent_t ev_c = nullptr;
      HT_TRY(P.rec(P.s_c, &ev_c));
      HT_TRY(P.wait(P.s_out, ev_c));
      HT_TRY(P.link_begin(P.s_out));
      P.used_out = true;
      if (a_host)
        HT_TRY(copy_rows(R, P.s_out, A_ckpt->ptr + c.dst0 * a_ld, a_stage[b], (size_t)ndst * a_ld * 4, hipMemcpyDeviceToHost));
      if (!h_dev)
        HT_TRY(copy_rows(R, P.s_out, H_out->ptr + c.dst0 * H_out->ld, h_stage[b], (size_t)ndst * H_out->ld * 4,
                         hipMemcpyDeviceToHost));
      HT_TRY(P.link_end(P.s_out));
      HT_TRY(P.rec(P.s_out, &ev_out[b]));
    }
  }
  HT_TRY(flush_dense());
  // later work on the compute stream sees every row at its home
  HT_TRY(P.wait(P.s_c, ev_out[0]));
  HT_TRY(P.wait(P.s_c, ev_out[1]));
  P.used_in = P.used_out = false;   // everything is ordered behind the compute stream now
  return HT_OK;
}

// Layer forward from a cached aggregate: h' = act(a W) per chunk, a^l read from A (HBM in place,
// or pinned host memory through a staging pair).  Used for layer 0 when a^0 = A_hat X of an earlier
// epoch is still valid.
int layer_fwd_from_ckpt(Run& R, const ht_layer_desc* desc, const ht_tensor* A, const float* W, ht_tensor* H_out) {
  ht_ctx* ctx = R.ctx;
  const ht_graph* g = R.g;
  const int di = desc->d_in, dn = desc->d_out;
  HT_TRY(check_tensor(ctx, A, g->V, di, "A_ckpt"));
  HT_TRY(check_tensor(ctx, H_out, g->V, dn, "H_out"));
  const bool a_host = A->loc == HT_LOC_HOST_PINNED;
  const bool h_dev = H_out->loc == HT_LOC_DEVICE;
  const int64_t mx = std::max<int64_t>(g->max_ndst, 1);
  float* a_stage[2] = {nullptr, nullptr};
  float* h_stage[2] = {nullptr, nullptr};
  if (a_host) {
    HT_TRY(ht_scratch(ctx, HT_S_ACHUNK, (size_t)mx * A->ld * 4 * 2, (void**)&a_stage[0]));
    a_stage[1] = a_stage[0] + mx * A->ld;
  }
  if (!h_dev) {
    HT_TRY(ht_scratch(ctx, HT_S_OCHUNK, (size_t)mx * H_out->ld * 4 * 2, (void**)&h_stage[0]));
    h_stage[1] = h_stage[0] + mx * H_out->ld;
  }
  Pipe P(ctx);
  if (a_host) {
    hipEvent_t ev_start = nullptr;
    HT_TRY(P.rec(P.s_c, &ev_start));
    HT_TRY(P.wait(P.s_in, ev_start));
    P.used_in = true;
  }
  hipEvent_t ev_out[2] = {nullptr, nullptr}, ev_cdone[2] = {nullptr, nullptr};
  int q = 0;
  for (int j = 0; j < g->n; ++j) {
    const ChunkMeta& c = g->chunks[j];
    const int64_t ndst = c.dst1 - c.dst0;
    if (ndst == 0) continue;
    const int b = q & 1;
    ++q;
    const float* a_rows = A->ptr + c.dst0 * A->ld;
    if (a_host) {
      hipEvent_t ev_in = nullptr;
      HT_TRY(P.wait(P.s_in, ev_cdone[b]));
      HT_TRY(copy_rows(R, P.s_in, a_stage[b], a_rows, (size_t)ndst * A->ld * 4, hipMemcpyHostToDevice));
      HT_TRY(P.rec(P.s_in, &ev_in));
      HT_TRY(P.wait(P.s_c, ev_in));
      a_rows = a_stage[b];
    }
    if (!h_dev) HT_TRY(P.wait(P.s_c, ev_out[b]));
    float* h_dst = h_dev ? H_out->ptr + c.dst0 * H_out->ld : h_stage[b];
    R.tm.begin(&R.st->t_gemm_ms);
    HT_TRY(ht_gemm_nn(ctx, P.s_c, a_rows, A->ld, W, h_dst, H_out->ld, ndst, di, dn, desc->act == HT_ACT_RELU));
    R.tm.end();
    R.st->n_gemm += 1;
    R.st->gemm_flops += 2.0 * ndst * di * dn;
    if (a_host) HT_TRY(P.rec(P.s_c, &ev_cdone[b]));
    if (!h_dev) {
      hipEvent_t ev_c = nullptr;
      HT_TRY(P.rec(P.s_c, &ev_c));
      HT_TRY(P.wait(P.s_out, ev_c));
      P.used_out = true;
      HT_TRY(copy_rows(R, P.s_out, H_out->ptr + c.dst0 * H_out->ld, h_stage[b], (size_t)ndst * H_out->ld * 4,
                       hipMemcpyDeviceToHost));
      HT_TRY(P.rec(P.s_out, &ev_out[b]));
    }
  }
  HT_TRY(P.wait(P.s_c, ev_out[0]));
  HT_TRY(P.wait(P.s_c, ev_out[1]));
  P.used_in = P.used_out = false;
  return HT_OK;
}

struct AccTask {
  hipEvent_t ready;   // the D2H of `rows` has finished
  float* grad;
  int64_t ld;
  const int32_t* ids;
  const float* rows;
  int64_t rows_ld;
  int64_t n;
  int d;
};

// Host-side gradient accumulation beside the GPU work (Alg. 3).  A worker
// thread waits for each task's D2H event on the host and adds the rows; the
// enqueueing thread only blocks when it is about to reuse a staging buffer whose
// task has not finished.  (A host function enqueued in a HIP stream would do the
// same, but it occupies a hardware queue other streams share while it runs.)
class AccWorker {
 public:
  AccWorker(ht_ctx* ctx) : ctx_(ctx) {}
  ~AccWorker() { finish(); }
  void start() {
    if (!th_.joinable()) th_ = std::thread([this] { run(); });
  }
  void push(const AccTask& t) {
    std::lock_guard<std::mutex> lk(mu_);
    q_.push_back(t);
    cv_.notify_all();
  }
  // block until at least `count` tasks have completed
  void wait_done(int64_t count) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return done_ >= count || failed_; });
  }
  void finish() {
    if (!th_.joinable()) return;
    {
      std::lock_guard<std::mutex> lk(mu_);
      stop_ = true;
      cv_.notify_all();
    }
    th_.join();
  }
  bool failed() const { return failed_; }
  double ms() const { return ms_; }

 private:
  void run() {
    (void)hipSetDevice(ctx_->device);
    int64_t next = 0;
    for (;;) {
      AccTask t;
      {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] { return stop_ || next < (int64_t)q_.size(); });
        if (next >= (int64_t)q_.size()) return;   // stop requested and queue drained
        t = q_[next];
      }
      if (hipEventSynchronize(t.ready) != hipSuccess) {
        std::lock_guard<std::mutex> lk(mu_);
        failed_ = true;
        cv_.notify_all();
        return;
      }
      auto t0 = std::chrono::steady_clock::now();
      cpu_accumulate(ctx_, t.grad, t.ld, t.ids, t.rows, t.rows_ld, t.n, t.d);
      const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
      {
        std::lock_guard<std::mutex> lk(mu_);
        ms_ += ms;
        ++next;
        done_ = next;
        cv_.notify_all();
      }
    }
  }
  ht_ctx* ctx_;
  std::thread th_;
  std::mutex mu_;
  std::condition_variable cv_;
  std::vector<AccTask> q_;
  int64_t done_ = 0;
  bool stop_ = false;
  std::atomic<bool> failed_{false};   // read by the enqueueing thread without the lock
  double ms_ = 0.0;
};

int layer_bwd_impl(Run& R, const ht_layer_desc* desc, const ht_tensor* ckpt, const float* W, const ht_tensor* dH_out,
                   const ht_tensor* H_out, ht_tensor* dH_in, float* dW) {
  ht_ctx* ctx = R.ctx;
  const ht_graph* g = R.g;
  hipStream_t st = ctx->stream;
  const int di = desc->d_in, dn = desc->d_out;
  HT_TRY(check_tensor(ctx, ckpt, g->V, di, "ckpt"));
  HT_TRY(check_tensor(ctx, dH_out, g->V, dn, "dH_out"));
  if (H_out) HT_TRY(check_tensor(ctx, H_out, g->V, dn, "H_out"));
  if (dH_in) HT_TRY(check_tensor(ctx, dH_in, g->V, di, "dH_in"));
  if (!W || !dW) return ht_set_err(ctx, HT_EINVAL, "W or dW is null");
  if (desc->ckpt_kind != HT_CKPT_AGG && desc->ckpt_kind != HT_CKPT_INPUT)
    return ht_set_err(ctx, HT_EINVAL, "unknown checkpoint kind %d", desc->ckpt_kind);
  const bool relu = desc->act == HT_ACT_RELU;
  const bool agg_ckpt = desc->ckpt_kind == HT_CKPT_AGG;
  const int64_t mx = std::max<int64_t>(g->max_ndst, 1);
  const int64_t ld_i = ht_row_pitch(di, true), ld_o = ht_row_pitch(dn, true);

  // forward-side inputs
  bool agg_buffer = false;
  float* Hin = nullptr;
  float* nbuf = nullptr;
  if (!agg_ckpt) {
    HT_TRY(resolve_gather(ctx, desc->gather_mode, ckpt, &agg_buffer));
    HT_TRY(gpu_ptr(ctx, ckpt, &Hin));
    if (agg_buffer) HT_TRY(ht_scratch(ctx, HT_S_NBUF, (size_t)g->cache_rows * ckpt->ld * 4, (void**)&nbuf));
  }
  // gradient side: direct accumulation into dH_in (HBM) or through the in-place gradient buffer
  bool gbuffer = false;
  if (dH_in) HT_TRY(resolve_gather(ctx, desc->gather_mode, dH_in, &gbuffer));

  const bool a_host = agg_ckpt && ckpt->loc != HT_LOC_DEVICE;
  const bool dh_host = dH_out->loc != HT_LOC_DEVICE;
  const bool ho_host = relu && H_out && H_out->loc != HT_LOC_DEVICE;
  const bool in_host = a_host || dh_host || ho_host;   // some rows arrive through the input stream
  float* a_stage[2] = {nullptr, nullptr};
  float* dh_stage[2] = {nullptr, nullptr};
  float* z_stage[2] = {nullptr, nullptr};
  float *dz_chunk = nullptr, *da_chunk = nullptr, *gbuf = nullptr;
  const int64_t a_ld = agg_ckpt ? ckpt->ld : ld_i;
  // The dense work (mask, grad W, grad a) of neighbouring chunks runs as one launch over their joint row range when
  // everything it touches is in HBM and no buffer is updated in place between chunks: chunks are balanced by edges, and a
  // hub chunk of a thousand rows cannot fill the matrix cores.  The grouping depends on the graph and on where the
  // tensors live only, so every intermediate-data mode sums grad W in the same order.  Each group is a run of chunks
  // adjacent in schedule and in vertex order, closed once it holds HT_DENSE_MERGE_ROWS rows; elsewhere one chunk each.
  const bool merge_ok = !in_host && !agg_buffer && !(dH_in && gbuffer);
  std::vector<std::pair<int, int>> groups;
  int64_t gmax = mx;
  for (int j = 0; j < g->n;) {
    int k = j;
    if (merge_ok && g->chunks[j].dst1 > g->chunks[j].dst0)
      while (k + 1 < g->n && g->chunks[k + 1].dst1 > g->chunks[k + 1].dst0 && g->chunks[k + 1].dst0 == g->chunks[k].dst1 &&
             g->chunks[k].dst1 - g->chunks[j].dst0 < HT_DENSE_MERGE_ROWS)
        ++k;
    groups.emplace_back(j, k);
    gmax = std::max(gmax, g->chunks[k].dst1 - g->chunks[j].dst0);
    j = k + 1;
  }
  if (!agg_ckpt || a_host) {
    HT_TRY(ht_scratch(ctx, HT_S_ACHUNK, (size_t)gmax * a_ld * 4 * 2, (void**)&a_stage[0]));
    a_stage[1] = a_stage[0] + gmax * a_ld;
  }
  if (dh_host) {
    HT_TRY(ht_scratch(ctx, HT_S_OCHUNK, (size_t)mx * dH_out->ld * 4 * 2, (void**)&dh_stage[0]));
    dh_stage[1] = dh_stage[0] + mx * dH_out->ld;
  }
  if (relu) {
    const int64_t zl = H_out ? H_out->ld : ld_o;
    if (!H_out || ho_host) {
      HT_TRY(ht_scratch(ctx, HT_S_ZCHUNK, (size_t)gmax * zl * 4 * 2, (void**)&z_stage[0]));
      z_stage[1] = z_stage[0] + gmax * zl;
    }
    HT_TRY(ht_scratch(ctx, HT_S_DZCHUNK, (size_t)gmax * ld_o * 4, (void**)&dz_chunk));
  }
  if (dH_in) {
    HT_TRY(ht_scratch(ctx, HT_S_DACHUNK, (size_t)gmax * ld_i * 4, (void**)&da_chunk));
    if (gbuffer) HT_TRY(ht_scratch(ctx, HT_S_MISC, (size_t)g->cache_rows * ld_i * 4, (void**)&gbuf));
  }
  // CPU-side accumulation (Alg. 3): host copy of the leave lists, device and pinned staging pairs
  // When the schedule loads every row once per pass, each row also leaves exactly once, after the last
  // chunk that adds to it: if dH_in is known to hold zeros the rows are stored straight to their home
  // by a link kernel, no host-side add.
  const bool store_home = dH_in && gbuffer && dH_in->loc == HT_LOC_HOST_PINNED && g->single_leave && R.dhin_is_zero;
  const bool cpu_accum = dH_in && gbuffer && dH_in->loc == HT_LOC_HOST_PINNED && !store_home;
  float* dhin_gpu = nullptr;
  if (store_home) HT_TRY(gpu_ptr(ctx, dH_in, &dhin_gpu));
  constexpr int NLV = 4;   // depth of the leave staging rings: D2H runs ahead of the host-side adds
  constexpr int64_t LEAVE_BATCH = 262144;   // rows per compaction / D2H / host-add task
  float* leave_dev[NLV] = {};
  float* leave_pin[NLV] = {};
  if (cpu_accum) {
    int64_t mxl = 1;
    for (const ChunkMeta& c : g->chunks) mxl = std::max(mxl, c.n_leave);
    mxl = std::min(mxl, LEAVE_BATCH);
    if (g->leave_host.empty()) {
      g->leave_host.resize((size_t)std::max<int64_t>(g->v_load, 1));
      HT_HIP(ctx, hipMemcpy(g->leave_host.data(), g->leave.p, (size_t)g->v_load * 4, hipMemcpyDeviceToHost));
    }
    HT_TRY(ht_scratch(ctx, HT_S_LEAVE, (size_t)mxl * ld_i * 4 * NLV, (void**)&leave_dev[0]));
    HT_TRY(ht_host_scratch(ctx, 0, (size_t)mxl * ld_i * 4 * NLV, (void**)&leave_pin[0]));
    for (int k = 1; k < NLV; ++k) {
      leave_dev[k] = leave_dev[0] + (int64_t)k * mxl * ld_i;
      leave_pin[k] = leave_pin[0] + (int64_t)k * mxl * ld_i;
    }
    (void)host_threads(ctx);
  }

  Pipe P(ctx);
  AccWorker worker(ctx);   // declared after P: joined before P's destructor waits for the streams
  if (cpu_accum) worker.start();
  P.fence = (in_host || cpu_accum || store_home) && !ctx->no_link_fence;
  if (in_host) {
    hipEvent_t ev_start = nullptr;
    HT_TRY(P.rec(P.s_c, &ev_start));
    HT_TRY(P.wait(P.s_in, ev_start));
    P.used_in = true;
  }
  hipEvent_t ev_cdone[2] = {nullptr, nullptr};     // compute that read the input staging pair b has finished
  hipEvent_t ev_leave_free[NLV] = {};              // D2H out of leave_dev[r] has finished
  int n_left = 0;
  bool first = true;
  int q = 0;
  // ---- rows that the schedule releases after a chunk leave the gradient buffer (Alg. 3)
  hipEvent_t ev_stored = nullptr;   // the last store of leaving rows straight to their home
  auto leave_rows = [&](const ChunkMeta& c) -> int {
    if (!(dH_in && gbuffer && c.n_leave > 0)) return HT_OK;
    if (store_home) {
      hipEvent_t ev_done = nullptr, ev_st = nullptr;
      HT_TRY(P.rec(P.s_c, &ev_done));
      HT_TRY(P.wait(P.s_out, ev_done));
      HT_TRY(P.link_begin(P.s_out));
      P.used_out = true;
      const int id = R.tm.begin_on(&R.st->t_copy_ms, P.s_out);
      HT_TRY(ht_gather_rows(ctx, P.s_out, gbuf, ld_i, g->leave_slot.p + c.leave_off, dhin_gpu, dH_in->ld,
                            g->leave.p + c.leave_off, c.n_leave, di, nullptr, ctx->link_blocks));
      R.tm.end_id(id);
      R.st->bytes_d2h += c.n_leave * (int64_t)di * 4;
      HT_TRY(P.link_end(P.s_out));
      HT_TRY(P.rec(P.s_out, &ev_st));
      ev_stored = ev_st;   // waited for before the next aggregation writes freed positions, and at the end
    } else if (!cpu_accum) {
      HT_TRY(ht_add_rows(ctx, st, gbuf, ld_i, g->leave_slot.p + c.leave_off, dH_in->ptr, dH_in->ld,
                         g->leave.p + c.leave_off, c.n_leave, di));
    } else {
      // compaction on the compute stream (the next chunk overwrites freed positions), D2H on the
      // output stream, the add on the host beside the next chunks' GPU work
      for (int64_t k0 = 0; k0 < c.n_leave; k0 += LEAVE_BATCH) {
        const int64_t nk = std::min(LEAVE_BATCH, c.n_leave - k0);
        const int64_t off = c.leave_off + k0;
        const int r = n_left++ % NLV;
        HT_TRY(P.wait(P.s_c, ev_leave_free[r]));
        HT_TRY(ht_gather_rows(ctx, st, gbuf, ld_i, g->leave_slot.p + off, leave_dev[r], ld_i, nullptr, nk, di, nullptr));
        hipEvent_t ev_comp = nullptr;
        HT_TRY(P.rec(P.s_c, &ev_comp));
        HT_TRY(P.wait(P.s_out, ev_comp));
        if (n_left > NLV) worker.wait_done(n_left - NLV);   // the host has consumed leave_pin[r]
        if (worker.failed()) return ht_set_err(ctx, HT_EHIP, "host-side accumulation: waiting for a copy failed");
        HT_TRY(P.link_begin(P.s_out));
        P.used_out = true;
        HT_TRY(copy_rows(R, P.s_out, leave_pin[r], leave_dev[r], (size_t)nk * ld_i * 4, hipMemcpyDeviceToHost));
        HT_TRY(P.link_end(P.s_out));
        HT_TRY(P.rec(P.s_out, &ev_leave_free[r]));
        worker.push(AccTask{ev_leave_free[r], dH_in->ptr, dH_in->ld, g->leave_host.data() + off, leave_pin[r], ld_i, nk, di});
      }
    }
    return HT_OK;
  };
  for (const auto& grp : groups) {
    const int j0 = grp.first, j1 = grp.second;
    const ChunkMeta& c = g->chunks[j0];                       // the group's first chunk: its rows start the range
    const int64_t ndst = g->chunks[j1].dst1 - c.dst0;         // destination rows of the whole group
    if (ndst == 0) {   // no destinations: no edges, no neighbours; the schedule may still release rows here
      HT_TRY(leave_rows(c));
      continue;
    }
    const int b = q & 1;
    ++q;
    // ---- inputs (Alg. 1)
    const float* a_rows = nullptr;
    const float* dh_rows = nullptr;
    const float* ref = nullptr;
    int64_t ref_ld = 0;
    if (in_host) {
      HT_TRY(P.wait(P.s_in, ev_cdone[b]));
      HT_TRY(P.link_begin(P.s_in));
    }
    if (agg_ckpt) {
      if (a_host) {
        HT_TRY(copy_rows(R, P.s_in, a_stage[b], ckpt->ptr + c.dst0 * a_ld, (size_t)ndst * a_ld * 4, hipMemcpyHostToDevice));
        a_rows = a_stage[b];
      } else {
        a_rows = ckpt->ptr + c.dst0 * a_ld;
      }
    }
    if (dh_host) {
      HT_TRY(copy_rows(R, P.s_in, dh_stage[b], dH_out->ptr + c.dst0 * dH_out->ld, (size_t)ndst * dH_out->ld * 4,
                       hipMemcpyHostToDevice));
      dh_rows = dh_stage[b];
    } else {
      dh_rows = dH_out->ptr + c.dst0 * dH_out->ld;
    }
    if (relu && H_out) {
      ref_ld = H_out->ld;
      if (ho_host) {
        HT_TRY(copy_rows(R, P.s_in, z_stage[b], H_out->ptr + c.dst0 * H_out->ld, (size_t)ndst * H_out->ld * 4,
                         hipMemcpyHostToDevice));
        ref = z_stage[b];
      } else {
        ref = H_out->ptr + c.dst0 * H_out->ld;
      }
    }
    if (in_host) {
      HT_TRY(P.link_end(P.s_in));
      hipEvent_t ev_in = nullptr;
      HT_TRY(P.rec(P.s_in, &ev_in));
      HT_TRY(P.wait(P.s_c, ev_in));
    }
    // ---- compute
    if (!agg_ckpt) {   // pure recomputation: aggregate again from h^l, chunk by chunk into the group's rows
      for (int j = j0; j <= j1; ++j) {
        const ChunkMeta& cj = g->chunks[j];
        if (agg_buffer) HT_TRY(gather_chunk(R, j, ckpt, Hin, di, nbuf, st));
        HT_TRY(P.agg_begin());
        HT_TRY(spmm_chunk(R, j, agg_buffer, agg_buffer ? nbuf : Hin, ckpt->ld, di, a_stage[b] + (cj.dst0 - c.dst0) * a_ld, a_ld));
        HT_TRY(P.agg_end());
      }
      a_rows = a_stage[b];
    }
    const float* dz_rows = dh_rows;
    int64_t dz_ld = dH_out->ld;
    if (relu) {
      if (!H_out) {  // re-forward of the update stage (Alg. 1)
        R.tm.begin(&R.st->t_gemm_ms);
        HT_TRY(ht_gemm_nn(ctx, st, a_rows, a_ld, W, z_stage[0], ld_o, ndst, di, dn, 0));
        R.tm.end();
        R.st->n_gemm += 1;
        R.st->gemm_flops += 2.0 * ndst * di * dn;
        ref = z_stage[0];
        ref_ld = ld_o;
      }
      HT_TRY(ht_relu_mask(ctx, st, dh_rows, dH_out->ld, ref, ref_ld, dz_chunk, ld_o, ndst, dn));
      dz_rows = dz_chunk;
      dz_ld = ld_o;
    }
    R.tm.begin(&R.st->t_gemm_ms);
    HT_TRY(ht_gemm_tn(ctx, st, a_rows, a_ld, dz_rows, dz_ld, dW, ndst, di, dn, first ? 0 : 1));
    R.tm.end();
    R.st->n_gemm += 1;
    R.st->gemm_flops += 2.0 * ndst * di * dn;
    first = false;
    if (dH_in) {
      R.tm.begin(&R.st->t_gemm_ms);
      HT_TRY(ht_gemm_nt(ctx, st, dz_rows, dz_ld, W, da_chunk, ld_i, ndst, dn, di, 0));
      R.tm.end();
      R.st->n_gemm += 1;
      R.st->gemm_flops += 2.0 * ndst * di * dn;
    }
    if (in_host) HT_TRY(P.rec(P.s_c, &ev_cdone[b]));   // the staged inputs have been consumed
    for (int j = j0; j <= j1; ++j) {
      const ChunkMeta& cj = g->chunks[j];
      if (dH_in) {
        float* partial = nullptr;
        const int64_t out_ld = gbuffer ? ld_i : dH_in->ld;
        if (cj.bwd.n_part > 0) HT_TRY(ht_scratch(ctx, HT_S_SPART, (size_t)g->max_bpart * out_ld * 4, (void**)&partial));
        SpmmArgs a{};
        a.it_row = cj.bwd.row; a.it_e0 = cj.bwd.e0; a.it_len = cj.bwd.len; a.it_part = cj.bwd.part; a.n_items = cj.bwd.n_items;
        a.n_edges = cj.nnz;
        a.fx_row = cj.bwd.fx_row; a.fx_part0 = cj.bwd.fx_part0; a.fx_nseg = cj.bwd.fx_nseg; a.n_fix = cj.bwd.n_fix;
        if (g->merged) {
          a.idx = g->usdst.p + cj.ue0;
          a.w_edge = g->uw_bwd.p + cj.ue0;
          a.n_edges = cj.nu;
        } else {
          a.idx = g->sdst.p + cj.e0;
          a.ew = g->s.p + cj.dst0;
        }
        a.src = da_chunk + (cj.dst0 - c.dst0) * ld_i;      // the chunk's rows inside the group's grad a
        a.src_ld = ld_i;
        a.d = di;
        a.out = gbuffer ? gbuf : dH_in->ptr;
        a.out_ld = out_ld;
        a.out_idx = gbuffer ? g->gslot.p + cj.nbr_off : g->nbr.p + cj.nbr_off;
        a.post = g->s.p;
        a.post_idx = g->nbr.p + cj.nbr_off;
        a.accumulate = 1;
        a.partial = partial;
        a.max_slabs = ctx->slabs_bwd;
        HT_TRY(P.wait(P.s_c, ev_stored));   // positions freed by the last store are written from here on
        HT_TRY(P.agg_begin());
        R.tm.begin(&R.st->t_spmm_bwd_ms);
        HT_TRY(ht_spmm_launch(ctx, st, a));
        R.tm.end();
        HT_TRY(P.agg_end());
        R.st->n_spmm_bwd += 1;
        R.st->edges += cj.nnz;
        R.st->spmm_bwd_alg_bytes += spmm_alg_bytes(cj, di);
      }
      HT_TRY(leave_rows(cj));
    }
  }
  if (first) HT_TRY(ht_fill_zero(ctx, st, dW, (size_t)di * dn * 4));
  if (store_home) {   // dH_in is complete for later work on the stream
    HT_TRY(P.wait(P.s_c, ev_stored));
    P.used_out = false;
  }
  if (cpu_accum) {
    // the gradient tensor is complete once every host-side add has run
    worker.finish();
    if (worker.failed()) return ht_set_err(ctx, HT_EHIP, "host-side accumulation: waiting for a copy failed");
    R.st->t_cpu_accum_ms += worker.ms();
    P.used_out = false;
  }
  P.used_in = false;   // every input copy was waited for by the compute stream
  return HT_OK;
}

// ---- update-first order: H' = act(A_hat (H W)).  Same function as Eq. 2 (both stages are
// linear), aggregating rows of width d_out.  Everything lives in HBM here.

int need_hbm(ht_ctx* ctx, const ht_tensor* t, const char* name) {
  if (t->loc != HT_LOC_DEVICE)
    return ht_set_err(ctx, HT_ESHAPE, "update-first order: %s must be in HBM", name);
  return HT_OK;
}

// Aggregation arguments of chunk j at width d: forward (rows = destinations, reading rows of
// `src` by global id) or backward (rows = sources N_j, reading the chunk's destination rows).
void agg_args_direct(const ht_graph* g, const ChunkMeta& c, bool fwd, SpmmArgs* a) {
  const ItemSet& it = fwd ? c.fwd : c.bwd;
  a->it_row = it.row; a->it_e0 = it.e0; a->it_len = it.len; a->it_part = it.part; a->n_items = it.n_items;
  a->fx_row = it.fx_row; a->fx_part0 = it.fx_part0; a->fx_nseg = it.fx_nseg; a->n_fix = it.n_fix;
  a->n_edges = c.nnz;
  if (g->merged) {
    a->idx = (fwd ? g->ucol.p : g->usdst.p) + c.ue0;
    a->w_edge = (fwd ? g->uw_fwd.p : g->uw_bwd.p) + c.ue0;
    a->n_edges = c.nu;
  } else {
    a->idx = fwd ? g->col.p + c.e0 : g->sdst.p + c.e0;
    a->ew = fwd ? g->s.p : g->s.p + c.dst0;
  }
}

int layer_fwd_update_first(Run& R, const ht_layer_desc* desc, const ht_tensor* H_in, const float* W, ht_tensor* H_out) {
  ht_ctx* ctx = R.ctx;
  const ht_graph* g = R.g;
  hipStream_t st = ctx->stream;
  const int di = desc->d_in, dn = desc->d_out;
  HT_TRY(check_tensor(ctx, H_in, g->V, di, "H_in"));
  HT_TRY(check_tensor(ctx, H_out, g->V, dn, "H_out"));
  HT_TRY(need_hbm(ctx, H_in, "H_in"));
  HT_TRY(need_hbm(ctx, H_out, "H_out"));
  if (!W) return ht_set_err(ctx, HT_EINVAL, "W is null");
  const int64_t ld_t = ht_row_pitch(dn, true);
  float* T = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_TFULL, (size_t)std::max<int64_t>(g->V, 1) * ld_t * 4, (void**)&T));
  // t = H_in W for every vertex (row ranges keep the launches within the grid limits)
  const int64_t step = (int64_t)1 << 22;
  for (int64_t r0 = 0; r0 < g->V; r0 += step) {
    const int64_t nr = std::min(step, g->V - r0);
    R.tm.begin(&R.st->t_gemm_ms);
    HT_TRY(ht_gemm_nn(ctx, st, H_in->ptr + r0 * H_in->ld, H_in->ld, W, T + r0 * ld_t, ld_t, nr, di, dn, 0));
    R.tm.end();
    R.st->n_gemm += 1;
    R.st->gemm_flops += 2.0 * nr * di * dn;
  }
  const int li = R.layer < HT_MAX_LAYERS ? R.layer : HT_MAX_LAYERS - 1;
  for (int j = 0; j < g->n; ++j) {
    const ChunkMeta& c = g->chunks[j];
    if (c.dst1 == c.dst0) continue;
    float* partial = nullptr;
    if (c.fwd.n_part > 0) HT_TRY(ht_scratch(ctx, HT_S_SPART, (size_t)g->max_fpart * H_out->ld * 4, (void**)&partial));
    SpmmArgs a{};
    agg_args_direct(g, c, true, &a);
    a.src = T; a.src_ld = ld_t; a.d = dn;
    a.out = H_out->ptr + c.dst0 * H_out->ld; a.out_ld = H_out->ld; a.out_idx = nullptr;
    a.post = g->s.p + c.dst0; a.post_idx = nullptr;
    a.accumulate = 0;
    a.relu = desc->act == HT_ACT_RELU;
    a.partial = partial;
    a.max_slabs = ctx->slabs_fwd;
    a.tm = &R.tm;
    a.t_items = &R.st->t_agg_fwd_layer_ms[li];
    a.t_fix = &R.st->t_agg_fix_ms;
    HT_TRY(ht_spmm_launch(ctx, st, a));
    R.st->n_spmm_fwd += 1;
    R.st->n_agg_fwd_layer[li] += 1;
    R.st->edges += c.nnz;
    R.st->spmm_fwd_alg_bytes += spmm_alg_bytes(c, dn);
    R.st->agg_fwd_layer_alg_bytes[li] += spmm_alg_bytes(c, dn);
  }
  return HT_OK;
}

int layer_bwd_update_first(Run& R, const ht_layer_desc* desc, const ht_tensor* H_in, const float* W,
                           const ht_tensor* dH_out, const ht_tensor* H_out, ht_tensor* dH_in, float* dW) {
  ht_ctx* ctx = R.ctx;
  const ht_graph* g = R.g;
  hipStream_t st = ctx->stream;
  const int di = desc->d_in, dn = desc->d_out;
  const bool relu = desc->act == HT_ACT_RELU;
  HT_TRY(check_tensor(ctx, H_in, g->V, di, "ckpt"));
  HT_TRY(check_tensor(ctx, dH_out, g->V, dn, "dH_out"));
  HT_TRY(need_hbm(ctx, H_in, "ckpt"));
  HT_TRY(need_hbm(ctx, dH_out, "dH_out"));
  if (relu && !H_out) return ht_set_err(ctx, HT_EINVAL, "update-first backward with ReLU needs H_out");
  if (H_out) {
    HT_TRY(check_tensor(ctx, H_out, g->V, dn, "H_out"));
    HT_TRY(need_hbm(ctx, H_out, "H_out"));
  }
  if (dH_in) {
    HT_TRY(check_tensor(ctx, dH_in, g->V, di, "dH_in"));
    HT_TRY(need_hbm(ctx, dH_in, "dH_in"));
  }
  if (!W || !dW) return ht_set_err(ctx, HT_EINVAL, "W or dW is null");
  const int64_t ld_t = ht_row_pitch(dn, true);
  const int64_t mx = std::max<int64_t>(g->max_ndst, 1);
  float *dT = nullptr, *dz_chunk = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_TFULL, (size_t)std::max<int64_t>(g->V, 1) * ld_t * 4, (void**)&dT));
  if (relu) HT_TRY(ht_scratch(ctx, HT_S_DZCHUNK, (size_t)mx * ld_t * 4, (void**)&dz_chunk));
  HT_TRY(ht_fill_zero(ctx, st, dT, (size_t)g->V * ld_t * 4));
  // dt[N_j] += s_u * sum_v s_v dz[v], chunk by chunk
  for (int j = 0; j < g->n; ++j) {
    const ChunkMeta& c = g->chunks[j];
    const int64_t ndst = c.dst1 - c.dst0;
    if (ndst == 0) continue;
    const float* dz_rows = dH_out->ptr + c.dst0 * dH_out->ld;
    int64_t dz_ld = dH_out->ld;
    if (relu) {
      HT_TRY(ht_relu_mask(ctx, st, dz_rows, dz_ld, H_out->ptr + c.dst0 * H_out->ld, H_out->ld, dz_chunk, ld_t, ndst, dn));
      dz_rows = dz_chunk;
      dz_ld = ld_t;
    }
    float* partial = nullptr;
    if (c.bwd.n_part > 0) HT_TRY(ht_scratch(ctx, HT_S_SPART, (size_t)g->max_bpart * ld_t * 4, (void**)&partial));
    SpmmArgs a{};
    agg_args_direct(g, c, false, &a);
    a.src = dz_rows; a.src_ld = dz_ld; a.d = dn;
    a.out = dT; a.out_ld = ld_t;
    a.out_idx = g->nbr.p + c.nbr_off;
    a.post = g->s.p; a.post_idx = g->nbr.p + c.nbr_off;
    a.accumulate = 1;
    a.partial = partial;
    a.max_slabs = ctx->slabs_bwd;
    R.tm.begin(&R.st->t_spmm_bwd_ms);
    HT_TRY(ht_spmm_launch(ctx, st, a));
    R.tm.end();
    R.st->n_spmm_bwd += 1;
    R.st->edges += c.nnz;
    R.st->spmm_bwd_alg_bytes += spmm_alg_bytes(c, dn);
  }
  // dW = h^T dt, dH_in += dt W^T over row ranges
  const int64_t step = (int64_t)1 << 22;
  bool first = true;
  for (int64_t r0 = 0; r0 < g->V; r0 += step) {
    const int64_t nr = std::min(step, g->V - r0);
    R.tm.begin(&R.st->t_gemm_ms);
    HT_TRY(ht_gemm_tn(ctx, st, H_in->ptr + r0 * H_in->ld, H_in->ld, dT + r0 * ld_t, ld_t, dW, nr, di, dn, first ? 0 : 1));
    R.tm.end();
    R.st->n_gemm += 1;
    R.st->gemm_flops += 2.0 * nr * di * dn;
    first = false;
    if (dH_in) {
      R.tm.begin(&R.st->t_gemm_ms);
      HT_TRY(ht_gemm_nt(ctx, st, dT + r0 * ld_t, ld_t, W, dH_in->ptr + r0 * dH_in->ld, dH_in->ld, nr, dn, di, 1));
      R.tm.end();
      R.st->n_gemm += 1;
      R.st->gemm_flops += 2.0 * nr * di * dn;
    }
  }
  if (first) HT_TRY(ht_fill_zero(ctx, st, dW, (size_t)di * dn * 4));
  return HT_OK;
}

int finish(Run& R, ht_stats* user, const std::chrono::steady_clock::time_point& t0, bool sync) {
  ht_ctx* ctx = R.ctx;
  if (sync || user) {
    HT_HIP(ctx, hipStreamSynchronize(ctx->stream));
    HT_TRY(R.tm.resolve());
  }
  ctx->ev_next = 0;
  if (user) {
    for (int l = 0; l < HT_MAX_LAYERS; ++l) R.st->t_spmm_fwd_ms += R.st->t_agg_fwd_layer_ms[l];
    R.st->t_spmm_fwd_ms += R.st->t_agg_fix_ms;
    R.st->t_total_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    *user = *R.st;
  }
  return HT_OK;
}

}  // namespace

void ht_epoch_ws_free(ht_ctx* ctx) {
  EpochWs* ws = ctx->ws;
  if (!ws) return;
  (void)hipStreamSynchronize(ctx->stream);
  for (size_t i = 0; i < ws->dev_ptrs.size(); ++i) ht_dev_free(ctx, ws->dev_ptrs[i], ws->dev_bytes_of[i]);
  for (void* p : ws->host_ptrs) (void)hipHostFree(p);
  if (ws->graph_exec) (void)hipGraphExecDestroy(ws->graph_exec);
  delete ws;
  ctx->ws = nullptr;
}

namespace {

int ws_tensor(ht_ctx* ctx, EpochWs* ws, int64_t V, int32_t d, int res, ht_tensor* t) {
  t->rows = V;
  t->cols = d;
  t->ld = ht_row_pitch(d, res != HT_RES_HOST);
  const size_t bytes = (size_t)V * t->ld * 4;
  if (res == HT_RES_HOST) {
    void* p = nullptr;
    hipError_t e = hipHostMalloc(&p, bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      return ht_set_err(ctx, HT_ENOMEM, "hipHostMalloc(%zu): %s", bytes, hipGetErrorString(e));
    }
    ws->host_ptrs.push_back(p);
    t->ptr = (float*)p;
    t->loc = HT_LOC_HOST_PINNED;
  } else {
    void* p = nullptr;
    HT_TRY(ht_dev_alloc(ctx, &p, bytes));
    ws->dev_ptrs.push_back(p);
    ws->dev_bytes_of.push_back(bytes);
    t->ptr = (float*)p;
    t->loc = HT_LOC_DEVICE;
  }
  return HT_OK;
}

int zero_tensor(ht_ctx* ctx, ht_tensor* t) {
  const size_t bytes = (size_t)t->rows * t->ld * 4;
  if (t->loc == HT_LOC_DEVICE) return ht_fill_zero(ctx, ctx->stream, t->ptr, bytes);
  HT_HIP(ctx, hipStreamSynchronize(ctx->stream));
  std::memset(t->ptr, 0, bytes);
  return HT_OK;
}

}  // namespace

extern "C" {

int ht_layer_fwd(ht_ctx* ctx, const ht_graph* g, const ht_layer_desc* desc, const ht_tensor* H_in, const float* W,
                 ht_tensor* H_out, ht_tensor* A_ckpt, ht_stats* stats) {
  if (!ctx) return HT_EINVAL;
  if (!g || !desc || !H_in || !H_out) return ht_set_err(ctx, HT_EINVAL, "ht_layer_fwd: null argument");
  if (g->ctx != ctx) return ht_set_err(ctx, HT_ESTATE, "graph belongs to another context");
  if (desc->d_in <= 0 || desc->d_out <= 0) return ht_set_err(ctx, HT_ESHAPE, "layer widths must be positive");
  HT_HIP(ctx, hipSetDevice(ctx->device));
  auto t0 = std::chrono::steady_clock::now();
  ht_stats local{};
  Run R(ctx, g, &local, stats != nullptr);
  if (desc->order != HT_ORDER_AGG_FIRST && desc->order != HT_ORDER_UPDATE_FIRST)
    return ht_set_err(ctx, HT_EINVAL, "unknown stage order %d", desc->order);
  int rc = desc->order == HT_ORDER_UPDATE_FIRST ? layer_fwd_update_first(R, desc, H_in, W, H_out)
                                                : layer_fwd_impl(R, desc, H_in, W, H_out, A_ckpt);
  if (rc != HT_OK) {
    (void)hipStreamSynchronize(ctx->stream);
    ctx->ev_next = 0;
    return rc;
  }
  return finish(R, stats, t0, false);
}

// ht_layer_fwd for callers that cannot allocate: the same kernels in the same order, with the two scratch buffers of
// the all-in-HBM path (the packed copy of W, the partial sums of cut rows) taken from the device's static array.
int ht_layer_fwd_static(ht_ctx* ctx, const ht_graph* g, const ht_layer_desc* desc, const ht_tensor* H_in, const float* W,
                        ht_tensor* H_out, ht_tensor* A_ckpt) {
  if (!ctx) return HT_EINVAL;
  if (!g || !desc || !H_in || !H_out || !A_ckpt || !W) return ht_set_err(ctx, HT_EINVAL, "ht_layer_fwd_static: null argument");
  if (g->ctx != ctx) return ht_set_err(ctx, HT_ESTATE, "graph belongs to another context");
  if (desc->d_in <= 0 || desc->d_out <= 0) return ht_set_err(ctx, HT_ESHAPE, "layer widths must be positive");
  if (desc->order != HT_ORDER_AGG_FIRST) return ht_set_err(ctx, HT_EINVAL, "ht_layer_fwd_static: aggregate-first order only");
  if (desc->gather_mode == HT_GATHER_BUFFER)
    return ht_set_err(ctx, HT_EINVAL, "ht_layer_fwd_static: the neighbour buffer is not available here (rows are read in place)");
  if (H_in->loc != HT_LOC_DEVICE || H_out->loc != HT_LOC_DEVICE || A_ckpt->loc != HT_LOC_DEVICE)
    return ht_set_err(ctx, HT_ESHAPE, "ht_layer_fwd_static: H_in, H_out and A_ckpt must be in HBM");
  // sizes are checked against the static array before anything is launched
  const size_t need_w = (((size_t)desc->d_in + 15) & ~(size_t)15) * (((size_t)desc->d_out + 127) & ~(size_t)127) * 4;
  const size_t need_p = (size_t)g->max_fpart * (size_t)A_ckpt->ld * 4;
  if (need_w + need_p + 512 > HT_STATIC_SCRATCH_BYTES)
    return ht_set_err(ctx, HT_ENOMEM, "ht_layer_fwd_static: this layer needs %zu bytes of scratch memory (packed W %zu, partial sums "
                      "of %lld cut rows' items %zu); the static array holds %zu: use ht_layer_fwd", need_w + need_p, need_w,
                      (long long)g->max_fpart, need_p, HT_STATIC_SCRATCH_BYTES);
  HT_HIP(ctx, hipSetDevice(ctx->device));
  ht_stats local{};
  Run R(ctx, g, &local, false);
  ht_static_begin(ctx);
  int rc = layer_fwd_impl(R, desc, H_in, W, H_out, A_ckpt);
  ht_static_end(ctx);
  ctx->ev_next = 0;
  if (rc != HT_OK) (void)hipStreamSynchronize(ctx->stream);
  return rc;
}

int ht_layer_bwd(ht_ctx* ctx, const ht_graph* g, const ht_layer_desc* desc, const ht_tensor* ckpt, const float* W,
                 const ht_tensor* dH_out, const ht_tensor* H_out, ht_tensor* dH_in, float* dW, ht_stats* stats) {
  if (!ctx) return HT_EINVAL;
  if (!g || !desc || !ckpt || !dH_out) return ht_set_err(ctx, HT_EINVAL, "ht_layer_bwd: null argument");
  if (g->ctx != ctx) return ht_set_err(ctx, HT_ESTATE, "graph belongs to another context");
  if (desc->d_in <= 0 || desc->d_out <= 0) return ht_set_err(ctx, HT_ESHAPE, "layer widths must be positive");
  HT_HIP(ctx, hipSetDevice(ctx->device));
  auto t0 = std::chrono::steady_clock::now();
  ht_stats local{};
  Run R(ctx, g, &local, stats != nullptr);
  if (desc->order != HT_ORDER_AGG_FIRST && desc->order != HT_ORDER_UPDATE_FIRST)
    return ht_set_err(ctx, HT_EINVAL, "unknown stage order %d", desc->order);
  int rc = desc->order == HT_ORDER_UPDATE_FIRST ? layer_bwd_update_first(R, desc, ckpt, W, dH_out, H_out, dH_in, dW)
                                                : layer_bwd_impl(R, desc, ckpt, W, dH_out, H_out, dH_in, dW);
  if (rc != HT_OK) {
    (void)hipStreamSynchronize(ctx->stream);
    ctx->ev_next = 0;
    return rc;
  }
  return finish(R, stats, t0, false);
}

int ht_epoch(ht_ctx* ctx, const ht_graph* g, const ht_model* model, const ht_tensor* X, const int32_t* labels,
             const ht_plan_opts* plan, float* loss_out, ht_stats* stats) {
  if (!ctx) return HT_EINVAL;
  if (!g || !model || !X || !labels || !loss_out) return ht_set_err(ctx, HT_EINVAL, "ht_epoch: null argument");
  if (g->ctx != ctx) return ht_set_err(ctx, HT_ESTATE, "graph belongs to another context");
  const int L = model->n_layers;
  if (L < 1 || !model->dims || !model->W) return ht_set_err(ctx, HT_EINVAL, "ht_epoch: bad model");
  for (int l = 0; l <= L; ++l)
    if (model->dims[l] <= 0) return ht_set_err(ctx, HT_ESHAPE, "ht_epoch: layer widths must be positive");
  for (int l = 0; l < L; ++l)
    if (!model->W[l]) return ht_set_err(ctx, HT_EINVAL, "ht_epoch: W[%d] is null", l);
  HT_HIP(ctx, hipSetDevice(ctx->device));
  HT_TRY(check_tensor(ctx, X, g->V, model->dims[0], "X"));
  auto t0 = std::chrono::steady_clock::now();
  const int64_t V = g->V;

  // ---- residency plan (Sec. 4.2 sized to this GPU)
  int res_h = plan ? plan->res_h : HT_RES_AUTO, res_a = plan ? plan->res_a : HT_RES_AUTO,
      res_g = plan ? plan->res_g : HT_RES_AUTO;
  int inter = plan ? plan->inter : HT_INTER_AUTO;
  const int gather_mode = plan ? plan->gather_mode : HT_GATHER_AUTO;
  int64_t budget = plan ? plan->hbm_budget_bytes : 0;
  if (budget == 0) {
    size_t fr = 0, tot = 0;
    HT_HIP(ctx, hipMemGetInfo(&fr, &tot));
    budget = (int64_t)fr - ((int64_t)2 << 30);
    // buffers of a previous epoch with the same shape are reused, so count them as free
    if (ctx->ws)
      for (size_t b : ctx->ws->dev_bytes_of) budget += (int64_t)b;
  }
  auto bytes_of = [&](int l0, int l1) {
    int64_t b = 0;
    for (int l = l0; l <= l1; ++l) b += V * ht_row_pitch(model->dims[l], true) * 4;
    return b;
  };
  int64_t left = budget;
  // the output layer's logits and their gradient stay in HBM (the loss runs on them in place)
  left -= 2 * bytes_of(L, L);
  if (res_g == HT_RES_AUTO) { if (L > 1 && bytes_of(1, L - 1) <= left) { res_g = HT_RES_HBM; left -= bytes_of(1, L - 1); } else res_g = L > 1 ? HT_RES_HOST : HT_RES_HBM; }
  bool a_spills = false;      // the planner, not the caller, put a^l in host memory
  if (inter == HT_INTER_RECOMPUTE) res_a = HT_RES_HBM;   // no checkpoint tensors exist: nothing to place
  else if (res_a == HT_RES_AUTO) {
    if (bytes_of(0, L - 1) <= left) { res_a = HT_RES_HBM; left -= bytes_of(0, L - 1); }
    else { res_a = HT_RES_HOST; a_spills = true; }
  }
  if (res_h == HT_RES_AUTO) { if (L > 1 && bytes_of(1, L - 1) <= left) { res_h = HT_RES_HBM; left -= bytes_of(1, L - 1); } else res_h = L > 1 ? HT_RES_HOST : HT_RES_HBM; }
  if (inter == HT_INTER_AUTO && a_spills) {
    // Sec. 4.2's trade-off priced for this GPU.  Host-side cache: a^l crosses the link twice.  Recomputation:
    // the rows of a host-resident h^l that the buffer schedule loads cross it once more, and every layer
    // is aggregated a second time.
    double t_cache = 0.0, t_again = 0.0;
    const double pairs = (double)(g->merged ? g->n_unique : g->Ep);
    for (int l = 0; l < L; ++l) {
      const double row = 4.0 * (double)model->dims[l];
      const bool in_host = l == 0 ? X->loc == HT_LOC_HOST_PINNED : res_h == HT_RES_HOST;
      t_cache += 2.0 * (double)V * row / HT_LINK_BYTES_PER_S;
      t_again += (in_host ? (double)g->v_load * row / HT_LINK_BYTES_PER_S : 0.0) + pairs * row / HT_GATHER_BYTES_PER_S;
    }
    if (t_again < t_cache) {
      inter = HT_INTER_RECOMPUTE;
      res_a = HT_RES_HBM;
    }
  }
  if (inter == HT_INTER_AUTO) inter = res_h == HT_RES_HBM ? HT_INTER_MASK : HT_INTER_HYBRID;
  if (inter != HT_INTER_MASK && inter != HT_INTER_HYBRID && inter != HT_INTER_RECOMPUTE)
    return ht_set_err(ctx, HT_EINVAL, "ht_epoch: unknown intermediate-data mode %d", inter);
  const bool recompute = inter == HT_INTER_RECOMPUTE;
  // ---- stage order per layer: update-first only where every tensor of the layer is in HBM
  const int order = plan ? plan->order : HT_ORDER_AGG_FIRST;
  if (order != HT_ORDER_AGG_FIRST && order != HT_ORDER_UPDATE_FIRST && order != HT_ORDER_AUTO)
    return ht_set_err(ctx, HT_EINVAL, "ht_epoch: unknown stage order %d", order);
  const bool want_reuse0 = plan && plan->reuse_input_aggregate && !recompute;
  uint32_t upd_mask = 0;
  if (order != HT_ORDER_AGG_FIRST && L <= 32 && gather_mode != HT_GATHER_BUFFER) {
    for (int l = want_reuse0 ? 1 : 0; l < L; ++l) {   // (a^0 is only kept by the printed stage order)
      const bool in_hbm = l == 0 ? X->loc == HT_LOC_DEVICE : res_h == HT_RES_HBM;
      const bool out_hbm = l == L - 1 || res_h == HT_RES_HBM;
      const bool gout_hbm = l == L - 1 || res_g == HT_RES_HBM;
      const bool gin_hbm = l == 0 || res_g == HT_RES_HBM;
      const bool narrower = model->dims[l + 1] < model->dims[l];
      if (in_hbm && out_hbm && gout_hbm && gin_hbm && (order == HT_ORDER_UPDATE_FIRST || narrower)) upd_mask |= 1u << l;
    }
  }

  // ---- workspace
  EpochWs* ws = ctx->ws;
  bool reuse = ws && ws->V == V && (int)ws->dims.size() == L + 1 && ws->res_h == res_h && ws->res_a == res_a &&
               ws->res_g == res_g && ws->upd_mask == upd_mask && ws->no_ckpt == recompute;
  if (reuse)
    for (int l = 0; l <= L; ++l) reuse = reuse && ws->dims[l] == model->dims[l];
  const bool reuse0 = reuse && want_reuse0 && ws->a0_of == X->ptr && ws->a0_graph == g->serial && ws->a[0].ptr;
  if (!reuse) {
    ht_epoch_ws_free(ctx);
    ws = new (std::nothrow) EpochWs();
    if (!ws) return ht_set_err(ctx, HT_ENOMEM, "ht_epoch: host allocation failed");
    ctx->ws = ws;
    ws->V = V;
    ws->dims.assign(model->dims, model->dims + L + 1);
    ws->res_h = res_h; ws->res_a = res_a; ws->res_g = res_g;
    ws->upd_mask = upd_mask;
    ws->no_ckpt = recompute;
    ws->h.assign(L + 1, ht_tensor{});
    ws->a.assign(L, ht_tensor{});
    ws->gh.assign(L + 1, ht_tensor{});
    ws->dW.assign(L, nullptr);
    int rc = HT_OK;
    for (int l = 1; l <= L && rc == HT_OK; ++l) rc = ws_tensor(ctx, ws, V, model->dims[l], l == L ? HT_RES_HBM : res_h, &ws->h[l]);
    for (int l = 0; l < L && rc == HT_OK; ++l)
      if (!((upd_mask >> l) & 1) && !recompute) rc = ws_tensor(ctx, ws, V, model->dims[l], res_a, &ws->a[l]);
    for (int l = 1; l <= L && rc == HT_OK; ++l) rc = ws_tensor(ctx, ws, V, model->dims[l], l == L ? HT_RES_HBM : res_g, &ws->gh[l]);
    for (int l = 0; l < L && rc == HT_OK; ++l) {
      void* p = nullptr;
      const size_t b = (size_t)model->dims[l] * model->dims[l + 1] * 4;
      rc = ht_dev_alloc(ctx, &p, b);
      if (rc == HT_OK) { ws->dW[l] = (float*)p; ws->dev_ptrs.push_back(p); ws->dev_bytes_of.push_back(b); }
    }
    if (rc == HT_OK) {
      void* p = nullptr;
      rc = ht_dev_alloc(ctx, &p, 16);
      if (rc == HT_OK) { ws->loss_dev = (float*)p; ws->dev_ptrs.push_back(p); ws->dev_bytes_of.push_back(16); }
    }
    if (rc != HT_OK) {
      ht_epoch_ws_free(ctx);
      return rc;
    }
  }

  ht_stats local{};
  Run R(ctx, g, &local, stats != nullptr);
  if (plan && plan->stats_detail == HT_STATS_AGG_FWD) {
    R.tm.only_lo = &local.t_agg_fwd_layer_ms[0];
    R.tm.only_hi = &local.t_agg_fwd_layer_ms[0] + HT_MAX_LAYERS;
  } else if (plan && plan->stats_detail != HT_STATS_ALL)
    return ht_set_err(ctx, HT_EINVAL, "ht_epoch: unknown stats_detail %d", plan->stats_detail);
  auto fail = [&](int rc) {
    (void)hipStreamSynchronize(ctx->stream);
    ctx->ev_next = 0;
    return rc;
  };
  // Host-resident gradient tensors that the backward pass adds into start as zeros.  They are not
  // touched before the backward pass, so a helper thread clears them beside the forward pass
  // instead of the GPU waiting for a memset between two layers.
  auto stored_once = [&](int l) {   // a never-evicting gradient buffer stores every row of a host-resident grad h^l exactly once
    return g->single_leave && g->v_load == V && ws->gh[l].loc == HT_LOC_HOST_PINNED && gather_mode != HT_GATHER_DIRECT;
  };
  struct Joiner {
    std::thread th;
    ~Joiner() { if (th.joinable()) th.join(); }
  } zeroer;
  {
    std::vector<ht_tensor*> todo;
    for (int l = 1; l < L; ++l)
      if (ws->gh[l].loc == HT_LOC_HOST_PINNED && !stored_once(l)) todo.push_back(&ws->gh[l]);
    if (!todo.empty())
      zeroer.th = std::thread([todo] {
        for (ht_tensor* t : todo) std::memset(t->ptr, 0, (size_t)t->rows * t->ld * 4);
      });
  }
  // ---- the epoch's stream work.  With every tensor in HBM it is kernels on one stream only, so it
  // can be recorded once into a HIP graph and replayed (ht_plan_opts.use_graph): the first epoch of a
  // key runs eagerly (it sizes the scratch memory, which a capture may not allocate), the second is
  // captured, instantiated and launched, later ones are one graph launch.
  bool in_capture = false;
  auto enqueue = [&]() -> int {
    // ---- forward (Alg. 1)
    for (int l = 0; l < L; ++l) {
      ht_layer_desc d{};
      d.d_in = model->dims[l]; d.d_out = model->dims[l + 1];
      d.act = l < L - 1 ? HT_ACT_RELU : HT_ACT_NONE;
      d.gather_mode = gather_mode;
      R.layer = l;
      const bool upd = (upd_mask >> l) & 1;
      d.order = upd ? HT_ORDER_UPDATE_FIRST : HT_ORDER_AGG_FIRST;
      int rc = upd                ? layer_fwd_update_first(R, &d, l == 0 ? X : &ws->h[l], model->W[l], &ws->h[l + 1])
               : (l == 0 && reuse0) ? layer_fwd_from_ckpt(R, &d, &ws->a[0], model->W[0], &ws->h[1])
                                    : layer_fwd_impl(R, &d, l == 0 ? X : &ws->h[l], model->W[l], &ws->h[l + 1],
                                                     recompute ? nullptr : &ws->a[l]);
      if (rc != HT_OK) {
        ws->a0_of = nullptr;
        return rc;
      }
      if (l == 0) {   // a^0 = A_hat X is in a[0] from here on (the backward pass only reads it)
        const bool kept = !upd && !recompute;
        ws->a0_of = kept ? X->ptr : nullptr;
        ws->a0_graph = kept ? g->serial : 0;
      }
    }
    // ---- downstream task and its gradient (Alg. 1)
    {
      R.tm.begin(&R.st->t_loss_ms);
      int rc = ht_softmax_ce(ctx, ctx->stream, ws->h[L].ptr, ws->h[L].ld, labels, V, model->dims[L], ws->gh[L].ptr,
                             ws->gh[L].ld, ws->loss_dev);
      R.tm.end();
      if (rc != HT_OK) return rc;
    }
    if (in_capture)
      if (const char* dbg = getenv("HT_GRAPH_DEBUG"))
        if (atoi(dbg) == 3) {   // a launch the runtime rejects on the host, to exercise the fallback after a broken capture
          k_noop<<<1, 4096, 0, ctx->stream>>>();
          HT_LAUNCH_CHECK(ctx);
        }
    // ---- backward (Alg. 1)
    for (int l = L - 1; l >= 0; --l) {
      ht_layer_desc d{};
      d.d_in = model->dims[l]; d.d_out = model->dims[l + 1];
      d.act = l < L - 1 ? HT_ACT_RELU : HT_ACT_NONE;
      d.gather_mode = gather_mode;
      d.ckpt_kind = recompute ? HT_CKPT_INPUT : HT_CKPT_AGG;
      R.dhin_is_zero = false;
      if (l > 0) {
        if (ws->gh[l].loc == HT_LOC_HOST_PINNED) {
          if (zeroer.th.joinable()) zeroer.th.join();     // cleared beside the forward pass (or stored exactly once)
        } else {
          int rc = zero_tensor(ctx, &ws->gh[l]);
          if (rc != HT_OK) return rc;
        }
        R.dhin_is_zero = true;
      }
      R.layer = l;
      const bool mask_ok = inter == HT_INTER_MASK || (recompute && ws->h[l + 1].loc == HT_LOC_DEVICE);
      const ht_tensor* mask_from = (mask_ok && l < L - 1) ? &ws->h[l + 1] : nullptr;
      const ht_tensor* ckpt = recompute ? (l == 0 ? X : &ws->h[l]) : &ws->a[l];
      const bool upd = (upd_mask >> l) & 1;
      d.order = upd ? HT_ORDER_UPDATE_FIRST : HT_ORDER_AGG_FIRST;
      int rc = upd ? layer_bwd_update_first(R, &d, l == 0 ? X : &ws->h[l], model->W[l], &ws->gh[l + 1],
                                            l < L - 1 ? &ws->h[l + 1] : nullptr, l > 0 ? &ws->gh[l] : nullptr, ws->dW[l])
                   : layer_bwd_impl(R, &d, ckpt, model->W[l], &ws->gh[l + 1], mask_from,
                                    l > 0 ? &ws->gh[l] : nullptr, ws->dW[l]);
      if (rc != HT_OK) return rc;
    }
    // ---- parameter update (Alg. 1)
    R.tm.begin(&R.st->t_update_ms);
    for (int l = 0; l < L; ++l) {
      int rc = ht_sgd(ctx, ctx->stream, model->W[l], ws->dW[l], (int64_t)model->dims[l] * model->dims[l + 1], model->lr);
      if (rc != HT_OK) return rc;
    }
    R.tm.end();
    return HT_OK;
  };
  const bool all_hbm = X->loc == HT_LOC_DEVICE && res_h == HT_RES_HBM && res_g == HT_RES_HBM && (recompute || res_a == HT_RES_HBM);
  std::vector<uintptr_t> key;
  if (plan && plan->use_graph && all_hbm && !stats) {
    key = {(uintptr_t)g->serial, (uintptr_t)ctx->scratch_gen, (uintptr_t)X->ptr, (uintptr_t)X->ld, (uintptr_t)labels, (uintptr_t)inter, (uintptr_t)upd_mask,
           (uintptr_t)reuse0, (uintptr_t)gather_mode, (uintptr_t)L};
    uint32_t lr_bits;
    std::memcpy(&lr_bits, &model->lr, 4);
    key.push_back(lr_bits);
    for (int l = 0; l < L; ++l) key.push_back((uintptr_t)model->W[l]);
  }
  bool launched = false;
  if (!key.empty() && ws->graph_exec && ws->graph_key == key) {
    hipError_t e = hipGraphLaunch(ws->graph_exec, ctx->stream);
    if (e != hipSuccess) return fail(ht_set_err(ctx, HT_EHIP, "hipGraphLaunch: %s", hipGetErrorString(e)));
    launched = true;
    ++ctx->graph_launches;
  } else if (!key.empty() && ws->warm_key == key && ws->bad_key != key) {
    if (ws->graph_exec) {
      (void)hipGraphExecDestroy(ws->graph_exec);
      ws->graph_exec = nullptr;
      ws->graph_key.clear();
    }
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) return fail(ht_set_err(ctx, HT_EHIP, "hipStreamBeginCapture: %s", hipGetErrorString(e)));
    in_capture = true;
    int rc = enqueue();
    in_capture = false;
    e = hipStreamEndCapture(ctx->stream, &graph);
    if (const char* dbg = getenv("HT_GRAPH_DEBUG"))
      if (atoi(dbg) == 2 && rc == HT_OK) rc = ht_set_err(ctx, HT_ESTATE, "capture discarded on request");   // exercises the fallback
    if (rc == HT_OK && e == hipSuccess && graph) {
      e = hipGraphInstantiate(&ws->graph_exec, graph, nullptr, nullptr, 0);
      if (e == hipSuccess) e = hipGraphLaunch(ws->graph_exec, ctx->stream);
      if (e == hipSuccess) {
        ws->graph_key = key;
        launched = true;
        ++ctx->graph_launches;
      } else if (ws->graph_exec) {
        (void)hipGraphExecDestroy(ws->graph_exec);
        ws->graph_exec = nullptr;
      }
    }
    if (graph) (void)hipGraphDestroy(graph);
    if (!launched) {   // nothing has run: this epoch runs eagerly below, and the key is not tried again
      if (getenv("HT_GRAPH_DEBUG"))
        fprintf(stderr, "ht_epoch: graph capture failed (enqueue rc %d: %s; hip: %s)\n", rc, ctx->err.c_str(), hipGetErrorString(e));
      (void)hipGetLastError();
      ws->bad_key = key;
      ws->a0_of = reuse0 ? ws->a0_of : nullptr;
    }
  }
  if (!launched) {
    const int rc = enqueue();
    if (rc != HT_OK) return fail(rc);
    ws->warm_key = key;
  }
  {
    hipError_t e = hipMemcpyAsync(loss_out, ws->loss_dev, 4, hipMemcpyDeviceToHost, ctx->stream);
    if (e != hipSuccess) return fail(ht_set_err(ctx, HT_EHIP, "loss copy: %s", hipGetErrorString(e)));
  }
  local.plan_inter = inter;
  local.plan_res_h = res_h;
  local.plan_res_a = recompute ? 0 : res_a;
  local.plan_res_g = res_g;
  return finish(R, stats, t0, true);
}

int ht_tensor_zero(ht_ctx* ctx, ht_tensor* t) {
  if (!ctx) return HT_EINVAL;
  if (!t || !t->ptr || t->rows < 0 || t->ld < t->cols || (t->ld & 3))
    return ht_set_err(ctx, HT_EINVAL, "ht_tensor_zero: bad tensor");
  HT_HIP(ctx, hipSetDevice(ctx->device));
  HT_TRY(zero_tensor(ctx, t));
  HT_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return HT_OK;
}

int ht_epoch_buffer(ht_ctx* ctx, int32_t kind, int32_t layer, ht_tensor* out) {
  if (!ctx || !out) return HT_EINVAL;
  EpochWs* ws = ctx->ws;
  if (!ws) return ht_set_err(ctx, HT_ESTATE, "no epoch has run on this context");
  const int L = (int)ws->dims.size() - 1;
  switch (kind) {
    case HT_BUF_H:
      if (layer < 1 || layer > L) return ht_set_err(ctx, HT_EINVAL, "layer out of range");
      *out = ws->h[layer];
      return HT_OK;
    case HT_BUF_A:
      if (layer < 0 || layer >= L) return ht_set_err(ctx, HT_EINVAL, "layer out of range");
      if (!ws->a[layer].ptr) return ht_set_err(ctx, HT_ESTATE, "layer %d keeps no aggregate checkpoint", layer);
      *out = ws->a[layer];
      return HT_OK;
    case HT_BUF_GH:
      if (layer < 1 || layer > L) return ht_set_err(ctx, HT_EINVAL, "layer out of range");
      *out = ws->gh[layer];
      return HT_OK;
    case HT_BUF_DW:
      if (layer < 0 || layer >= L) return ht_set_err(ctx, HT_EINVAL, "layer out of range");
      out->ptr = ws->dW[layer];
      out->rows = ws->dims[layer];
      out->cols = ws->dims[layer + 1];
      out->ld = ws->dims[layer + 1];
      out->loc = HT_LOC_DEVICE;
      return HT_OK;
    default:
      return ht_set_err(ctx, HT_EINVAL, "unknown buffer kind %d", kind);
  }
}

int ht_tensor_to_host(ht_ctx* ctx, const ht_tensor* t, float* dst) {
  if (!ctx || !t || !dst) return HT_EINVAL;
  if (!t->ptr || t->rows < 0 || t->cols <= 0 || t->ld < t->cols) return ht_set_err(ctx, HT_ESHAPE, "bad tensor");
  HT_HIP(ctx, hipStreamSynchronize(ctx->stream));
  if (t->rows == 0) return HT_OK;
  // rows [r0, r1) of `from` (pitch ld) into the dense destination, on the host cores
  auto pack = [&](const float* from, int64_t r0, int64_t r1) {
    const int nt = (int)std::min<int64_t>(host_threads(ctx), std::max<int64_t>(1, (r1 - r0) / 4096));
    auto work = [&](int64_t a, int64_t b) {
      for (int64_t r = a; r < b; ++r)
        std::memcpy(dst + r * t->cols, from + (r - r0) * t->ld, (size_t)t->cols * 4);
    };
    if (nt <= 1) return work(r0, r1);
    std::vector<std::thread> th;
    const int64_t per = (r1 - r0 + nt - 1) / nt;
    for (int k = 0; k < nt; ++k) {
      const int64_t a = r0 + k * per, b = std::min(r1, a + per);
      if (a < b) th.emplace_back(work, a, b);
    }
    for (auto& x : th) x.join();
  };
  if (t->loc != HT_LOC_DEVICE) {
    pack(t->ptr, 0, t->rows);
    return HT_OK;
  }
  // HBM: whole padded rows through a page-locked bounce buffer (a pitched copy into pageable
  // memory runs at a fraction of the link rate), then packed on the host
  const int64_t rows_per = std::max<int64_t>(1, ((int64_t)64 << 20) / (t->ld * 4));
  float* bounce = nullptr;
  HT_TRY(ht_host_scratch(ctx, 1, (size_t)rows_per * t->ld * 4, (void**)&bounce));
  for (int64_t r0 = 0; r0 < t->rows; r0 += rows_per) {
    const int64_t r1 = std::min(t->rows, r0 + rows_per);
    HT_HIP(ctx, hipMemcpy(bounce, t->ptr + r0 * t->ld, (size_t)(r1 - r0) * t->ld * 4, hipMemcpyDeviceToHost));
    pack(bounce, r0, r1);
  }
  return HT_OK;
}

}  // extern "C"

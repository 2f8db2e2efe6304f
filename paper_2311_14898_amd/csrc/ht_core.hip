// Context, error reporting, allocation accounting, event timers.
#include <cstdarg>
#include <cstdlib>

#include "ht_internal.h"

#include <mutex>

// Scratch memory of the allocation-free entry point (ht_layer_fwd_static): part of the code object, so every GPU the
// library runs on holds HT_STATIC_SCRATCH_BYTES of it from load to exit, and no call has to allocate.  In host code
// this name is only a handle for hipGetSymbolAddress; kernels get the device address taken below.  (No
// __attribute__((used)) here: it pins the device symbol to local binding, and the runtime, which finds the variable
// by name in the code object, aborts when it cannot; referenced from host code alone the compiler exports it.)
static __device__ __align__(256) unsigned char scratch[HT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int HT_MAX_DEVICES = 64;
std::mutex g_static_mu;
unsigned char* g_static_ptr[HT_MAX_DEVICES] = {};

// Address of `scratch` on the current device (each GPU has its own copy at its own address); taken once per device.
int static_scratch_address(int device, unsigned char** out) {
  *out = nullptr;
  if (device < 0 || device >= HT_MAX_DEVICES) return HT_EINVAL;
  std::lock_guard<std::mutex> lk(g_static_mu);
  if (!g_static_ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return HT_EHIP;
    }
    g_static_ptr[device] = (unsigned char*)p;
  }
  *out = g_static_ptr[device];
  return HT_OK;
}
}  // namespace

void ht_static_begin(ht_ctx* ctx) {
  ctx->static_mode = true;
  ctx->static_used = 0;
  for (int i = 0; i < HT_N_SCRATCH; ++i) ctx->static_off[i] = ctx->static_len[i] = 0;
}

void ht_static_end(ht_ctx* ctx) { ctx->static_mode = false; }

int ht_set_err(ht_ctx* ctx, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf;
  return code;
}

int ht_dev_alloc(ht_ctx* ctx, void** out, size_t bytes) {
  *out = nullptr;
  if (bytes == 0) return HT_OK;
  if (ctx->static_mode) return ht_set_err(ctx, HT_ESTATE, "a device allocation of %zu bytes was asked for inside the allocation-free entry point", bytes);
  if (ctx->hbm_budget > 0 && ctx->hbm_used + (int64_t)bytes > ctx->hbm_budget)
    return ht_set_err(ctx, HT_ENOMEM, "HBM budget exceeded: %lld in use + %zu requested > %lld",
                      (long long)ctx->hbm_used, bytes, (long long)ctx->hbm_budget);
  hipError_t e = hipMalloc(out, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    *out = nullptr;
    return ht_set_err(ctx, HT_ENOMEM, "hipMalloc(%zu): %s", bytes, hipGetErrorString(e));
  }
  ctx->hbm_used += (int64_t)bytes;
  return HT_OK;
}

void ht_dev_free(ht_ctx* ctx, void* p, size_t bytes) {
  if (!p) return;
  (void)hipFree(p);
  if (ctx) ctx->hbm_used -= (int64_t)bytes;
}

int ht_scratch(ht_ctx* ctx, int slot, size_t bytes, void** out) {
  if (ctx->static_mode) {
    // a piece of the static array per slot: cut at the slot's first request of this call, kept for its later ones
    *out = nullptr;
    if (!ctx->static_base) return ht_set_err(ctx, HT_ESTATE, "the static scratch array has no address on this device");
    if (ctx->static_len[slot] < bytes) {
      if (ctx->static_len[slot] != 0)
        return ht_set_err(ctx, HT_ESTATE, "scratch slot %d grew from %zu to %zu bytes inside one allocation-free call", slot,
                          ctx->static_len[slot], bytes);
      const size_t off = (ctx->static_used + 255) & ~(size_t)255;
      if (bytes > HT_STATIC_SCRATCH_BYTES || off > HT_STATIC_SCRATCH_BYTES - bytes)
        return ht_set_err(ctx, HT_ENOMEM, "the allocation-free entry point needs %zu more bytes of scratch memory (slot %d) after "
                          "%zu in use; its static array holds %zu: use the allocating entry point for this size", bytes, slot,
                          ctx->static_used, HT_STATIC_SCRATCH_BYTES);
      ctx->static_off[slot] = off;
      ctx->static_len[slot] = bytes;
      ctx->static_used = off + bytes;
    }
    *out = ctx->static_base + ctx->static_off[slot];
    return HT_OK;
  }
  if (ctx->scratch_bytes[slot] < bytes) {
    if (ctx->scratch[slot]) {
      HT_HIP(ctx, hipStreamSynchronize(ctx->stream));
      ht_dev_free(ctx, ctx->scratch[slot], ctx->scratch_bytes[slot]);
      ctx->scratch[slot] = nullptr;
      ctx->scratch_bytes[slot] = 0;
    }
    size_t want = bytes + bytes / 8 + 256;
    int rc = ht_dev_alloc(ctx, &ctx->scratch[slot], want);
    if (rc != HT_OK) return rc;
    ctx->scratch_bytes[slot] = want;
    ++ctx->scratch_gen;
  }
  *out = ctx->scratch[slot];
  return HT_OK;
}

int ht_host_scratch(ht_ctx* ctx, int slot, size_t bytes, void** out) {
  if (ctx->hscratch_bytes[slot] < bytes) {
    if (ctx->hscratch[slot]) {
      HT_HIP(ctx, hipDeviceSynchronize());
      (void)hipHostFree(ctx->hscratch[slot]);
      ctx->hscratch[slot] = nullptr;
      ctx->hscratch_bytes[slot] = 0;
    }
    size_t want = bytes + bytes / 8 + 256;
    hipError_t e = hipHostMalloc(&ctx->hscratch[slot], want, hipHostMallocDefault);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      ctx->hscratch[slot] = nullptr;
      return ht_set_err(ctx, HT_ENOMEM, "hipHostMalloc(%zu): %s", want, hipGetErrorString(e));
    }
    ctx->hscratch_bytes[slot] = want;
  }
  *out = ctx->hscratch[slot];
  return HT_OK;
}

hipEvent_t ht_event(ht_ctx* ctx) {
  if (ctx->ev_next == ctx->ev_pool.size()) {
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    ctx->ev_pool.push_back(e);
  }
  return ctx->ev_pool[ctx->ev_next++];
}

int Timer::begin_on(double* acc, hipStream_t s) {
  if (!on) return -1;
  if (only_lo && (acc < only_lo || acc >= only_hi)) return -1;
  hipEvent_t a = ht_event(ctx), b = ht_event(ctx);
  if (!a || !b) {
    on = false;
    return -1;
  }
  (void)hipEventRecord(a, s);
  ev.push_back(Ent{a, b, s, acc});
  return (int)ev.size() - 1;
}

void Timer::end_id(int id) {
  if (!on || id < 0 || id >= (int)ev.size()) return;
  (void)hipEventRecord(ev[id].b, ev[id].s);
}

int Timer::resolve() {
  for (size_t i = 0; i < ev.size(); ++i) {
    float ms = 0.f;
    hipError_t e = hipEventElapsedTime(&ms, ev[i].a, ev[i].b);
    if (e != hipSuccess) return ht_set_err(ctx, HT_EHIP, "hipEventElapsedTime: %s", hipGetErrorString(e));
    *ev[i].dst += (double)ms;
  }
  ev.clear();
  return HT_OK;
}

void ht_epoch_ws_free(ht_ctx* ctx);

extern "C" {

int ht_ctx_create(ht_ctx** out, int device, void* hip_stream) {
  if (!out) return HT_EINVAL;
  *out = nullptr;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return HT_EHIP;
  if (hipSetDevice(device) != hipSuccess) return HT_EHIP;
  ht_ctx* c = new (std::nothrow) ht_ctx();
  if (!c) return HT_ENOMEM;
  c->device = device;
  if (static_scratch_address(device, &c->static_base) != HT_OK) {
    delete c;
    return HT_EHIP;
  }
  if (const char* v = getenv("HT_AGG_VARIANT")) c->agg_variant = atoi(v);
  if (const char* v = getenv("HT_LINK_BLOCKS")) c->link_blocks = atoi(v) > 0 ? atoi(v) : 64;
  if (const char* v = getenv("HT_GATHER_BLOCKS")) c->gather_blocks = atoi(v) > 0 ? atoi(v) : 128;
  if (const char* v = getenv("HT_XCD_CONTIG")) c->xcd_contig = atoi(v);
  if (const char* v = getenv("HT_NO_LINK_FENCE")) c->no_link_fence = atoi(v);
  if (const char* v = getenv("HT_LINK_MEMCPY")) c->link_memcpy = atoi(v);
  if (const char* v = getenv("HT_SLABS_FWD")) c->slabs_fwd = atoi(v);
  if (const char* v = getenv("HT_SLABS_BWD")) c->slabs_bwd = atoi(v);
  if (const char* v = getenv("HT_AGG_UNROLL")) c->agg_unroll = atoi(v) == 8 ? 8 : 4;
  if (const char* v = getenv("HT_AGG_UNIFORM")) c->agg_uniform = atoi(v);
  if (const char* v = getenv("HT_SLAB_ALIGN")) c->slab_align = atoi(v);
  if (const char* v = getenv("HT_FUSE_UPDATE")) c->fuse_update = atoi(v);
  if (const char* v = getenv("HT_AGG_PHASES")) c->agg_phases = atoi(v) > 1 ? atoi(v) : 1;
  if (const char* v = getenv("HT_LINK_BLOCK_ROWS")) c->link_block_rows = atoll(v) > 0 ? atoll(v) : c->link_block_rows;
  if (hip_stream) {
    c->stream = (hipStream_t)hip_stream;
  } else {
    if (hipStreamCreate(&c->stream) != hipSuccess) {
      delete c;
      return HT_EHIP;
    }
    c->own_stream = true;
  }
  for (int i = 0; i < 3; ++i)
    if (hipStreamCreate(&c->side[i]) != hipSuccess) {
      delete c;
      return HT_EHIP;
    }
  *out = c;
  return HT_OK;
}

int ht_ctx_destroy(ht_ctx* ctx) {
  if (!ctx) return HT_EINVAL;
  (void)hipSetDevice(ctx->device);
  (void)hipStreamSynchronize(ctx->stream);
  for (int i = 0; i < 3; ++i)
    if (ctx->side[i]) {
      (void)hipStreamSynchronize(ctx->side[i]);
      (void)hipStreamDestroy(ctx->side[i]);
    }
  ht_epoch_ws_free(ctx);
  for (int i = 0; i < HT_N_SCRATCH; ++i)
    if (ctx->scratch[i]) ht_dev_free(ctx, ctx->scratch[i], ctx->scratch_bytes[i]);
  for (int i = 0; i < 4; ++i)
    if (ctx->hscratch[i]) (void)hipHostFree(ctx->hscratch[i]);
  for (hipEvent_t e : ctx->ev_pool) (void)hipEventDestroy(e);
  if (ctx->own_stream) (void)hipStreamDestroy(ctx->stream);
  delete ctx;
  return HT_OK;
}

int ht_sync(ht_ctx* ctx) {
  if (!ctx) return HT_EINVAL;
  HT_HIP(ctx, hipStreamSynchronize(ctx->stream));
  for (int i = 0; i < 3; ++i) HT_HIP(ctx, hipStreamSynchronize(ctx->side[i]));
  return HT_OK;
}

int64_t ht_ctx_graph_launches(const ht_ctx* ctx) { return ctx ? ctx->graph_launches : -1; }

int ht_ctx_set_hbm_budget(ht_ctx* ctx, int64_t bytes) {
  if (!ctx || bytes < 0) return HT_EINVAL;
  ctx->hbm_budget = bytes;
  return HT_OK;
}

const char* ht_strerror(int code) {
  switch (code) {
    case HT_OK: return "ok";
    case HT_EINVAL: return "invalid argument";
    case HT_ENOMEM: return "out of memory or over the byte budget";
    case HT_EHIP: return "HIP runtime error";
    case HT_ESHAPE: return "tensor shape, pitch or location does not fit";
    case HT_ESTATE: return "call not valid in this state";
    default: return "unknown error code";
  }
}

const char* ht_last_error(const ht_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int ht_memory_model(int64_t V, int32_t n_layers, const int32_t* dims, double* vertex_bytes,
                    double* intermediate_bytes) {
  if (V < 0 || n_layers < 1 || !dims) return HT_EINVAL;
  double sum = 0.0;
  for (int l = 0; l <= n_layers; ++l) sum += dims[l];
  if (vertex_bytes) *vertex_bytes = (double)V * sum * 4.0 * 2.0;
  double mid = 0.0;
  for (int l = 1; l < n_layers; ++l) mid += 2.0 * dims[l];
  mid += 3.0 * dims[n_layers];
  if (intermediate_bytes) *intermediate_bytes = (double)V * mid * 4.0;
  return HT_OK;
}

double ht_chunk_rows_model(int64_t V, int32_t n_chunks, double alpha) {
  if (n_chunks <= 0) return 0.0;
  return (1.0 + alpha) * (double)V / (double)n_chunks;
}

double ht_comm_cost_model(int64_t v_ori, int64_t v_p2p, int64_t v_ru, int64_t bytes_per_row, double t_hd, double t_dd,
                          double t_ru) {
  if (v_ru < 0 || v_ru > v_p2p || v_p2p > v_ori || bytes_per_row < 0) return -1.0;
  const double b = (double)bytes_per_row;
  double c = 0.0;
  const int64_t parts[3] = {v_ru, v_ori - v_p2p, v_p2p - v_ru};
  const double thr[3] = {t_hd, t_dd, t_ru};
  for (int k = 0; k < 3; ++k) {
    if (parts[k] == 0) continue;
    if (!(thr[k] > 0.0)) return -1.0;
    c += (double)parts[k] * b / thr[k];
  }
  return c;
}

}  // extern "C"

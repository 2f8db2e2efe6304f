// Internal declarations shared by the translation units of libhongtu.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <chrono>
#include <cstdio>
#include <string>
#include <vector>

#include "../../include/hongtu.h"

// Edges one forward aggregation work item covers at most (backward items take half).  Rows
// longer than this are cut into several items whose partial sums are added in item order.
// Shorter items read a narrower range of source rows, which is what keeps them in L2.
constexpr int HT_SEG = 256;

struct EpochWs;

enum {
  HT_S_PACKW = 0, HT_S_TNPART, HT_S_LOSS, HT_S_ACHUNK, HT_S_OCHUNK, HT_S_ZCHUNK, HT_S_DZCHUNK, HT_S_DACHUNK,
  HT_S_NBUF, HT_S_SPART, HT_S_LEAVE, HT_S_MISC, HT_S_TFULL, HT_S_TFULL2, HT_S_GATV, HT_S_GATE, HT_S_GATWS, HT_S_GATP,
  HT_S_LINK0, HT_S_LINK1, HT_S_LINK2, HT_S_SCAN, HT_S_RSORT, HT_N_SCRATCH
};

struct ht_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  bool own_stream = false;
  hipStream_t side[3] = {nullptr, nullptr, nullptr};  // input (gather / H2D), output (D2H), host-function streams
  std::string err;
  int64_t hbm_budget = 0;  // 0 = unlimited
  int64_t hbm_used = 0;
  std::vector<hipEvent_t> ev_pool;
  size_t ev_next = 0;
  EpochWs* ws = nullptr;  // buffers of the last ht_epoch
  // device scratch that calls keep between invocations (grow-only)
  int64_t graph_launches = 0; // epochs that ran as one HIP graph launch
  uint64_t scratch_gen = 0;   // bumped whenever a scratch slot is (re)allocated: captured pointers into scratch are stale then
  void* scratch[HT_N_SCRATCH] = {};
  size_t scratch_bytes[HT_N_SCRATCH] = {};
  // The device's statically allocated scratch array (ht_core.hip), its address taken once at ht_ctx_create.
  // While static_mode is set (inside ht_layer_fwd_static) ht_scratch hands out pieces of it and nothing allocates.
  unsigned char* static_base = nullptr;
  bool static_mode = false;
  size_t static_used = 0;
  size_t static_off[HT_N_SCRATCH] = {};
  size_t static_len[HT_N_SCRATCH] = {};
  // pinned host scratch (slots 0-2: D2H staging of gradient rows; HT_HS_READBACK: small counts read back by ht_partition)
  void* hscratch[4] = {nullptr, nullptr, nullptr, nullptr};
  size_t hscratch_bytes[4] = {0, 0, 0, 0};
  int xcd_contig = 0;     // 1: XCDs take contiguous parts of the item list instead of interleaving it
                          // (HT_XCD_CONTIG; measured slower at cfg2: 30.7 vs 26.0 ms per epoch)
  int no_link_fence = 0;  // 1: let aggregation kernels overlap link traffic (HT_NO_LINK_FENCE, for A/B runs)
  int link_blocks = 64;   // workgroups of a kernel that moves rows over the host link (HT_LINK_BLOCKS)
  int gather_blocks = 128; // workgroups of the neighbour-row gather from host memory (HT_GATHER_BLOCKS): beside a D2H
                           // copy the gather's read requests queue behind the write data, and more waves keep more in flight
  int link_memcpy = 0;    // hipMemcpyAsync for contiguous host<->device row ranges: 1 both ways, 2 to the host only, 3 from the host only (HT_LINK_MEMCPY)
  int slabs_fwd = 0, slabs_bwd = 0;  // caps on feature slabs (HT_SLABS_FWD / HT_SLABS_BWD), 0 = by width
  int agg_unroll = 4;     // HT_AGG_UNROLL: row reads in flight per lane (4 or 8)
  int agg_uniform = 1;    // HT_AGG_UNIFORM=0: no wave-uniform fast path for one-edge-per-step shapes
  int slab_align = 1;     // HT_SLAB_ALIGN=0: do not round slabs to whole cache lines
  int agg_phases = 1;     // HT_AGG_PHASES: slabs are spread over this many consecutive launches
  int64_t link_block_rows = (int64_t)1 << 20;   // HT_LINK_BLOCK_ROWS: rows per staged block of a host-resident tensor (GAT path)
  int agg_variant = 0;  // 0: feature slabs per XCD; 1: full-width rows per wave (HT_AGG_VARIANT, for A/B runs)
  int fuse_update = 0;  // HT_FUSE_UPDATE=1: layers that keep no aggregate run aggregate + transform as one kernel (A/B)
  int n_threads = 0;  // host threads for CPU-side accumulation (0 = chosen on first use)
};

int ht_set_err(ht_ctx* ctx, int code, const char* fmt, ...);

#define HT_HIP(ctx, call)                                                                  \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess)                                                                  \
      return ht_set_err((ctx), e_ == hipErrorOutOfMemory ? HT_ENOMEM : HT_EHIP, "%s: %s",  \
                        #call, hipGetErrorString(e_));                                     \
  } while (0)

#define HT_TRY(expr)            \
  do {                          \
    int rc_ = (expr);           \
    if (rc_ != HT_OK) return rc_; \
  } while (0)

#define HT_LAUNCH_CHECK(ctx) HT_HIP(ctx, hipGetLastError())

// HT_STATIC_SCRATCH_BYTES (hongtu.h): bytes of the statically allocated device scratch array that the
// allocation-free entry point works in.
void ht_static_begin(ht_ctx* ctx);   // ht_scratch serves from the static array until ht_static_end
void ht_static_end(ht_ctx* ctx);

// Device allocation with budget accounting.
int ht_dev_alloc(ht_ctx* ctx, void** out, size_t bytes);
void ht_dev_free(ht_ctx* ctx, void* p, size_t bytes);
// Grow-only scratch slot (kept on the context).
int ht_scratch(ht_ctx* ctx, int slot, size_t bytes, void** out);
// Grow-only pinned host scratch.
constexpr int HT_HS_READBACK = 3;
int ht_host_scratch(ht_ctx* ctx, int slot, size_t bytes, void** out);

template <typename T>
struct DevArr {
  T* p = nullptr;
  size_t n = 0;
  ht_ctx* ctx = nullptr;
  bool owned = true;   // false: a view into a block that another DevArr owns
  DevArr() = default;
  DevArr(const DevArr&) = delete;
  DevArr& operator=(const DevArr&) = delete;
  DevArr(DevArr&& o) noexcept : p(o.p), n(o.n), ctx(o.ctx), owned(o.owned) { o.p = nullptr; o.n = 0; }
  DevArr& operator=(DevArr&& o) noexcept {
    if (this != &o) {
      release();
      p = o.p; n = o.n; ctx = o.ctx; owned = o.owned;
      o.p = nullptr; o.n = 0;
    }
    return *this;
  }
  ~DevArr() { release(); }
  int alloc(ht_ctx* c, size_t count) {
    release();
    ctx = c;
    n = count;
    owned = true;
    if (count == 0) return HT_OK;
    return ht_dev_alloc(c, (void**)&p, count * sizeof(T));
  }
  void release() {
    if (p && owned) ht_dev_free(ctx, p, n * sizeof(T));
    p = nullptr;
    n = 0;
  }
  size_t bytes() const { return n * sizeof(T); }
};

// Arrays of one lifetime carved out of one device allocation: an allocation and its release cost tens of
// microseconds each whatever their size, and ht_partition makes dozens.  add() every array first, then
// alloc(), then take() them in the same order; every array starts on a 256-byte boundary.
struct DevBlock {
  DevArr<char> mem;
  size_t planned = 0, taken = 0;
  static size_t pad(size_t b) { return (b + 255) & ~(size_t)255; }
  template <typename T>
  void add(size_t count) { planned += pad(count * sizeof(T)); }
  int alloc(ht_ctx* c) { taken = 0; return mem.alloc(c, planned > 0 ? planned : 1); }
  template <typename T>
  void take(DevArr<T>& a, size_t count) {
    a.release();
    a.ctx = mem.ctx;
    a.owned = false;
    a.n = count;
    a.p = (T*)(mem.p + taken);
    taken += pad(count * sizeof(T));
  }
  void release() { mem.release(); planned = taken = 0; }
};

static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- primitives (ht_prims.hip) -------------------------------------------------------
// Exclusive prefix sum of n values into out[0..n); out[n] = total when want_total.
// Rates the epoch planner prices its choices with (measured on MI355X: host link beside compute,
// rows gathered per second by the aggregation kernel, in bytes).
constexpr double HT_LINK_BYTES_PER_S = 45e9;
constexpr double HT_GATHER_BYTES_PER_S = 15e12;

// Row pitch (in floats) of a library-allocated [rows x d] matrix: a multiple of 4 (16-byte
// vectors); in HBM, rows start on 128-byte cache lines when that costs at most 3 % more memory,
// so a feature slab never shares a line with the slab of another XCD; in pinned host memory rows
// start on 64-byte boundaries: a row read over the link then splits into whole 64-byte requests
// (rows at a 400-byte pitch were gathered at 22 GB/s beside a D2H copy that fell to 29 GB/s; at a
// 448-byte pitch 26-34 GB/s beside 46-50 GB/s).
inline int64_t ht_row_pitch(int32_t d, bool device) {
  const int64_t p4 = ((int64_t)d + 3) & ~(int64_t)3, p16 = ((int64_t)d + 15) & ~(int64_t)15, p32 = ((int64_t)d + 31) & ~(int64_t)31;
  if (!device) return p16;
  return p32 * 100 <= p4 * 103 ? p32 : p4;
}

int ht_scan_i32(ht_ctx* ctx, const int32_t* in, int64_t* out, int64_t n, bool want_total);
int ht_scan_i64(ht_ctx* ctx, const int64_t* in, int64_t* out, int64_t n, bool want_total);
// Stable LSD radix sort of 64-bit keys on bits [bit_lo, bit_hi).  keys and tmp
// have n entries; returns in *sorted which of the two holds the result.
int ht_radix_sort_u64(ht_ctx* ctx, uint64_t* keys, uint64_t* tmp, int64_t n, int bit_lo, int bit_hi,
                      uint64_t** sorted);
// Bitmap helpers: words are uint64, bit b of word w is element 64*w + b.
// pref[w] = number of set bits before word w; pref[nw] = total.
int ht_bitmap_prefix(ht_ctx* ctx, const uint64_t* bm, int64_t nw, int32_t* cnt_tmp, int64_t* pref);
// Writes the indices of set bits, ascending, to out (size pref[nw]).
int ht_bitmap_expand(ht_ctx* ctx, const uint64_t* bm, int64_t nw, const int64_t* pref, int32_t* out);

// ---- graph -------------------------------------------------------------------------------
// Work items of one aggregation direction of one chunk: a row with at most
// HT_SEG edges is one item; a longer row is cut into items of HT_SEG edges whose
// partial sums are added in item order by a second kernel.
struct ItemSet {
  DevArr<char> blob;          // one allocation behind the arrays below
  int32_t* row = nullptr;     // [n_items] row of the item (local to the chunk)
  int64_t* e0 = nullptr;      // [n_items] first edge, relative to the chunk's first edge
  int32_t* len = nullptr;     // [n_items] edges in the item (<= HT_SEG)
  int32_t* part = nullptr;    // [n_items] -1: the row's only item; else index of its partial sum
  int32_t* fx_row = nullptr;  // [n_fix] rows with several items
  int32_t* fx_part0 = nullptr;
  int32_t* fx_nseg = nullptr;
  int64_t n_items = 0, n_part = 0, n_fix = 0;
};

struct ChunkMeta {
  int64_t dst0 = 0, dst1 = 0;  // destination range
  int64_t e0 = 0, nnz = 0;     // edge range in the global CSC arrays
  int64_t ue0 = 0, nu = 0;     // range of distinct (destination, source) pairs in the merged arrays (= e0, nnz when not merged)
  int64_t nsrc = 0;            // |N_j|
  int64_t nbr_off = 0;         // offset of N_j in the nbr / slot arenas
  int64_t sptr_off = 0;        // offset of sptr_j in the sptr arena (nbr_off + j)
  int64_t n_reuse = 0, n_load = 0, n_leave = 0;
  int64_t reuse_off = 0, load_off = 0, leave_off = 0;
  ItemSet fwd, bwd;            // rows = destinations / rows = local sources
};

struct ht_graph {
  ht_ctx* ctx = nullptr;
  uint64_t serial = 0;         // unique per ht_partition call in this process: tells graphs at one address apart
  int64_t V = 0, Ep = 0;
  int32_t n = 0;
  int32_t add_self_loops = 1;
  bool single_leave = false;   // schedule-aware buffer that loads (and so releases) every row once per pass
  DevArr<int64_t> indptr;      // [V+1]
  DevArr<int32_t> col;         // [E'] global source ids
  DevArr<float> s;             // [V] D^-1/2
  std::vector<int64_t> bounds; // [n+1] host, in vertex-id order
  std::vector<int32_t> order;  // [n] schedule position -> chunk id (identity unless chunks were reorganised)
  std::vector<ChunkMeta> chunks;
  DevArr<int32_t> nbr;         // [v_ori] N_j lists
  DevArr<int32_t> col_local;   // [E']
  DevArr<int32_t> col_slot;    // [E'] buffer position of each edge's source
  DevArr<int64_t> sptr;        // [v_ori + n] per-chunk offsets, rebased to 0
  DevArr<int32_t> sdst;        // [E'] local destinations grouped by local source
  DevArr<int32_t> slot;        // [v_ori] buffer position of N_j[i]
  DevArr<int32_t> gslot;       // [v_ori] slot | (1<<31 when N_j[i] is newly loaded)
  DevArr<int32_t> reuse;       // [v_ori - v_load]
  DevArr<int32_t> load;        // [v_load]
  DevArr<int32_t> load_slot;   // [v_load]
  DevArr<int32_t> leave;       // [v_load] rows leaving after each chunk (everything still buffered after the last)
  DevArr<int32_t> leave_slot;  // [v_load]
  // Duplicate edges merged for the aggregation kernels (built when at least 5 % of the edges repeat
  // a pair): one entry per distinct pair, its multiplicity folded into the weight.  The arrays above
  // stay the canonical ones (export, parity).
  bool merged = false;
  int64_t n_unique = 0;
  DevArr<int64_t> uindptr;     // [V+1] row offsets in distinct-pair space
  DevArr<int32_t> ucol;        // [n_unique] source of each distinct pair, CSC order
  DevArr<int32_t> ucol_slot;   // [n_unique] its buffer position
  DevArr<float> uw_fwd;        // [n_unique] multiplicity * s[source]
  DevArr<float> umult;         // [n_unique] multiplicity (for rows already scaled in the buffer)
  DevArr<int64_t> usptr;       // [v_ori + n] per-chunk by-source offsets in distinct-pair space
  DevArr<int32_t> usdst;       // [n_unique] local destination of each distinct pair, by-source order
  DevArr<float> uw_bwd;        // [n_unique] multiplicity * s[destination]
  DevArr<float> umult_bwd;     // [n_unique] multiplicity, by-source order
  DevBlock blk_pairs, blk_chunks;   // the allocations behind the distinct-pair arrays and the per-chunk arenas
  DevArr<char> items_mem;           // the allocation behind the chunks' work-item lists
  int64_t v_ori = 0, v_ru = 0, v_load = 0;  // v_load: rows actually loaded per pass with this buffer
  int64_t max_nsrc = 0, max_ndst = 0, max_nnz = 0, max_fpart = 0, max_bpart = 0;
  int64_t cache_rows = 0;
  int32_t cache_policy = 0;    // HT_CACHE_*
  double partition_ms = 0.0;
  mutable std::vector<int32_t> leave_host;  // host copy of `leave`, made on first use by the CPU-side adds
  int64_t hbm_bytes() const;
};

// ---- compute kernels' host launchers -----------------------------------------------------
// Aggregation over work items (ht_spmm.hip).  One wave (or a lane group of it)
// owns an item; sums are taken in edge order, partial sums in item order.
struct SpmmArgs {
  // items
  const int32_t* it_row;
  const int64_t* it_e0;
  const int32_t* it_len;
  const int32_t* it_part;
  int64_t n_items;
  int64_t n_edges;        // edges covered by the items (for launch heuristics)
  const int32_t* fx_row;
  const int32_t* fx_part0;
  const int32_t* fx_nseg;
  int64_t n_fix;
  // edges
  const int32_t* idx;     // per edge: row of `src` to read (chunk-relative pointer)
  const float* ew;        // per-edge weight table indexed by idx (nullable: weight 1)
  const float* w_edge = nullptr;  // per-edge weights in edge order (takes precedence over ew)
  const float* src;       // source matrix
  int64_t src_ld;
  int32_t d;              // valid columns
  // output
  float* out;             // output matrix
  int64_t out_ld;
  const int32_t* out_idx; // row r -> output row (nullable: r); bit 31 set => overwrite even when accumulating
  const float* post;      // per-row factor
  const int32_t* post_idx;// row r -> index into post (nullable: r)
  int32_t accumulate;     // 1: out += value
  float* partial;         // [n_part x out_ld] workspace
  int relu = 0;           // clamp the finished row at 0 (only without accumulate)
  int max_slabs = 0;      // cap on the number of feature slabs (0 = by width)
  // optional timing of the two kernels (null: not timed)
  struct Timer* tm = nullptr;
  double* t_items = nullptr;
  double* t_fix = nullptr;
};
int ht_spmm_launch(ht_ctx* ctx, hipStream_t st, const SpmmArgs& a);
// Only the second kernel: rows fx_row[] = their partial rows added in item order (d, out*, partial, fx_* are read).
int ht_spmm_fix_launch(ht_ctx* ctx, hipStream_t st, const SpmmArgs& a);

// Row gather / scatter (ht_spmm.hip)
// dst[dst_idx[k]] = scale[src_idx[k]] * src[src_idx[k]]   (scale nullable)
int ht_gather_rows(ht_ctx* ctx, hipStream_t st, const float* src, int64_t src_ld, const int32_t* src_idx,
                   float* dst, int64_t dst_ld, const int32_t* dst_idx, int64_t n_rows, int32_t d,
                   const float* scale, int max_blocks = 0);
// Contiguous copy by a kernel with a small grid; src/dst may be device or GPU-addressable host memory.
int ht_copy_link(ht_ctx* ctx, hipStream_t st, void* dst, const void* src, size_t bytes, int blocks);
// dst[dst_idx[k]] += src[src_idx[k]]  (dst_idx unique inside one call)
int ht_add_rows(ht_ctx* ctx, hipStream_t st, const float* src, int64_t src_ld, const int32_t* src_idx,
                float* dst, int64_t dst_ld, const int32_t* dst_idx, int64_t n_rows, int32_t d);

// Dense transform (ht_gemm.hip)
// C[M x N] = A[M x K] B[K x N], optional ReLU, C rows pitch ldc.  B is row-major dense [K x N].
int ht_gemm_nn(ht_ctx* ctx, hipStream_t st, const float* A, int64_t lda, const float* B, float* C, int64_t ldc,
               int64_t M, int32_t K, int32_t N, int relu);
// C[M x K] = A[M x N] B[K x N]^T
int ht_gemm_nt(ht_ctx* ctx, hipStream_t st, const float* A, int64_t lda, const float* B, float* C, int64_t ldc,
               int64_t M, int32_t N, int32_t K, int accumulate);
// C[K x N] (+)= A[M x K]^T B[M x N]; fixed-order reduction over M slices.
int ht_gemm_tn(ht_ctx* ctx, hipStream_t st, const float* A, int64_t lda, const float* B, int64_t ldb, float* C,
               int64_t M, int32_t K, int32_t N, int accumulate);

// Aggregate + transform of one chunk in one kernel, the aggregate kept in LDS (ht_fused.hip)
int ht_agg_update_fused(ht_ctx* ctx, hipStream_t st, const ht_graph* g, const ChunkMeta& c, const float* H_in, int64_t in_ld,
                        int32_t d_in, const float* W, int32_t d_out, int relu, float* H_out, int64_t out_ld);

// Elementwise / loss (ht_elem.hip)
// dz = dh * [ref > 0]
int ht_relu_mask(ht_ctx* ctx, hipStream_t st, const float* dh, int64_t ld_dh, const float* ref, int64_t ld_ref,
                 float* dz, int64_t ld_dz, int64_t rows, int32_t cols);
int ht_softmax_ce(ht_ctx* ctx, hipStream_t st, const float* logits, int64_t ld, const int32_t* labels, int64_t V,
                  int32_t C, float* grad, int64_t ld_g, float* loss_dev /*1 float*/);
int ht_sgd(ht_ctx* ctx, hipStream_t st, float* W, const float* dW, int64_t n, float lr);
int ht_fill_zero(ht_ctx* ctx, hipStream_t st, void* p, size_t bytes);

// stats helpers: HIP-event pairs around phases, each on the stream that runs the phase
struct Timer {
  ht_ctx* ctx;
  hipStream_t st;  // default stream for begin()/end()
  bool on;
  struct Ent {
    hipEvent_t a, b;
    hipStream_t s;
    double* dst;
  };
  std::vector<Ent> ev;
  const double *only_lo = nullptr, *only_hi = nullptr;   // when set: time only accumulators inside [only_lo, only_hi)
  Timer(ht_ctx* c, hipStream_t s, bool enabled) : ctx(c), st(s), on(enabled) {}
  int last = -1;   // id of the pair opened by the last begin() (-1: that phase is not timed)
  void begin(double* acc) { last = begin_on(acc, st); }
  void end() { end_id(last); last = -1; }
  int begin_on(double* acc, hipStream_t s);  // returns an id for end_id (-1 when timing is off)
  void end_id(int id);
  int resolve();  // after the streams are synchronised
};
hipEvent_t ht_event(ht_ctx* ctx);

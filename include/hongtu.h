/*
 * hongtu.h -- C ABI of the MI355X-native hot path of partition-based
 * full-graph GCN training (one GPU).
 *
 * The calls follow the paper's statement of the problem (Alg. 1: graph,
 * features and parameterised layers in, updated layers out):
 *
 *   ht_partition   Sec. 4.1 (range chunks of destinations with all their
 *                  in-edges), Sec. 5.1 step 2 (reuse / load split between
 *                  adjacently scheduled chunks), Sec. 6 (in-place buffer
 *                  positions, topology rewritten to index the buffer).
 *   ht_layer_fwd   Alg. 2 (reuse + sparse load of neighbour rows),
 *                  Alg. 1 (forward of one layer, output to its home),
 *                  Eq. 2 (aggregate, then linear + ReLU).
 *   ht_layer_bwd   Alg. 1 (checkpoint reload, re-forward of the
 *                  update stage, backward), Alg. 3 (neighbour
 *                  gradients back to the gradient buffer), Sec. 2.3 (backward
 *                  of the update), Sec. 4.1 (backward of the aggregate).
 *   ht_epoch       Alg. 1 end to end with the recomputation-caching hybrid of
 *                  Sec. 4.2, a softmax cross-entropy downstream task and an SGD
 *                  parameter update.
 *
 * Conventions
 *   - Every function returns an int status: HT_OK (0) or a negative HT_E* code.
 *     Nothing throws across this boundary.  ht_strerror() names a code;
 *     ht_last_error() gives the detail of the last failure on a context.
 *   - Vertex tensors are fp32, row-major, [rows x cols] with a row pitch `ld`
 *     in floats; ld >= cols and ld % 4 == 0 (rows are read as 16-byte vectors).
 *     Columns cols..ld-1 are padding: never read as data, may be overwritten.
 *     Advice, not a requirement: a pitch of whole 64-byte blocks (ld % 16 == 0)
 *     for tensors in host memory, of whole 128-byte lines (ld % 32 == 0) in HBM;
 *     the library's own tensors are laid out so.
 *   - `loc` says where a tensor lives: HT_LOC_DEVICE (HBM of the context's GPU)
 *     or HT_LOC_HOST_PINNED (page-locked host memory the GPU can address, e.g.
 *     hipHostMalloc or torch pin_memory).  Plain pageable memory is not accepted.
 *   - The caller owns every tensor and weight buffer it passes and keeps it
 *     alive until ht_sync() returns.  The library owns ht_ctx, ht_graph and
 *     its workspaces.  Inputs are never modified except where marked in/out.
 *   - Work is enqueued on the context's stream (and side streams the library
 *     owns); results are complete after ht_sync(), or on return when a
 *     non-null ht_stats is passed (filling it needs a sync).
 *   - Without the GPU or the built library there is no fallback: calls fail.
 */
#ifndef HONGTU_H
#define HONGTU_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ht_ctx ht_ctx;
typedef struct ht_graph ht_graph;

enum {
  HT_OK = 0,
  HT_EINVAL = -1, /* bad argument (null pointer, negative size, id out of range) */
  HT_ENOMEM = -2, /* device or pinned allocation failed, or byte budget exceeded */
  HT_EHIP = -3,   /* a HIP runtime call failed; see ht_last_error()              */
  HT_ESHAPE = -4, /* tensor shape / pitch / location does not fit the call       */
  HT_ESTATE = -5  /* call not valid in the object's current state                */
};

enum { HT_LOC_DEVICE = 0, HT_LOC_HOST_PINNED = 1 };
#define HT_MAX_LAYERS 8

/* fp32 matrix view, see "Conventions". */
typedef struct {
  float *ptr;
  int64_t rows;
  int32_t cols;
  int64_t ld;
  int32_t loc;
} ht_tensor;

/* ------------------------------------------------------------------ context */

/* Create a context on GPU `device`.  `hip_stream` is a hipStream_t the caller
 * owns (e.g. torch's current stream) or NULL for a library-owned stream. */
int ht_ctx_create(ht_ctx **out, int device, void *hip_stream);
int ht_ctx_destroy(ht_ctx *ctx);
/* Block until all work enqueued through ctx has finished. */
int ht_sync(ht_ctx *ctx);
/* Cap on bytes the library may allocate in HBM through this context
 * (0 = no cap).  Exceeding it makes the allocating call return HT_ENOMEM. */
int ht_ctx_set_hbm_budget(ht_ctx *ctx, int64_t bytes);
/* Number of ht_epoch calls on this context that ran as one HIP graph launch
 * (ht_plan_opts.use_graph); -1 for a null context. */
int64_t ht_ctx_graph_launches(const ht_ctx *ctx);
const char *ht_strerror(int code);
const char *ht_last_error(const ht_ctx *ctx);

/* ---------------------------------------------------------------- partition */

enum { HT_BALANCE_EDGES = 0, HT_BALANCE_VERTICES = 1 };
enum { HT_PTR_DEVICE = 0, HT_PTR_HOST = 1 };
/* Which rows the in-place neighbour buffer keeps between chunks:
 *   HT_CACHE_ADJACENT  Sec. 5.1 step 2: rows of N_j ^ N_{j-1} stay, every other row is released
 *                      after its chunk, whatever the buffer's size
 *   HT_CACHE_FARTHEST  a row is released right after the last chunk that needs it; a row with a
 *                      later use is released only when the buffer (cache_rows rows) needs the
 *                      room, and then the rows whose next use lies farthest ahead in the chunk
 *                      schedule go first (equal next use: smaller id first).  The schedule is
 *                      known when the graph is partitioned, so this is the rule that loads the
 *                      fewest rows a buffer of that size can; in the backward pass the rows that
 *                      leave (Alg. 3) are spread over the pass instead of waiting for its end. */
enum { HT_CACHE_ADJACENT = 0, HT_CACHE_FARTHEST = 1 };

typedef struct {
  int32_t add_self_loops; /* 1: add one (v,v) entry per vertex                          */
  int32_t balance_mode;   /* HT_BALANCE_EDGES: b_j = min{v: indptr[v] >= ceil(j E'/n)};
                             HT_BALANCE_VERTICES: b_j = floor(j V / n)                  */
  int32_t ptr_loc;        /* where src/dst live: HT_PTR_DEVICE or HT_PTR_HOST (any host memory) */
  int32_t reorder_chunks; /* 1: schedule the chunks in the greedy max-overlap order of Alg. 4,
                             phase 2 (chunk 0 first, then always the unplaced chunk whose N_k
                             shares most vertices with the chunk placed last; ties: smallest
                             id); 0: in vertex-id order.  Chunk j below means schedule position j */
  int64_t cache_rows;     /* rows of the in-place neighbour buffer: 0 = max_j |N_j| (rows of
                             N_j ^ N_{j-1} are reused, the rest evicted, as in Sec. 5.1);
                             > 0 = that many rows (at least max_j |N_j|); -1 = as many rows as
                             there are distinct sources, with HT_CACHE_FARTHEST: every row is
                             loaded once per pass and stays until its last use               */
  int32_t cache_policy;   /* HT_CACHE_* (cache_rows = -1 implies HT_CACHE_FARTHEST)        */
  int32_t reserved;
} ht_part_opts;

/* Edge list (src[i] -> dst[i]), 0 <= id < V < 2^31, E >= 0, duplicates kept.
 * Builds, on the GPU: the CSC by destination with ascending sources inside a
 * destination; n_chunks contiguous destination ranges; per chunk j the
 * ascending unique source list N_j, every edge's position in N_j, the same
 * edges grouped by source for the backward pass, the reuse set N_j ^ N_{j-1},
 * the load set N_j \ N_{j-1} and a buffer position for every member of N_j
 * such that reused vertices keep theirs; and the row volumes V_ori, V_+ru.
 * src/dst stay the caller's and are not modified.  *out is library-owned. */
int ht_partition(ht_ctx *ctx, int64_t V, int64_t E, const int32_t *src, const int32_t *dst,
                 int32_t n_chunks, const ht_part_opts *opts, ht_graph **out);
int ht_graph_destroy(ht_graph *g);

typedef struct {
  int64_t V;
  int64_t E_stored; /* edges incl. added self-loops                    */
  int32_t n_chunks;
  int32_t reserved;
  int64_t v_ori;    /* sum_j |N_j|                       (Sec. 5.3)    */
  int64_t v_ru;     /* |N_0| + sum_{j>=1} |N_j \ N_{j-1}| (Sec. 5.3)    */
  double alpha;     /* replication factor v_ori / V       (Sec. 2.4)   */
  int64_t max_nsrc; /* max_j |N_j|                                      */
  int64_t max_ndst; /* max_j |V_j|                                      */
  int64_t max_nnz;  /* max_j E'_j                                       */
  int64_t cache_rows;
  int64_t hbm_bytes;    /* device bytes held by the graph object        */
  int64_t v_load;       /* rows loaded per pass with this buffer (= v_ru
                           unless cache_rows = -1)                      */
  double partition_ms;  /* wall time of ht_partition                    */
} ht_graph_info;

typedef struct {
  int64_t dst_begin, dst_end; /* V_j = [dst_begin, dst_end)  */
  int64_t nnz;                /* E'_j                        */
  int64_t n_src;              /* |N_j|                       */
  int64_t n_reuse, n_load;    /* rows of N_j already buffered / fetched (|N_j ^ N_{j-1}|, |N_j \ N_{j-1}| with HT_CACHE_ADJACENT) */
  int64_t n_leave;            /* rows released after this chunk (after the last: all still buffered) */
} ht_chunk_info;

/* Caller-allocated host arrays to receive chunk j; any pointer may be NULL to
 * skip that array.  Sizes follow ht_chunk_info. */
typedef struct {
  int64_t *indptr;    /* [|V_j|+1] CSC offsets rebased to 0                       */
  int32_t *col;       /* [E'_j]    global source of each edge, CSC order           */
  int32_t *nbr;       /* [|N_j|]   N_j ascending                                   */
  int32_t *col_local; /* [E'_j]    position of each edge's source in N_j           */
  int64_t *sptr;      /* [|N_j|+1] offsets of the by-source grouping               */
  int32_t *sdst;      /* [E'_j]    local destination (v - dst_begin) of each entry */
  int32_t *reuse;     /* [n_reuse] N_j ^ N_{j-1} ascending                         */
  int32_t *load;      /* [n_load]  N_j \ N_{j-1} ascending                         */
  int32_t *slot;      /* [|N_j|]   buffer position of N_j[i]                       */
  int32_t *leave;     /* [n_leave] rows released after this chunk, ascending       */
} ht_chunk_host;

int ht_graph_info_get(const ht_graph *g, ht_graph_info *out);
int ht_graph_chunk_info(const ht_graph *g, int32_t j, ht_chunk_info *out);
int ht_graph_export_chunk(const ht_graph *g, int32_t j, ht_chunk_host *out);
/* Global CSC and the normalisation s_v = D_v^{-1/2} (D_v = stored in-degree),
 * copied to caller-allocated host arrays (any may be NULL). */
int ht_graph_export_csc(const ht_graph *g, int64_t *indptr /*V+1*/, int32_t *col /*E_stored*/,
                        float *s /*V*/, int64_t *bounds /*n_chunks+1*/);
/* order[j] = id (position in vertex-id order) of the chunk scheduled at position j; the identity
 * unless reorder_chunks was set. */
int ht_graph_chunk_order(const ht_graph *g, int32_t *order /*n_chunks*/);

/* Partition reorganisation for m GPUs (Alg. 4, both phases) and the communication
 * volumes of Sec. 5.3, computed on one GPU as a planning step: sets of vertex
 * ids only, no second GPU is touched.  g holds m*n chunks in vertex-id order
 * (ht_partition with n_chunks = m*n, reorder_chunks = 0): chunk i*n + k is
 * subgraph k of partition i, and batch j of the initial layout is subgraph j of
 * every partition.
 *   Phase 1: the batches start as partition 0's subgraphs, U_j = N_0j; the
 *   partitions 1..m-1 in turn give batch j = 0..n-1 their not yet assigned
 *   subgraph k with the largest |N_ik ^ U_j|, and U_j grows by N_ik.
 *   Phase 2: batch 0 runs first, then always the unplaced batch whose union
 *   shares the most vertices with the union of the batch placed last.
 *   Ties go to the smallest index (the paper does not say).
 * layout (host, m*n entries): layout[i*n + j] = subgraph of partition i that
 * runs in batch j.  before / after (host, 3 entries each, may be NULL):
 * {V_ori, V_+p2p, V_+ru} in rows per pass for the initial and the reorganised
 * layout; with ht_comm_cost_model they give Eq. 4.  With m = 1 phase 1 is void,
 * the layout is the chunk order that reorder_chunks = 1 applies, and V_+p2p =
 * V_ori.  Temporary HBM: (m*n + n) * V / 8 bytes.  Synchronous.
 * HT_EINVAL: m < 1 or not a divisor of the chunk count; HT_ESTATE: g was built
 * with reorder_chunks = 1 or belongs to another context. */
int ht_graph_reorganize(ht_ctx *ctx, const ht_graph *g, int32_t m, int32_t *layout, int64_t *before,
                        int64_t *after);

/* -------------------------------------------------------------------- layer */

enum { HT_ACT_NONE = 0, HT_ACT_RELU = 1 };
/* How neighbour rows reach the aggregation (Alg. 2):
 *   HT_GATHER_AUTO    direct when H_in is in HBM, buffer otherwise
 *   HT_GATHER_DIRECT  read rows of H_in in place (H_in must be in HBM)
 *   HT_GATHER_BUFFER  keep N_j's rows in the in-place neighbour buffer: rows of
 *                     N_j ^ N_{j-1} stay, rows of N_j \ N_{j-1} are fetched from
 *                     H_in (HBM or pinned host) into freed positions */
enum { HT_GATHER_AUTO = 0, HT_GATHER_DIRECT = 1, HT_GATHER_BUFFER = 2 };
/* What the backward pass starts from (Sec. 4.2):
 *   HT_CKPT_AGG    the cached aggregate output a^l: AGGREGATE is skipped, only
 *                  the update stage is recomputed (the hybrid)
 *   HT_CKPT_INPUT  the layer input h^l: the aggregate is recomputed as well */
enum { HT_CKPT_AGG = 0, HT_CKPT_INPUT = 1 };
/* Order of the two stages of a layer.  Eq. 2 aggregates first and transforms the
 * aggregate, which is what Sec. 4.2's hybrid caches.  Because both stages are
 * linear, H' = act(A_hat (H W)) is the same function; it aggregates rows of
 * width d_out instead of d_in, which moves fewer bytes when d_out < d_in.
 *   HT_ORDER_AGG_FIRST     a = A_hat H ; H' = act(a W)            (Eq. 2 as printed)
 *   HT_ORDER_UPDATE_FIRST  t = H W     ; H' = act(A_hat t)
 * UPDATE_FIRST needs every vertex tensor of the call in HBM. */
enum { HT_ORDER_AGG_FIRST = 0, HT_ORDER_UPDATE_FIRST = 1, HT_ORDER_AUTO = 2 };

typedef struct {
  int32_t d_in, d_out;
  int32_t act;         /* HT_ACT_* applied after the linear transform */
  int32_t gather_mode; /* HT_GATHER_*                                  */
  int32_t ckpt_kind;   /* HT_CKPT_* (backward only)                    */
  int32_t order;       /* HT_ORDER_AGG_FIRST or HT_ORDER_UPDATE_FIRST  */
} ht_layer_desc;

/* Timings are HIP-event times on the stream that ran the work, summed over
 * the call; byte and row counters are exact. */
typedef struct {
  double t_total_ms;
  double t_gather_ms;     /* neighbour-row gather into the buffer            */
  double t_spmm_fwd_ms;   /* aggregation kernels, forward                    */
  double t_spmm_bwd_ms;   /* aggregation kernels, backward                   */
  double t_gemm_ms;       /* dense transform and its gradient GEMMs          */
  double t_loss_ms;
  double t_copy_ms;       /* contiguous H2D / D2H copies of chunk rows       */
  double t_cpu_accum_ms;  /* host-side gradient accumulation                 */
  double t_update_ms;
  int64_t n_spmm_fwd, n_spmm_bwd, n_gemm; /* kernel launches behind the times */
  int64_t edges;             /* stored edges aggregated (forward + backward)     */
  int64_t rows_loaded;       /* neighbour rows fetched into the buffer           */
  int64_t rows_reused;       /* neighbour rows reused in place                   */
  int64_t bytes_h2d;         /* host -> HBM bytes actually moved                 */
  int64_t bytes_d2h;         /* HBM -> host bytes actually moved                 */
  int64_t bytes_h2d_nodedup; /* what the neighbour loads would move per chunk without reuse */
  double spmm_fwd_alg_bytes; /* compulsory bytes of the forward aggregation launches */
  double spmm_bwd_alg_bytes;
  double gemm_flops;
  /* Forward aggregation per layer (index = layer in ht_epoch, 0 in ht_layer_*):
   * time of the main aggregation kernel alone (the partial-sum pass of cut
   * rows is in t_agg_fix_ms), its launches and compulsory bytes. */
  double t_agg_fwd_layer_ms[HT_MAX_LAYERS];
  double agg_fwd_layer_alg_bytes[HT_MAX_LAYERS];
  int64_t n_agg_fwd_layer[HT_MAX_LAYERS];
  double t_agg_fix_ms;
  /* GAT layers: neighbour softmax, destination pass, source pass (with its partial-row pass) */
  double t_gat_softmax_ms, t_gat_dst_ms, t_gat_src_ms;
  /* what ht_epoch's planner settled on: HT_INTER_*, then HT_RES_* of h^l, a^l and grad h^l
   * (0 after calls that plan nothing) */
  int32_t plan_inter, plan_res_h, plan_res_a, plan_res_g;
} ht_stats;

/* Forward of one layer over all chunks in schedule order:
 *   a[V_j] = s_v * sum_{e in in(v)} s_{u_e} H_in[u_e]      (aggregate, Eq. 2)
 *   H_out[V_j] = act(a[V_j] W)                              (update,   Eq. 2)
 * H_in [V x d_in], H_out [V x d_out]: device or pinned host.  W: device,
 * row-major [d_in x d_out], dense.  A_ckpt [V x d_in] (nullable): receives the
 * aggregate output as the recomputation checkpoint.
 * With desc->order = HT_ORDER_UPDATE_FIRST: t = H_in W for every vertex, then
 * H_out[V_j] = act(s_v * sum s_{u_e} t[u_e]); A_ckpt is not written (there is
 * no aggregate of width d_in); H_in and H_out must be in HBM, else HT_ESHAPE. */
int ht_layer_fwd(ht_ctx *ctx, const ht_graph *g, const ht_layer_desc *desc, const ht_tensor *H_in,
                 const float *W, ht_tensor *H_out, ht_tensor *A_ckpt, ht_stats *stats);

/* ht_layer_fwd for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * result as ht_layer_fwd (the same kernels in the same order), restricted to
 * the all-in-HBM path: H_in, H_out and A_ckpt (required) in device memory,
 * aggregate-first order, rows read in place (no neighbour buffer), no stats.
 * Its two scratch buffers (the tile-padded copy of W and the partial sums of
 * destination rows cut into several work items) live in an array that is part
 * of the library's code object: HT_STATIC_SCRATCH_BYTES (16 MiB) on every GPU
 * the library runs on, held until the process ends; its address is taken at
 * ht_ctx_create.  The call allocates nothing and frees nothing.  A layer that
 * needs more scratch than the array holds is refused with HT_ENOMEM before
 * anything is launched (ht_last_error says how much it needs); ht_layer_fwd
 * handles those.  All contexts on one GPU share the array and it keeps the last
 * call's contents (every word that is read is written first by the same call):
 * calls that overlap in time on one GPU, from any stream or context, race.
 * Asynchronous on the context's stream like ht_layer_fwd. */
#define HT_STATIC_SCRATCH_BYTES (16u << 20)
int ht_layer_fwd_static(ht_ctx *ctx, const ht_graph *g, const ht_layer_desc *desc, const ht_tensor *H_in,
                        const float *W, ht_tensor *H_out, ht_tensor *A_ckpt);

/* Backward of one layer over all chunks:
 *   z = a W (recomputed) ; dz = dH_out * [z > 0] (no mask when act = none)
 *   dW = a^T dz (overwritten) ; da = dz W^T ; dH_in[N_j] += s_u * sum s_v da[v]
 * ckpt: a^l (HT_CKPT_AGG) or h^l (HT_CKPT_INPUT).  H_out (nullable): when
 * given, the ReLU derivative is taken from [H_out > 0] and z is not recomputed.
 * dH_in (nullable: no input gradient wanted) is in/out: ACCUMULATED into, the
 * caller zeroes it.  All vertex tensors: device or pinned host.
 * With desc->order = HT_ORDER_UPDATE_FIRST (all tensors in HBM): ckpt is the
 * layer input h^l; dz as above (H_out is required when act = relu);
 * dt[N_j] += s_u * sum s_v dz[v] ; dW = h^T dt (overwritten) ; dH_in += dt W^T. */
int ht_layer_bwd(ht_ctx *ctx, const ht_graph *g, const ht_layer_desc *desc, const ht_tensor *ckpt,
                 const float *W, const ht_tensor *dH_out, const ht_tensor *H_out, ht_tensor *dH_in,
                 float *dW, ht_stats *stats);

/* ---------------------------------------------------------------- GAT layer */

/* One attention head of Eq. 3 over the stored edges (multi-edges count once
 * each, the self-loop is an edge like any other):
 *   t = H W ;  y_e = a_dst . t_v + a_src . t_u  for e = (u -> v)
 *   alpha_e = exp(LeakyReLU(y_e)) / sum over v's in-edges ;  H'_v = act(sum alpha_e t_u)
 * a_dst / a_src are the halves of a^l that meet the destination's / the
 * source's half of the concatenation [W h_v || W h_u]; the D^-1/2 weights of
 * the GCN path are not used. */
typedef struct {
  int32_t d_in, d_out; /* d_out <= 1024 */
  int32_t act;         /* HT_ACT_*                                  */
  float slope;         /* LeakyReLU slope for y <= 0, in [0, 1]     */
} ht_gat_desc;

/* Forward over all chunks.  H_in [V x d_in], H_out [V x d_out]: HBM or pinned
 * host memory.  W [d_in x d_out] row-major dense, a_dst, a_src [d_out]: device.
 * The parameterised rows t = H W of all vertices are held in HBM during the
 * call ([V x d_out] of library scratch), so a host-resident tensor is read or
 * written once, in contiguous row ranges, and no neighbour row crosses the
 * host link.  Nothing of size O(E) and no parameterised row outlives the call. */
int ht_gat_layer_fwd(ht_ctx *ctx, const ht_graph *g, const ht_gat_desc *desc, const ht_tensor *H_in,
                     const float *W, const float *a_dst, const float *a_src, ht_tensor *H_out,
                     ht_stats *stats);

/* Backward by recomputation from the layer input (Sec. 4.2: models with
 * computation on edges recompute instead of caching O(|E|) data): t, the
 * scores and the coefficients are computed again, then
 *   dz = dH_out * [H_out > 0] (no mask when act = none)
 *   dW, da_dst, da_src: overwritten;  dH_in (nullable): ACCUMULATED into.
 * H_out is the forward result (also read for the softmax's backward); every
 * vertex tensor in HBM or pinned host memory (host-resident ones are staged in
 * contiguous row ranges; dt [V x d_out] is library scratch in HBM);
 * dW [d_in x d_out], da_dst, da_src [d_out]: device. */
int ht_gat_layer_bwd(ht_ctx *ctx, const ht_graph *g, const ht_gat_desc *desc, const ht_tensor *H_in,
                     const float *W, const float *a_dst, const float *a_src, const ht_tensor *H_out,
                     const ht_tensor *dH_out, ht_tensor *dH_in, float *dW, float *da_dst, float *da_src,
                     ht_stats *stats);

/* where a class of vertex tensors lives (also used by ht_plan_opts below) */
enum { HT_RES_AUTO = 0, HT_RES_HBM = 1, HT_RES_HOST = 2 };
typedef struct {
  int32_t n_layers;    /* <= HT_MAX_LAYERS                                  */
  int32_t res_h;       /* HT_RES_AUTO / HT_RES_HBM: h^l, grad h^l in HBM;
                          HT_RES_HOST: h^1..h^{L-1} and their gradients in
                          pinned host memory (library-owned)                */
  const int32_t *dims; /* host, n_layers + 1 widths                         */
  float *const *W;     /* host arrays of n_layers device pointers, in/out   */
  float *const *a_dst; /* [dims[l+1]] each                                  */
  float *const *a_src;
  float lr;
  float slope;
} ht_gat_model;

/* Alg. 1 with GAT layers: forward (ReLU between layers, none after the
 * last), softmax cross-entropy over labelled vertices (labels[v] >= 0, device
 * int32 [V]), backward with each layer's intermediates recomputed from its
 * input, W -= lr dW and a -= lr da.  X [V x dims[0]]: HBM or pinned host.
 * loss_out: host float, valid on return (the call synchronises). */
int ht_gat_epoch(ht_ctx *ctx, const ht_graph *g, const ht_gat_model *model, const ht_tensor *X,
                 const int32_t *labels, float *loss_out, ht_stats *stats);

/* -------------------------------------------------------------------- epoch */

/* HT_INTER_AUTO picks per the byte budget; MASK keeps h^{l+1} in HBM and reads
 * ReLU' from it; HYBRID caches a^l and recomputes z = a W in the backward pass
 * (Sec. 4.2, Fig. 5(c)); RECOMPUTE keeps no a^l at all: the backward pass
 * gathers and aggregates again from h^l (Fig. 5(b)), then recomputes z unless
 * h^{l+1} is in HBM to read ReLU' from.  AUTO caches a^l in HBM when the byte
 * budget allows; when it does not, it compares what the host-side cache costs
 * (a^l written and read back over the host link, Fig. 5(c)) with what
 * recomputation costs (neighbour rows of a host-resident h^l fetched once
 * more, and the aggregation run again, Fig. 5(b)) at this GPU's measured link
 * and gather rates, and takes the cheaper one. */
enum { HT_INTER_AUTO = 0, HT_INTER_MASK = 1, HT_INTER_HYBRID = 2, HT_INTER_RECOMPUTE = 3 };

typedef struct {
  int32_t n_layers;
  int32_t reserved;
  const int32_t *dims; /* host, n_layers + 1 widths                        */
  float *const *W;     /* host array of n_layers device pointers, in/out   */
  float lr;
  int32_t reserved2;
} ht_model;

typedef struct {
  int32_t res_h;  /* residency of h^l (l >= 1) : HT_RES_*                  */
  int32_t res_a;  /* residency of the checkpoints a^l                      */
  int32_t res_g;  /* residency of the gradients grad h^l                   */
  int32_t inter;  /* HT_INTER_*                                            */
  int32_t gather_mode;
  int32_t order;  /* HT_ORDER_*: AGG_FIRST (0, Eq. 2 as printed) for every layer;
                   * UPDATE_FIRST / AUTO: update first in the layers whose tensors
                   * are all in HBM (AUTO: only where d_out < d_in)         */
  int64_t hbm_budget_bytes; /* 0 = what the device reports free, minus a margin */
  int32_t reuse_input_aggregate; /* 1: the caller promises that X and the graph are the same as in the
                   * previous ht_epoch call on this context.  a^0 = A_hat X does not depend on
                   * the parameters, so the copy the previous epoch cached for its backward pass
                   * is taken instead of gathering and aggregating layer 0 again (layer 0 then
                   * keeps the printed stage order whatever `order` says).  Ignored on the
                   * first epoch, after a change of shape, plan or X pointer, and with
                   * HT_INTER_RECOMPUTE.  Not part of the paper's method: 0 reproduces it. */
  int32_t use_graph; /* 1: when every tensor of the epoch is in HBM and no stats are asked for, the
                   * epoch's kernels are captured into a HIP graph on the second call with the same
                   * graph, X, labels, parameter pointers, lr and plan, and replayed from then on
                   * (same kernels, same order: same bits).  Ignored otherwise. */
  int32_t stats_detail; /* what a non-null ht_stats times with event pairs on the streams:
                   * HT_STATS_ALL (0) every phase of every chunk; HT_STATS_AGG_FWD (1) only the
                   * forward aggregation kernels (t_agg_fwd_layer_ms, t_spmm_fwd_ms), the other
                   * t_* fields stay 0.  Counters (rows, bytes, edges, flops) are filled either way.
                   * Events cost a few microseconds each: a few per cent of a cfg2-sized epoch. */
  int32_t reserved;
} ht_plan_opts;
enum { HT_STATS_ALL = 0, HT_STATS_AGG_FWD = 1 };

/* One training epoch (Alg. 1): forward over layers and chunks, softmax
 * cross-entropy averaged over labelled vertices (labels[v] >= 0; device int32
 * [V]), backward, W^l -= lr * dW^l.  X = h^0 [V x dims[0]].  *loss_out is
 * written on the host before return (the call synchronises). */
int ht_epoch(ht_ctx *ctx, const ht_graph *g, const ht_model *model, const ht_tensor *X,
             const int32_t *labels, const ht_plan_opts *plan, float *loss_out, ht_stats *stats);

/* Zeros in every row of t (pad columns included), wherever it lives; for the
 * gradient tensors that ht_layer_bwd / ht_gat_layer_bwd accumulate into.  The call
 * synchronises. */
int ht_tensor_zero(ht_ctx *ctx, ht_tensor *t);

/* Views of the buffers the last ht_epoch on ctx left behind (valid until the
 * next ht_epoch with another shape, or ht_ctx_destroy):
 *   kind 0: h^l (l = 1..L)   1: a^l (l = 0..L-1)   2: grad h^l (l = 1..L)
 *   kind 3: dW^l as a [dims[l] x dims[l+1]] device matrix (l = 0..L-1) */
enum { HT_BUF_H = 0, HT_BUF_A = 1, HT_BUF_GH = 2, HT_BUF_DW = 3 };
int ht_epoch_buffer(ht_ctx *ctx, int32_t kind, int32_t layer, ht_tensor *out);
/* Copy the data columns of t (device or pinned host) into the dense host array
 * dst [rows x cols]; waits for the context's work first. */
int ht_tensor_to_host(ht_ctx *ctx, const ht_tensor *t, float *dst);

/* Byte accounting of the residency planner for a model on V vertices, as
 * counted in Table 1 of the paper (fp32): vertex data = h^l and grad h^l for
 * l = 0..L; intermediate data = two d_l-wide tensors per hidden layer output
 * (l = 1..L-1: pre-activation and activation) and three d_L-wide ones at the
 * output layer (logits, class probabilities, their gradient). */
int ht_memory_model(int64_t V, int32_t n_layers, const int32_t *dims, double *vertex_bytes,
                    double *intermediate_bytes);
/* Vertex rows one chunk needs resident: (1 + alpha) * V / n   (Sec. 4.3). */
double ht_chunk_rows_model(int64_t V, int32_t n_chunks, double alpha);
/* Communication cost of one pass over the chunks, Eq. 4 of the paper, in seconds:
 *   C = V_+ru / T_hd + (V_ori - V_+p2p) / T_dd + (V_+p2p - V_+ru) / T_ru
 * with the volumes in rows of bytes_per_row bytes and the three throughputs
 * (host link, GPU-to-GPU, in-place reuse) in bytes per second.  On one GPU
 * V_+p2p = V_ori and the middle term is void.  Returns -1 for a non-positive
 * throughput whose term is not void, or volumes that do not satisfy
 * v_ru <= v_p2p <= v_ori. */
double ht_comm_cost_model(int64_t v_ori, int64_t v_p2p, int64_t v_ru, int64_t bytes_per_row, double t_hd,
                          double t_dd, double t_ru);

#ifdef __cplusplus
}
#endif
#endif /* HONGTU_H */

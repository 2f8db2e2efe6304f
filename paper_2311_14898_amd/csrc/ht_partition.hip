// ht_partition: edge list -> CSC by destination -> contiguous chunks -> per
// chunk dedup remap (unique sorted sources, local indices), by-source grouping
// for the backward pass, reuse / load split between adjacent chunks, in-place
// buffer positions, aggregation work items.  All on the GPU.
//
// Sec. 4.1 (chunks = destination ranges with all in-edges), Sec. 5.1 step 2
// (N_j ^ N_{j-1} reused, N_j \ N_{j-1} loaded), Sec. 5.3 (V_ori, V_+ru),
// Sec. 6 (same buffer position for duplicated vertices of adjacent chunks;
// loaded rows take freed positions; topology rewritten to buffer positions).
#include <algorithm>
#include <atomic>
#include <cstdlib>

#include "ht_internal.h"

namespace {

constexpr int TB = 256;
inline unsigned nblk(int64_t n, int tb = TB) { return (unsigned)((n + tb - 1) / tb); }

__global__ void k_check_ids(const int32_t* __restrict__ src, const int32_t* __restrict__ dst, int64_t E, int64_t V,
                            int32_t* __restrict__ flag) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= E) return;
  int32_t u = src[i], v = dst[i];
  if (u < 0 || v < 0 || u >= V || v >= V) *flag = 1;
}

__global__ void k_pack_keys(const int32_t* __restrict__ src, const int32_t* __restrict__ dst, int64_t E, int64_t V,
                            int bitsV, int self_loops, uint64_t* __restrict__ keys) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n = E + (self_loops ? V : 0);
  if (i >= n) return;
  uint64_t u, v;
  if (i < E) {
    u = (uint64_t)(uint32_t)src[i];
    v = (uint64_t)(uint32_t)dst[i];
  } else {
    u = v = (uint64_t)(i - E);
  }
  keys[i] = (v << bitsV) | u;
}

__global__ void k_low_bits(const uint64_t* __restrict__ keys, int64_t n, uint64_t mask, int32_t* __restrict__ out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (int32_t)(keys[i] & mask);
}

// keys sorted by row = key >> shift; ptr[q] = first index whose row >= q, ptr[nrows] = n.
__global__ void k_boundaries(const uint64_t* __restrict__ keys, int64_t n, int shift, int64_t nrows,
                             int64_t* __restrict__ ptr) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int64_t r = (int64_t)(keys[i] >> shift);
  const int64_t rp = i > 0 ? (int64_t)(keys[i - 1] >> shift) : -1;
  for (int64_t q = rp + 1; q <= r; ++q) ptr[q] = i;
  if (i == n - 1)
    for (int64_t q = r + 1; q <= nrows; ++q) ptr[q] = n;
}

__global__ void k_norm(const int64_t* __restrict__ indptr, int64_t V, float* __restrict__ s) {
  int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= V) return;
  const int64_t D = indptr[v + 1] - indptr[v];
  s[v] = D > 0 ? (float)(1.0 / sqrt((double)D)) : 0.f;
}

// b[j] = min{ v in [0, V] : indptr[v] >= target[j] }
__global__ void k_bounds(const int64_t* __restrict__ indptr, int64_t V, const int64_t* __restrict__ target, int n,
                         int64_t* __restrict__ b) {
  int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const int64_t t = target[j];
  int64_t lo = 0, hi = V;  // indptr[V] >= t always
  while (lo < hi) {
    int64_t mid = (lo + hi) >> 1;
    if (indptr[mid] >= t) hi = mid; else lo = mid + 1;
  }
  b[j] = lo;
}

// The set of sources of a chunk, N_j, as a bitmap.  Marking bits directly needs an atomic OR per entry, and the
// XCDs' L2s only agree on a word through device-scope accesses, which travel to the memory side: with a plain
// test first, then a device-scope test, then the atomic, a 14 M-entry chunk took 258 us (346 without the plain
// test) and a 9.8 M-entry chunk of a 23 M-vertex graph 467 us.  So entries mark a byte per vertex with plain
// stores instead (every writer stores the same 1, the caches merge bytes on write-back, nothing has to be
// coherent before the kernel ends), and a second kernel packs 64 bytes into a word and clears them for the next
// chunk.  A repeated source follows its first copy (sources ascend inside a destination) and is skipped; a byte
// seen set (a cached view can only lag behind) is not stored again.
__global__ void k_mark_bytes(const int32_t* __restrict__ col, int64_t nnz, uint8_t* seen) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= nnz) return;
  const uint32_t u = (uint32_t)col[t];
  if (t > 0 && (uint32_t)col[t - 1] == u) return;
  if (!seen[u]) seen[u] = 1;
}
// bm[w] = bit b set iff seen[64 w + b]; the bytes (0 or 1 each) are cleared.  Eight bytes become eight bits by
// one multiplication: byte k sits at bit 8k and the factor's term 2^(56 - 7k) moves it to bit 56 + k; no two
// (byte, term) pairs meet in one bit, so nothing carries.
__global__ void k_pack_seen(uint8_t* seen, uint64_t* __restrict__ bm, int64_t nw) {
  int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= nw) return;
  ulonglong2* p = reinterpret_cast<ulonglong2*>(seen + w * 64);
  uint64_t bits = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const ulonglong2 v = p[q];
    bits |= ((v.x * 0x0102040810204080ull) >> 56) << (16 * q);
    bits |= ((v.y * 0x0102040810204080ull) >> 56) << (16 * q + 8);
    if (v.x | v.y) p[q] = make_ulonglong2(0ull, 0ull);
  }
  bm[w] = bits;
}

// bm = the distinct values of col[0..nnz) as a bitmap of nw words; seen: nw * 64 zero bytes, zero again afterwards
int mark_sources(ht_ctx* ctx, hipStream_t st, const int32_t* col, int64_t nnz, uint8_t* seen, int64_t nw, uint64_t* bm) {
  if (nnz > 0) {
    k_mark_bytes<<<nblk(nnz), TB, 0, st>>>(col, nnz, seen);
    HT_LAUNCH_CHECK(ctx);
  }
  k_pack_seen<<<nblk(nw), TB, 0, st>>>(seen, bm, nw);   // writes every word of bm
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

// Sum of up to three per-thread counts over the grid into totals[0..2]: waves by shuffles, the block's four waves
// through LDS, one atomic add per block and total (with one add per wave the adds of a 23 M-bit bitmap, all to the
// same three words, took 180 us).  Launch with a bounded grid; the callers stride.
__device__ __forceinline__ void block_add3(unsigned long long a, unsigned long long b, unsigned long long c,
                                           unsigned long long* __restrict__ totals, int ntot) {
  __shared__ unsigned long long part[4][3];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    a += __shfl_down(a, o, 64);
    b += __shfl_down(b, o, 64);
    c += __shfl_down(c, o, 64);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    part[wave][0] = a;
    part[wave][1] = b;
    part[wave][2] = c;
  }
  __syncthreads();
  if ((int)threadIdx.x < ntot) {
    unsigned long long t = 0;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += part[w][threadIdx.x];
    if (t) atomicAdd(&totals[threadIdx.x], t);
  }
}
constexpr int POPC_GRID = 256;
inline unsigned popc_grid(int64_t nw) { return (unsigned)std::max<int64_t>(1, std::min<int64_t>(nblk(nw), POPC_GRID)); }

// totals[0] += popc(cur), totals[1] += popc(cur & prev), totals[2] += popc(cur & res)
__global__ void __launch_bounds__(256) k_popc3(const uint64_t* __restrict__ cur, const uint64_t* __restrict__ prev,
                                               const uint64_t* __restrict__ res, int64_t nw,
                                               unsigned long long* __restrict__ totals) {
  unsigned long long a = 0, b = 0, c = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nw; i += (int64_t)gridDim.x * blockDim.x) {
    const uint64_t w = cur[i];
    a += __popcll(w);
    b += __popcll(w & prev[i]);
    c += __popcll(w & res[i]);
  }
  block_add3(a, b, c, totals, 3);
}

// ---- row-buffer schedule with a known future (release for room, farthest next use first)
// nxt[i] = position of the next chunk after j that needs N_j[i] (n: none); chunks are visited last to first
__global__ void k_next_use(const int32_t* __restrict__ nbr, int64_t n, int32_t* __restrict__ last, int32_t j,
                           int32_t* __restrict__ nxt) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int32_t u = nbr[i];
  nxt[i] = last[u];
  last[u] = j;
}
__global__ void k_set_nu(const int32_t* __restrict__ nbr, int64_t n, const int32_t* __restrict__ nxt,
                         int32_t* __restrict__ nu) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) nu[nbr[i]] = nxt[i];
}
// totals[0] += |R u cur|, totals[1] += |R ^ cur|
__global__ void __launch_bounds__(256) k_popc_union(const uint64_t* __restrict__ R, const uint64_t* __restrict__ cur,
                                                    int64_t nw, unsigned long long* __restrict__ totals) {
  unsigned long long a = 0, b = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nw; i += (int64_t)gridDim.x * blockDim.x) {
    a += __popcll(R[i] | cur[i]);
    b += __popcll(R[i] & cur[i]);
  }
  block_add3(a, b, 0, totals, 2);
}
// hist[nu[u]] += 1 for every u in the candidate set (integer counts: order does not matter).
// nbins <= HIST_LDS_BINS: counted per block in LDS first, so the few global bins see one add per block.
constexpr int HIST_LDS_BINS = 4096;
__global__ void k_hist_nu(const uint64_t* __restrict__ cand, int64_t nw, const int32_t* __restrict__ nu, int nbins,
                          unsigned int* __restrict__ hist) {
  __shared__ unsigned int h[HIST_LDS_BINS];
  const bool local = nbins <= HIST_LDS_BINS;
  if (local) {
    for (int b = threadIdx.x; b < nbins; b += blockDim.x) h[b] = 0;
    __syncthreads();
  }
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nw; i += (int64_t)gridDim.x * blockDim.x) {
    uint64_t w = cand[i];
    while (w) {
      const int b = __ffsll((long long)w) - 1;
      w &= w - 1;
      const int32_t x = nu[i * 64 + b];
      if (local) atomicAdd(&h[x], 1u);
      else atomicAdd(&hist[x], 1u);
    }
  }
  if (local) {
    __syncthreads();
    for (int b = threadIdx.x; b < nbins; b += blockDim.x)
      if (h[b]) atomicAdd(&hist[b], h[b]);
  }
}
// gt = candidates whose next use lies beyond t, eq = candidates whose next use is t
__global__ void k_select_nu(const uint64_t* __restrict__ cand, int64_t nw, const int32_t* __restrict__ nu, int32_t t,
                            uint64_t* __restrict__ gt, uint64_t* __restrict__ eq) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nw) return;
  uint64_t w = cand[i], g = 0, e = 0;
  while (w) {
    const int b = __ffsll((long long)w) - 1;
    w &= w - 1;
    const int32_t x = nu[i * 64 + b];
    if (x > t) g |= 1ull << b;
    else if (x == t) e |= 1ull << b;
  }
  gt[i] |= g;      // the row may already hold the rows that left after their last use
  eq[i] = e;
}
// rows of N_j that no later chunk needs: set in bm, counted into *count
__global__ void k_mark_dead(const int32_t* __restrict__ nbr, int64_t n, const int32_t* __restrict__ nxt, int32_t never,
                            uint32_t* bm32, unsigned long long* __restrict__ count) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool dead = i < n && nxt[i] == never;
  if (dead) {
    const uint32_t u = (uint32_t)nbr[i];
    atomicOr(&bm32[u >> 5], 1u << (u & 31));
  }
  const unsigned long long m = __ballot(dead);
  if ((threadIdx.x & 63) == 0 && m) atomicAdd(count, (unsigned long long)__popcll(m));
}
// out |= the m members of eq with the smallest ids (pref = exclusive prefix of eq's per-word popcounts)
__global__ void k_take_first(const uint64_t* __restrict__ eq, const int64_t* __restrict__ pref, int64_t nw, int64_t m,
                             uint64_t* __restrict__ out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nw) return;
  int64_t room = m - pref[i];
  if (room <= 0) return;
  uint64_t w = eq[i], keep = 0;
  while (w && room > 0) {
    const uint64_t low = w & (~w + 1);
    keep |= low;
    w ^= low;
    --room;
  }
  out[i] |= keep;
}

// out[k] += popc(bms[k] & last) for every candidate bitmap k (grid.y = k)
__global__ void k_overlap(const uint64_t* __restrict__ bms, int64_t nw, const uint64_t* __restrict__ last,
                          unsigned long long* __restrict__ out) {
  const int k = blockIdx.y;
  const uint64_t* bm = bms + (int64_t)k * nw;
  unsigned long long a = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nw; i += (int64_t)gridDim.x * blockDim.x)
    a += __popcll(bm[i] & last[i]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_down(a, o, 64);
  if ((threadIdx.x & 63) == 0 && a) atomicAdd(&out[k], a);
}

__global__ void k_bm_or(uint64_t* __restrict__ acc, const uint64_t* __restrict__ x, int64_t nw) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nw) acc[i] |= x[i];
}

// op 0: a & b   1: a & ~b
__global__ void k_bm_op(const uint64_t* __restrict__ a, const uint64_t* __restrict__ b, int64_t nw, int op,
                        uint64_t* __restrict__ out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nw) out[i] = op == 0 ? (a[i] & b[i]) : (a[i] & ~b[i]);
}

// a &= ~b
__global__ void k_bm_clear(uint64_t* __restrict__ a, const uint64_t* __restrict__ b, int64_t nw) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nw) a[i] &= ~b[i];
}

// rank of each edge's source among the set bits = its position in N_j
__global__ void k_remap(const int32_t* __restrict__ col, int64_t nnz, const uint64_t* __restrict__ bm,
                        const int64_t* __restrict__ pref, int32_t* __restrict__ col_local) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= nnz) return;
  const uint32_t u = (uint32_t)col[t];
  const uint64_t w = bm[u >> 6];
  const uint64_t below = (u & 63) ? (w & (~0ull >> (64 - (u & 63)))) : 0ull;
  col_local[t] = (int32_t)(pref[u >> 6] + __popcll(below));
}

// key = (local source << 32) | local destination, one thread per edge
__global__ void k_set_i64(int64_t* p, int64_t v) { *p = v; }

// a[at[i]] and b[at[i]] (b may be null) for a handful of positions
__global__ void k_gather_offsets(const int64_t* __restrict__ a, const int64_t* __restrict__ b, const int64_t* __restrict__ at,
                                 int64_t n, int64_t* __restrict__ out_a, int64_t* __restrict__ out_b) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  out_a[i] = a[at[i]];
  out_b[i] = b ? b[at[i]] : 0;
}

__global__ void k_csr_keys(const int64_t* __restrict__ indptr, int64_t dst0, int64_t dst1, int64_t e0, int64_t nnz,
                           const int32_t* __restrict__ col_local, uint64_t* __restrict__ keys) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= nnz) return;
  const int64_t e = e0 + t;
  int64_t lo = dst0, hi = dst1;  // find the last v with indptr[v] <= e
  while (hi - lo > 1) {
    int64_t mid = (lo + hi) >> 1;
    if (indptr[mid] <= e) lo = mid; else hi = mid;
  }
  keys[t] = ((uint64_t)(uint32_t)col_local[t] << 32) | (uint64_t)(uint32_t)(lo - dst0);
}

// leave list of the previous chunk: remember the position, free it
__global__ void k_evict(const int32_t* __restrict__ leave, int64_t n, int32_t* __restrict__ vslot,
                        uint32_t* freebm32, int32_t* __restrict__ leave_slot) {
  int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n) return;
  const int32_t u = leave[k];
  const int32_t sl = vslot[u];
  leave_slot[k] = sl;
  vslot[u] = -1;
  atomicOr(&freebm32[(uint32_t)sl >> 5], 1u << (sl & 31));
}

__global__ void k_assign(const int32_t* __restrict__ load, int64_t n, const int32_t* __restrict__ freelist,
                         int32_t* __restrict__ vslot, uint32_t* freebm32, int32_t* __restrict__ load_slot) {
  int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n) return;
  const int32_t sl = freelist[k];
  vslot[load[k]] = sl;
  load_slot[k] = sl;
  atomicAnd(&freebm32[(uint32_t)sl >> 5], ~(1u << (sl & 31)));
}

__global__ void k_lookup_slots(const int32_t* __restrict__ nbr, int64_t n, const int32_t* __restrict__ vslot,
                               const uint64_t* __restrict__ prev_bm, int32_t* __restrict__ slot,
                               int32_t* __restrict__ gslot) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint32_t u = (uint32_t)nbr[i];
  const int32_t sl = vslot[u];
  slot[i] = sl;
  const bool was = (prev_bm[u >> 6] >> (u & 63)) & 1ull;
  gslot[i] = was ? sl : (int32_t)((uint32_t)sl | 0x80000000u);
}

__global__ void k_map_i32(const int32_t* __restrict__ idx, int64_t n, const int32_t* __restrict__ table,
                          int32_t* __restrict__ out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = table[idx[i]];
}

__global__ void k_items_count(const int64_t* __restrict__ ptr, int64_t nrows, int HT_SEG, int32_t* __restrict__ nseg,
                              int32_t* __restrict__ npart, int32_t* __restrict__ isfix) {
  int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= nrows) return;
  const int64_t len = ptr[r + 1] - ptr[r];
  const int32_t k = len <= HT_SEG ? 1 : (int32_t)((len + HT_SEG - 1) / HT_SEG);
  nseg[r] = k;
  npart[r] = k > 1 ? k : 0;
  isfix[r] = k > 1 ? 1 : 0;
}

__global__ void k_items_fill(const int64_t* __restrict__ ptr, int64_t ptr0, int64_t nrows, int HT_SEG,
                             const int64_t* __restrict__ it_base, const int64_t* __restrict__ part_base,
                             const int64_t* __restrict__ fix_base, int32_t* __restrict__ it_row,
                             int64_t* __restrict__ it_e0, int32_t* __restrict__ it_len, int32_t* __restrict__ it_part,
                             int32_t* __restrict__ fx_row, int32_t* __restrict__ fx_part0,
                             int32_t* __restrict__ fx_nseg) {
  int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= nrows) return;
  const int64_t b = ptr[r] - ptr0, len = ptr[r + 1] - ptr[r];
  const int64_t t0 = it_base[r];
  const int32_t k = (int32_t)(it_base[r + 1] - t0);
  const int64_t p0 = part_base[r];
  for (int32_t q = 0; q < k; ++q) {
    it_row[t0 + q] = (int32_t)r;
    it_e0[t0 + q] = b + (int64_t)q * HT_SEG;
    const int64_t rem = len - (int64_t)q * HT_SEG;
    it_len[t0 + q] = (int32_t)(rem < HT_SEG ? rem : HT_SEG);
    it_part[t0 + q] = k > 1 ? (int32_t)(p0 + q) : -1;
  }
  if (k > 1) {
    const int64_t f = fix_base[r];
    fx_row[f] = (int32_t)r;
    fx_part0[f] = (int32_t)p0;
    fx_nseg[f] = k;
  }
}

// ---- merging of duplicate edges (a multigraph's repeated (u -> v) entries are adjacent in both
// sorted orders): one entry per distinct pair with weight multiplicity * s.
__global__ void k_dup_flags_u32(const int32_t* __restrict__ col, int64_t n, int32_t* __restrict__ flag) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n) flag[e] = (e == 0 || col[e] != col[e - 1]) ? 1 : 0;
}
__global__ void k_row_start_flags(const int64_t* __restrict__ indptr, int64_t V, int64_t n, int32_t* __restrict__ flag) {
  int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v < V && indptr[v] < n) flag[indptr[v]] = 1;
}
__global__ void k_dup_flags_u64(const uint64_t* __restrict__ keys, int64_t n, int32_t* __restrict__ flag) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n) flag[e] = (e == 0 || keys[e] != keys[e - 1]) ? 1 : 0;
}
// upos[u] = position of the u-th flagged entry; upos[nU] = n is written by the host
__global__ void k_flag_positions(const int32_t* __restrict__ flag, const int64_t* __restrict__ rank, int64_t n,
                                 int64_t* __restrict__ upos) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n && flag[e]) upos[rank[e]] = e;
}
// forward: ucol, weights mult*s[src] (rows read in place) and mult (rows pre-scaled in the buffer)
__global__ void k_merge_fwd(const int64_t* __restrict__ upos, int64_t nU, const int32_t* __restrict__ col,
                            const float* __restrict__ s, int32_t* __restrict__ ucol, float* __restrict__ uw,
                            float* __restrict__ umult) {
  int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= nU) return;
  const int64_t e = upos[u];
  const float m = (float)(upos[u + 1] - e);
  const int32_t c = col[e];
  ucol[u] = c;
  uw[u] = m * s[c];
  umult[u] = m;
}
__global__ void k_uindptr(const int64_t* __restrict__ indptr, const int64_t* __restrict__ rank, int64_t V, int64_t n,
                          int64_t nU, int64_t* __restrict__ uindptr) {
  int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v > V) return;
  const int64_t e = indptr[v];
  uindptr[v] = e < n ? rank[e] : nU;
}
__global__ void k_gather_i32_at(const int64_t* __restrict__ pos, int64_t pos_off, int64_t n, const int32_t* __restrict__ table,
                                int32_t* __restrict__ out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = table[pos[i] - pos_off];
}
// backward: per distinct (local source, local destination): usdst, weight mult*s[dst], compacted keys
__global__ void k_merge_bwd(const int64_t* __restrict__ upos, int64_t nU, const uint64_t* __restrict__ keys,
                            const float* __restrict__ s_chunk, int32_t* __restrict__ usdst, float* __restrict__ uw,
                            float* __restrict__ umult, uint64_t* __restrict__ ukeys) {
  int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= nU) return;
  const int64_t t = upos[u];
  const float m = (float)(upos[u + 1] - t);
  const uint64_t k = keys[t];
  const int32_t d = (int32_t)(k & 0xFFFFFFFFull);
  usdst[u] = d;
  uw[u] = m * s_chunk[d];
  umult[u] = m;
  ukeys[u] = k;
}

// Dispatch order of work items: by the first row they read (edges of a row are
// sorted by that index), so items in flight together read neighbouring rows.
__global__ void k_item_keys(const int64_t* __restrict__ it_e0, const int32_t* __restrict__ it_len, int64_t n,
                            const int32_t* __restrict__ idx, uint64_t* __restrict__ keys) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  const uint32_t first = it_len[t] > 0 ? (uint32_t)idx[it_e0[t]] : 0u;
  keys[t] = ((uint64_t)first << 32) | (uint64_t)(uint32_t)t;
}

__global__ void k_item_permute(const uint64_t* __restrict__ keys, int64_t n, const int32_t* __restrict__ row,
                               const int64_t* __restrict__ e0, const int32_t* __restrict__ len,
                               const int32_t* __restrict__ part, int32_t* __restrict__ row_o,
                               int64_t* __restrict__ e0_o, int32_t* __restrict__ len_o, int32_t* __restrict__ part_o) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  const uint32_t from = (uint32_t)(keys[t] & 0xFFFFFFFFull);
  row_o[t] = row[from];
  e0_o[t] = e0[from];
  len_o[t] = len[from];
  part_o[t] = part[from];
}

int bits_for(int64_t n) {  // bits needed for values 0..n-1 (at least 1)
  int b = 1;
  while (((int64_t)1 << b) < n) ++b;
  return b;
}

struct ItemTmp {
  DevBlock blk;
  DevArr<int32_t> nseg, npart, isfix;
  DevArr<int64_t> it_base, part_base, fix_base;
  DevArr<char> stage;   // items in row order, before they are permuted into dispatch order
  int64_t* totals = nullptr;   // pinned host memory for the three counts of a build_items call (set by the caller)
  // the graph's block for all work-item lists (set by the caller): a list takes the next bytes of it, or an
  // allocation of its own when the block is full
  char* arena = nullptr;
  size_t arena_cap = 0, arena_off = 0;
  int alloc(ht_ctx* ctx, int64_t maxrows) {
    for (int k = 0; k < 3; ++k) blk.add<int32_t>(maxrows);
    for (int k = 0; k < 3; ++k) blk.add<int64_t>(maxrows + 1);
    HT_TRY(blk.alloc(ctx));
    blk.take(nseg, maxrows);
    blk.take(npart, maxrows);
    blk.take(isfix, maxrows);
    blk.take(it_base, maxrows + 1);
    blk.take(part_base, maxrows + 1);
    blk.take(fix_base, maxrows + 1);
    return HT_OK;
  }
};

// ptr: device offsets of nrows+1 entries; ptr0: value to subtract so item edges are chunk-relative.
// idx: the chunk's per-edge row index array (what the aggregation reads), idx_range: its value range.
// keysA/keysB: scratch of at least n_items entries each.
int build_items(ht_ctx* ctx, ItemTmp& t, const int64_t* ptr, int64_t ptr0, int64_t nrows, const int32_t* idx,
                int64_t idx_range, uint64_t* keysA, uint64_t* keysB, bool order, int seg, ItemSet* out) {
  out->n_items = out->n_part = out->n_fix = 0;
  if (nrows == 0) return HT_OK;
  hipStream_t st = ctx->stream;
  k_items_count<<<nblk(nrows), TB, 0, st>>>(ptr, nrows, seg, t.nseg.p, t.npart.p, t.isfix.p);
  HT_LAUNCH_CHECK(ctx);
  HT_TRY(ht_scan_i32(ctx, t.nseg.p, t.it_base.p, nrows, true));
  HT_TRY(ht_scan_i32(ctx, t.npart.p, t.part_base.p, nrows, true));
  HT_TRY(ht_scan_i32(ctx, t.isfix.p, t.fix_base.p, nrows, true));
  int64_t* tot = t.totals;   // pinned: the three copies are queued without a stall each
  HT_HIP(ctx, hipMemcpyAsync(&tot[0], t.it_base.p + nrows, 8, hipMemcpyDeviceToHost, st));
  HT_HIP(ctx, hipMemcpyAsync(&tot[1], t.part_base.p + nrows, 8, hipMemcpyDeviceToHost, st));
  HT_HIP(ctx, hipMemcpyAsync(&tot[2], t.fix_base.p + nrows, 8, hipMemcpyDeviceToHost, st));
  HT_HIP(ctx, hipStreamSynchronize(st));
  out->n_items = tot[0];
  out->n_part = tot[1];
  out->n_fix = tot[2];
  // one allocation: e0 (8 B) first, then the 4-byte arrays
  const size_t ni = (size_t)tot[0], nf = (size_t)tot[2];
  const size_t bytes = ni * 8 + ni * 4 * 3 + nf * 4 * 3;
  if (t.arena && t.arena_off + DevBlock::pad(bytes) <= t.arena_cap) {
    out->blob.release();
    out->blob.ctx = ctx;
    out->blob.owned = false;
    out->blob.p = t.arena + t.arena_off;
    out->blob.n = bytes;
    t.arena_off += DevBlock::pad(bytes);
  } else {
    HT_TRY(out->blob.alloc(ctx, bytes));
  }
  struct Lay { int64_t* e0; int32_t *row, *len, *part, *fx_row, *fx_part0, *fx_nseg; };
  auto carve = [&](char* p) {
    Lay l;
    l.e0 = (int64_t*)p; p += ni * 8;
    l.row = (int32_t*)p; p += ni * 4;
    l.len = (int32_t*)p; p += ni * 4;
    l.part = (int32_t*)p; p += ni * 4;
    l.fx_row = (int32_t*)p; p += nf * 4;
    l.fx_part0 = (int32_t*)p; p += nf * 4;
    l.fx_nseg = (int32_t*)p;
    return l;
  };
  const Lay fin = carve(out->blob.p);
  out->e0 = fin.e0; out->row = fin.row; out->len = fin.len; out->part = fin.part;
  out->fx_row = fin.fx_row; out->fx_part0 = fin.fx_part0; out->fx_nseg = fin.fx_nseg;
  const bool sorted_items = order && ni > 1;
  // Items are made in row order; when they are to be dispatched in the order of the first row they read, they
  // are made in a staging block that outlives the chunk (no allocation per chunk) and permuted into place.
  Lay made = fin;
  if (sorted_items) {
    if (t.stage.n < bytes) HT_TRY(t.stage.alloc(ctx, bytes + bytes / 4));
    made = carve(t.stage.p);
    made.fx_row = fin.fx_row; made.fx_part0 = fin.fx_part0; made.fx_nseg = fin.fx_nseg;   // cut-row lists keep row order
  }
  k_items_fill<<<nblk(nrows), TB, 0, st>>>(ptr, ptr0, nrows, seg, t.it_base.p, t.part_base.p, t.fix_base.p, made.row,
                                          made.e0, made.len, made.part, made.fx_row, made.fx_part0, made.fx_nseg);
  HT_LAUNCH_CHECK(ctx);
  if (sorted_items) {
    k_item_keys<<<nblk((int64_t)ni), TB, 0, st>>>(made.e0, made.len, (int64_t)ni, idx, keysA);
    HT_LAUNCH_CHECK(ctx);
    uint64_t* sorted = nullptr;
    HT_TRY(ht_radix_sort_u64(ctx, keysA, keysB, (int64_t)ni, 32, 32 + bits_for(idx_range), &sorted));
    k_item_permute<<<nblk((int64_t)ni), TB, 0, st>>>(sorted, (int64_t)ni, made.row, made.e0, made.len, made.part, fin.row,
                                                    fin.e0, fin.len, fin.part);
    HT_LAUNCH_CHECK(ctx);
  }
  return HT_OK;
}

int partition_impl(ht_ctx* ctx, int64_t V, int64_t E, const int32_t* src_in, const int32_t* dst_in, int32_t n,
                   const ht_part_opts* opts, ht_graph* g) {
  hipStream_t st = ctx->stream;
  const int self_loops = opts ? (opts->add_self_loops != 0) : 1;
  const int mode = opts ? opts->balance_mode : HT_BALANCE_EDGES;
  const int ptr_loc = opts ? opts->ptr_loc : HT_PTR_DEVICE;
  const int64_t Ep = E + (self_loops ? V : 0);
  // the per-edge kernels take one thread per stored edge, and a launch holds fewer than 2^32 threads
  if (Ep >= ((int64_t)1 << 32) - 4096)
    return ht_set_err(ctx, HT_EINVAL, "ht_partition: %lld stored edges; fewer than 2^32 are supported", (long long)Ep);
  g->ctx = ctx;
  g->V = V;
  g->Ep = Ep;
  g->n = n;
  g->add_self_loops = self_loops;
  // pinned host memory for the small counts read back from the device: 8 words for the work-item counts,
  // then three lists of n + 1 boundary values
  int64_t* hpin = nullptr;
  {
    void* hp = nullptr;
    HT_TRY(ht_host_scratch(ctx, HT_HS_READBACK, (size_t)(8 + 3 * ((size_t)n + 1)) * 8, &hp));
    hpin = (int64_t*)hp;
  }

  // ---- edge list on the device
  DevArr<int32_t> src_copy, dst_copy;
  const int32_t* src = src_in;
  const int32_t* dst = dst_in;
  if (ptr_loc == HT_PTR_HOST && E > 0) {
    HT_TRY(src_copy.alloc(ctx, E));
    HT_TRY(dst_copy.alloc(ctx, E));
    HT_HIP(ctx, hipMemcpyAsync(src_copy.p, src_in, E * 4, hipMemcpyHostToDevice, st));
    HT_HIP(ctx, hipMemcpyAsync(dst_copy.p, dst_in, E * 4, hipMemcpyHostToDevice, st));
    src = src_copy.p;
    dst = dst_copy.p;
  }
  if (E > 0) {
    DevArr<int32_t> flag;
    HT_TRY(flag.alloc(ctx, 1));
    HT_HIP(ctx, hipMemsetAsync(flag.p, 0, 4, st));
    k_check_ids<<<nblk(E), TB, 0, st>>>(src, dst, E, V, flag.p);
    HT_LAUNCH_CHECK(ctx);
    int32_t bad = 0;
    HT_HIP(ctx, hipMemcpyAsync(&bad, flag.p, 4, hipMemcpyDeviceToHost, st));
    HT_HIP(ctx, hipStreamSynchronize(st));
    if (bad) return ht_set_err(ctx, HT_EINVAL, "ht_partition: a vertex id is outside [0, V)");
  }

  // ---- CSC by (destination, source)
  const int bitsV = bits_for(V);
  DevArr<uint64_t> keysA, keysB;
  const size_t nkeys = (size_t)std::max<int64_t>(std::max(Ep, V), 1) + 64;  // also holds one key per work item
  HT_TRY(keysA.alloc(ctx, nkeys));
  HT_TRY(keysB.alloc(ctx, nkeys));
  HT_TRY(g->indptr.alloc(ctx, (size_t)V + 1));
  HT_TRY(g->col.alloc(ctx, (size_t)(Ep > 0 ? Ep : 1)));
  HT_TRY(g->s.alloc(ctx, (size_t)V));
  HT_HIP(ctx, hipMemsetAsync(g->indptr.p, 0, (V + 1) * 8, st));
  if (Ep > 0) {
    k_pack_keys<<<nblk(Ep), TB, 0, st>>>(src, dst, E, V, bitsV, self_loops, keysA.p);
    HT_LAUNCH_CHECK(ctx);
    uint64_t* sorted = nullptr;
    HT_TRY(ht_radix_sort_u64(ctx, keysA.p, keysB.p, Ep, 0, 2 * bitsV, &sorted));
    k_low_bits<<<nblk(Ep), TB, 0, st>>>(sorted, Ep, ((uint64_t)1 << bitsV) - 1, g->col.p);
    HT_LAUNCH_CHECK(ctx);
    k_boundaries<<<nblk(Ep), TB, 0, st>>>(sorted, Ep, bitsV, V, g->indptr.p);
    HT_LAUNCH_CHECK(ctx);
  }
  k_norm<<<nblk(V), TB, 0, st>>>(g->indptr.p, V, g->s.p);
  HT_LAUNCH_CHECK(ctx);
  src_copy.release();
  dst_copy.release();

  // ---- duplicate edges: count the distinct (destination, source) pairs; merge when it pays
  const char* mg_env = getenv("HT_MERGE_DUPS");
  const bool merge_allowed = !(mg_env && atoi(mg_env) == 0);
  // flags and their ranks live in the two key buffers, which are idle between the sort above and the per-chunk
  // sorts below (releasing 12 bytes per edge of separate arrays took 49 ms on a 1.3 G-edge graph)
  struct { int32_t* p; } dflag{(int32_t*)keysA.p};
  struct { int64_t* p; } drank{(int64_t*)keysB.p};
  DevArr<int64_t> upos;
  int64_t nU = Ep;
  g->merged = false;
  if (merge_allowed && Ep > 0) {
    k_dup_flags_u32<<<nblk(Ep), TB, 0, st>>>(g->col.p, Ep, dflag.p);
    HT_LAUNCH_CHECK(ctx);
    k_row_start_flags<<<nblk(V), TB, 0, st>>>(g->indptr.p, V, Ep, dflag.p);
    HT_LAUNCH_CHECK(ctx);
    HT_TRY(ht_scan_i32(ctx, dflag.p, drank.p, Ep, true));
    HT_HIP(ctx, hipMemcpyAsync(&nU, drank.p + Ep, 8, hipMemcpyDeviceToHost, st));
    HT_HIP(ctx, hipStreamSynchronize(st));
    // merged arrays cost 16 B per distinct pair: worth it from about 5 % duplicates
    if ((double)nU <= 0.95 * (double)Ep) {
      g->merged = true;
      g->n_unique = nU;
      HT_TRY(upos.alloc(ctx, (size_t)nU + 1));
      {
        DevBlock& b = g->blk_pairs;
        b.add<int64_t>((size_t)V + 1);
        for (int k = 0; k < 7; ++k) b.add<int32_t>((size_t)nU);
        HT_TRY(b.alloc(ctx));
        b.take(g->uindptr, (size_t)V + 1);
        b.take(g->ucol, (size_t)nU);
        b.take(g->ucol_slot, (size_t)nU);
        b.take(g->uw_fwd, (size_t)nU);
        b.take(g->umult, (size_t)nU);
        b.take(g->usdst, (size_t)nU);
        b.take(g->uw_bwd, (size_t)nU);
        b.take(g->umult_bwd, (size_t)nU);
      }
      k_flag_positions<<<nblk(Ep), TB, 0, st>>>(dflag.p, drank.p, Ep, upos.p);
      HT_LAUNCH_CHECK(ctx);
      k_set_i64<<<1, 1, 0, st>>>(upos.p + nU, Ep);
      HT_LAUNCH_CHECK(ctx);
      k_merge_fwd<<<nblk(nU), TB, 0, st>>>(upos.p, nU, g->col.p, g->s.p, g->ucol.p, g->uw_fwd.p, g->umult.p);
      HT_LAUNCH_CHECK(ctx);
      k_uindptr<<<nblk(V + 1), TB, 0, st>>>(g->indptr.p, drank.p, V, Ep, nU, g->uindptr.p);
      HT_LAUNCH_CHECK(ctx);
      HT_HIP(ctx, hipStreamSynchronize(st));
    }
  }

  // ---- chunk boundaries
  g->bounds.assign(n + 1, 0);
  g->bounds[n] = V;
  if (mode == HT_BALANCE_VERTICES) {
    for (int j = 1; j < n; ++j) g->bounds[j] = (int64_t)(((__int128)j * V) / n);
  } else if (n > 1) {
    std::vector<int64_t> target(n - 1);
    for (int j = 1; j < n; ++j) target[j - 1] = (int64_t)((((__int128)j * Ep) + n - 1) / n);
    DevArr<int64_t> dt, db;
    HT_TRY(dt.alloc(ctx, n - 1));
    HT_TRY(db.alloc(ctx, n - 1));
    HT_HIP(ctx, hipMemcpyAsync(dt.p, target.data(), (n - 1) * 8, hipMemcpyHostToDevice, st));
    k_bounds<<<nblk(n - 1), TB, 0, st>>>(g->indptr.p, V, dt.p, n - 1, db.p);
    HT_LAUNCH_CHECK(ctx);
    HT_HIP(ctx, hipMemcpyAsync(&g->bounds[1], db.p, (n - 1) * 8, hipMemcpyDeviceToHost, st));
    HT_HIP(ctx, hipStreamSynchronize(st));
  }
  // edge offsets of the chunk boundaries, in both edge spaces: one gather, one copy back
  std::vector<int64_t> eoff(n + 1), ueoff(n + 1, 0);
  {
    const size_t nb1 = (size_t)n + 1;
    DevArr<int64_t> dq;
    HT_TRY(dq.alloc(ctx, 3 * nb1));
    int64_t* hb = hpin + 8;
    std::copy(g->bounds.begin(), g->bounds.end(), hb);
    HT_HIP(ctx, hipMemcpyAsync(dq.p, hb, nb1 * 8, hipMemcpyHostToDevice, st));
    k_gather_offsets<<<nblk((int64_t)nb1), TB, 0, st>>>(g->indptr.p, g->merged ? g->uindptr.p : nullptr, dq.p, (int64_t)nb1,
                                                       dq.p + nb1, dq.p + 2 * nb1);
    HT_LAUNCH_CHECK(ctx);
    HT_HIP(ctx, hipMemcpyAsync(hb + nb1, dq.p + nb1, 2 * nb1 * 8, hipMemcpyDeviceToHost, st));
    HT_HIP(ctx, hipStreamSynchronize(st));
    std::copy(hb + nb1, hb + 2 * nb1, eoff.begin());
    if (g->merged) std::copy(hb + 2 * nb1, hb + 3 * nb1, ueoff.begin());
  }
  g->chunks.clear();
  g->chunks.resize(n);
  for (int j = 0; j < n; ++j) {
    ChunkMeta& c = g->chunks[j];
    c.dst0 = g->bounds[j];
    c.dst1 = g->bounds[j + 1];
    c.e0 = eoff[j];
    c.nnz = eoff[j + 1] - eoff[j];
    c.ue0 = g->merged ? ueoff[j] : c.e0;
    c.nu = g->merged ? ueoff[j + 1] - ueoff[j] : c.nnz;
    g->max_ndst = std::max(g->max_ndst, c.dst1 - c.dst0);
    g->max_nnz = std::max(g->max_nnz, c.nnz);
  }

  // a buffer with room for every distinct source is the schedule-aware buffer at that size
  const bool keep_all = opts && opts->cache_rows == -1;
  const bool far_first = (opts && opts->cache_policy == HT_CACHE_FARTHEST) || keep_all;
  const int64_t nw = ceil_div64(V, 64);

  // ---- chunk reorganisation (Alg. 4, phase 2; one GPU, so a batch is one chunk): the first chunk
  // stays first, then the unplaced chunk whose neighbour set overlaps most with the chunk placed last
  // comes next (ties: smallest id).  All n neighbour bitmaps are kept for the n-1 greedy steps.
  g->order.resize(n);
  for (int j = 0; j < n; ++j) g->order[j] = j;
  // The chunks' neighbour bitmaps (bit u of row j: u is in N_j) are needed by the reorganisation, the counting
  // pass, the buffer simulation and the list pass.  When all n of them fit a modest share of the free memory
  // they are marked once and kept, row = original chunk id; otherwise each use marks its own again.
  DevArr<uint8_t> seen;   // one byte per vertex, zero between two uses
  HT_TRY(seen.alloc(ctx, (size_t)nw * 64));
  HT_HIP(ctx, hipMemsetAsync(seen.p, 0, (size_t)nw * 64, st));
  auto mark_chunk = [&](const ChunkMeta& c, uint64_t* bm) -> int {
    return mark_sources(ctx, st, g->col.p + c.e0, c.nnz, seen.p, nw, bm);
  };
  DevArr<uint64_t> allbm;
  {
    const size_t need = (size_t)n * (size_t)nw * 8;
    size_t free_b = 0, total_b = 0;
    HT_HIP(ctx, hipMemGetInfo(&free_b, &total_b));
    const bool want_reorder = opts && opts->reorder_chunks && n > 2;
    if (want_reorder || (need <= ((size_t)2 << 30) && need <= free_b / 16)) {
      HT_TRY(allbm.alloc(ctx, (size_t)n * nw));
      for (int j = 0; j < n; ++j) HT_TRY(mark_chunk(g->chunks[j], allbm.p + (size_t)j * nw));
    }
  }
  if (opts && opts->reorder_chunks && n > 2) {
    uint64_t* bms = allbm.p;
    DevArr<unsigned long long> ov;
    HT_TRY(ov.alloc(ctx, n));
    std::vector<unsigned long long> hov(n);
    std::vector<char> placed(n, 0);
    placed[0] = 1;
    const unsigned gx = (unsigned)std::min<int64_t>(ceil_div64(nw, TB), 64);
    for (int j = 1; j < n; ++j) {
      HT_HIP(ctx, hipMemsetAsync(ov.p, 0, (size_t)n * 8, st));
      k_overlap<<<dim3(gx, n), TB, 0, st>>>(bms, nw, bms + (size_t)g->order[j - 1] * nw, ov.p);
      HT_LAUNCH_CHECK(ctx);
      HT_HIP(ctx, hipMemcpyAsync(hov.data(), ov.p, (size_t)n * 8, hipMemcpyDeviceToHost, st));
      HT_HIP(ctx, hipStreamSynchronize(st));
      int best = -1;
      for (int k = 0; k < n; ++k)
        if (!placed[k] && (best < 0 || hov[k] > hov[best])) best = k;
      g->order[j] = best;
      placed[best] = 1;
    }
    std::vector<ChunkMeta> sorted_chunks(n);
    for (int j = 0; j < n; ++j) sorted_chunks[j] = std::move(g->chunks[g->order[j]]);
    g->chunks = std::move(sorted_chunks);
  }
  // bitmap of the chunk at schedule position j: the kept one, or marked afresh into `scratch`
  auto chunk_bm = [&](int j, uint64_t* scratch, uint64_t** out) -> int {
    if (allbm.p) {
      *out = allbm.p + (size_t)g->order[j] * nw;
      return HT_OK;
    }
    HT_TRY(mark_chunk(g->chunks[j], scratch));
    *out = scratch;
    return HT_OK;
  };

  // ---- pass 1: |N_j|, |N_j ^ N_{j-1}| and |N_j ^ (N_0 u ... u N_{j-1})| for every chunk, in schedule order
  DevBlock tmp1;
  DevArr<uint64_t> bmA, bmB, bmT, bmR;
  DevArr<unsigned long long> totals;
  for (int k = 0; k < 4; ++k) tmp1.add<uint64_t>(nw);
  tmp1.add<unsigned long long>((size_t)3 * n);
  HT_TRY(tmp1.alloc(ctx));
  tmp1.take(bmA, nw);
  tmp1.take(bmB, nw);
  tmp1.take(bmT, nw);
  tmp1.take(bmR, nw);
  tmp1.take(totals, (size_t)3 * n);
  HT_HIP(ctx, hipMemsetAsync(totals.p, 0, (size_t)3 * n * 8, st));
  uint64_t* cur = nullptr;
  uint64_t* prev = bmB.p;   // the previous chunk's set (none before the first chunk)
  HT_HIP(ctx, hipMemsetAsync(prev, 0, nw * 8, st));
  HT_HIP(ctx, hipMemsetAsync(bmR.p, 0, nw * 8, st));
  for (int j = 0; j < n; ++j) {
    HT_TRY(chunk_bm(j, (j & 1) ? bmB.p : bmA.p, &cur));
    k_popc3<<<popc_grid(nw), TB, 0, st>>>(cur, prev, bmR.p, nw, totals.p + 3 * j);
    HT_LAUNCH_CHECK(ctx);
    k_bm_or<<<nblk(nw), TB, 0, st>>>(bmR.p, cur, nw);
    HT_LAUNCH_CHECK(ctx);
    prev = cur;
  }
  std::vector<unsigned long long> htot(3 * n);
  HT_HIP(ctx, hipMemcpyAsync(htot.data(), totals.p, (size_t)3 * n * 8, hipMemcpyDeviceToHost, st));
  HT_HIP(ctx, hipStreamSynchronize(st));
  g->v_ori = g->v_ru = g->v_load = 0;
  for (int j = 0; j < n; ++j) {
    ChunkMeta& c = g->chunks[j];
    c.nsrc = (int64_t)htot[3 * j];
    c.nbr_off = g->v_ori;
    c.sptr_off = g->v_ori + j;
    g->v_ori += c.nsrc;
    g->v_ru += c.nsrc - (int64_t)htot[3 * j + 1];   // adjacent-chunk reuse only, as in Sec. 5.3
    g->max_nsrc = std::max(g->max_nsrc, c.nsrc);
  }
  int64_t n_distinct = 0;      // |N_0 u ... u N_{n-1}|
  for (int j = 0; j < n; ++j) n_distinct += g->chunks[j].nsrc - (int64_t)htot[3 * j + 2];
  int64_t C = opts ? opts->cache_rows : 0;
  if (keep_all) C = n_distinct;
  if (C <= 0) C = g->max_nsrc;
  if (C < g->max_nsrc)
    return ht_set_err(ctx, HT_EINVAL, "ht_partition: cache_rows %lld < max_j |N_j| = %lld", (long long)C,
                      (long long)g->max_nsrc);
  const size_t vo = (size_t)std::max<int64_t>(g->v_ori, 1);
  HT_TRY(g->nbr.alloc(ctx, vo));

  // ---- schedule of the buffer.  Adjacent reuse follows from the counts above; the schedule-aware
  // buffer (a row leaves after its last use, or for room with the farthest next use first) is
  // simulated chunk by chunk on bitmaps: the rows released before chunk j (= leaving after chunk
  // j-1) are kept as one bitmap per chunk for pass 2.
  std::vector<int64_t> n_reuse(n), n_leave(n, 0);
  DevArr<uint64_t> Ebm;      // [n x nw], row j: rows released before chunk j
  if (!far_first) {
    for (int j = 0; j < n; ++j) n_reuse[j] = (int64_t)htot[3 * j + 1];
  } else {
    DevArr<int32_t> nxt, last, nu;
    DevArr<unsigned int> hist;
    DevArr<unsigned long long> tot2, dead_cnt;
    DevArr<int32_t> cnt1;
    DevArr<int64_t> pref1;
    DevArr<uint64_t> eqbm;
    HT_TRY(nxt.alloc(ctx, vo));
    HT_TRY(last.alloc(ctx, (size_t)V));
    HT_TRY(nu.alloc(ctx, (size_t)V));
    HT_TRY(hist.alloc(ctx, (size_t)n + 1));
    HT_TRY(tot2.alloc(ctx, 2));
    HT_TRY(dead_cnt.alloc(ctx, (size_t)n));
    HT_HIP(ctx, hipMemsetAsync(dead_cnt.p, 0, (size_t)n * 8, st));
    HT_TRY(cnt1.alloc(ctx, nw));
    HT_TRY(pref1.alloc(ctx, nw + 1));
    HT_TRY(eqbm.alloc(ctx, nw));
    HT_TRY(Ebm.alloc(ctx, (size_t)n * nw));
    HT_HIP(ctx, hipMemsetAsync(Ebm.p, 0, (size_t)n * nw * 8, st));
    {
      std::vector<int32_t> init((size_t)V, n);
      HT_HIP(ctx, hipMemcpyAsync(last.p, init.data(), (size_t)V * 4, hipMemcpyHostToDevice, st));
      HT_HIP(ctx, hipMemcpyAsync(nu.p, init.data(), (size_t)V * 4, hipMemcpyHostToDevice, st));
      HT_HIP(ctx, hipStreamSynchronize(st));
    }
    // N_j lists and next uses, last chunk first
    uint64_t* bmj = nullptr;   // N_j as a bitmap
    for (int j = n - 1; j >= 0; --j) {
      const ChunkMeta& c = g->chunks[j];
      HT_TRY(chunk_bm(j, bmA.p, &bmj));
      HT_TRY(ht_bitmap_prefix(ctx, bmj, nw, cnt1.p, pref1.p));
      HT_TRY(ht_bitmap_expand(ctx, bmj, nw, pref1.p, g->nbr.p + c.nbr_off));
      if (c.nsrc > 0) {
        k_next_use<<<nblk(c.nsrc), TB, 0, st>>>(g->nbr.p + c.nbr_off, c.nsrc, last.p, j, nxt.p + c.nbr_off);
        HT_LAUNCH_CHECK(ctx);
      }
    }
    // forward simulation: bmR = resident rows
    HT_HIP(ctx, hipMemsetAsync(bmR.p, 0, nw * 8, st));
    std::vector<unsigned int> hh((size_t)n + 1);
    for (int j = 0; j < n; ++j) {
      const ChunkMeta& c = g->chunks[j];
      HT_TRY(chunk_bm(j, bmA.p, &bmj));
      HT_HIP(ctx, hipMemsetAsync(tot2.p, 0, 16, st));
      k_popc_union<<<popc_grid(nw), TB, 0, st>>>(bmR.p, bmj, nw, tot2.p);
      HT_LAUNCH_CHECK(ctx);
      unsigned long long t2[2];
      HT_HIP(ctx, hipMemcpyAsync(t2, tot2.p, 16, hipMemcpyDeviceToHost, st));
      HT_HIP(ctx, hipStreamSynchronize(st));
      n_reuse[j] = (int64_t)t2[1];
      const int64_t over = (int64_t)t2[0] - C;
      if (over > 0) {
        uint64_t* E = Ebm.p + (size_t)j * nw;
        k_bm_op<<<nblk(nw), TB, 0, st>>>(bmR.p, bmj, nw, 1, bmT.p);   // candidates: resident, not needed now
        HT_LAUNCH_CHECK(ctx);
        HT_HIP(ctx, hipMemsetAsync(hist.p, 0, ((size_t)n + 1) * 4, st));
        k_hist_nu<<<(unsigned)std::min<int64_t>(nblk(nw), 2048), TB, 0, st>>>(bmT.p, nw, nu.p, n + 1, hist.p);
        HT_LAUNCH_CHECK(ctx);
        HT_HIP(ctx, hipMemcpyAsync(hh.data(), hist.p, ((size_t)n + 1) * 4, hipMemcpyDeviceToHost, st));
        HT_HIP(ctx, hipStreamSynchronize(st));
        int32_t t = n;
        int64_t cum = 0, m = 0;
        for (; t >= 0; --t) {
          if (cum + (int64_t)hh[t] >= over) {
            m = over - cum;
            break;
          }
          cum += hh[t];
        }
        if (t < 0) return ht_set_err(ctx, HT_ESTATE, "ht_partition: buffer schedule ran out of rows to release");
        k_select_nu<<<nblk(nw), TB, 0, st>>>(bmT.p, nw, nu.p, t, E, eqbm.p);
        HT_LAUNCH_CHECK(ctx);
        HT_TRY(ht_bitmap_prefix(ctx, eqbm.p, nw, cnt1.p, pref1.p));
        k_take_first<<<nblk(nw), TB, 0, st>>>(eqbm.p, pref1.p, nw, m, E);
        HT_LAUNCH_CHECK(ctx);
        k_bm_clear<<<nblk(nw), TB, 0, st>>>(bmR.p, E, nw);
        HT_LAUNCH_CHECK(ctx);
        n_leave[j - 1] = over;     // j > 0 here: nothing is resident before the first chunk
      }
      k_bm_or<<<nblk(nw), TB, 0, st>>>(bmR.p, bmj, nw);
      HT_LAUNCH_CHECK(ctx);
      if (c.nsrc > 0) {
        k_set_nu<<<nblk(c.nsrc), TB, 0, st>>>(g->nbr.p + c.nbr_off, c.nsrc, nxt.p + c.nbr_off, nu.p);
        HT_LAUNCH_CHECK(ctx);
        if (j + 1 < n) {   // rows that no later chunk needs leave now (after the last chunk everything does)
          uint64_t* E1 = Ebm.p + (size_t)(j + 1) * nw;
          k_mark_dead<<<nblk(c.nsrc), TB, 0, st>>>(g->nbr.p + c.nbr_off, c.nsrc, nxt.p + c.nbr_off, n, (uint32_t*)E1,
                                                   dead_cnt.p + j);
          HT_LAUNCH_CHECK(ctx);
          k_bm_clear<<<nblk(nw), TB, 0, st>>>(bmR.p, E1, nw);
          HT_LAUNCH_CHECK(ctx);
        }
      }
    }
    if (n > 1) {
      std::vector<unsigned long long> hd((size_t)n);
      HT_HIP(ctx, hipMemcpyAsync(hd.data(), dead_cnt.p, (size_t)n * 8, hipMemcpyDeviceToHost, st));
      HT_HIP(ctx, hipStreamSynchronize(st));
      for (int j = 0; j + 1 < n; ++j) n_leave[j] += (int64_t)hd[j];
    }
    if (n > 0) {
      HT_HIP(ctx, hipMemsetAsync(tot2.p, 0, 16, st));
      k_popc_union<<<popc_grid(nw), TB, 0, st>>>(bmR.p, bmR.p, nw, tot2.p);
      HT_LAUNCH_CHECK(ctx);
      unsigned long long t2[2];
      HT_HIP(ctx, hipMemcpyAsync(t2, tot2.p, 16, hipMemcpyDeviceToHost, st));
      HT_HIP(ctx, hipStreamSynchronize(st));
      n_leave[n - 1] = (int64_t)t2[0];   // what is still resident leaves at the end of a pass
    }
  }
  for (int j = 0; j < n; ++j) {
    ChunkMeta& c = g->chunks[j];
    c.n_reuse = n_reuse[j];
    c.n_load = c.nsrc - c.n_reuse;
    c.reuse_off = c.nbr_off - g->v_load;
    c.load_off = g->v_load;
    g->v_load += c.n_load;
  }
  {
    int64_t off = 0;
    for (int j = 0; j < n; ++j) {
      ChunkMeta& c = g->chunks[j];
      if (far_first) c.n_leave = n_leave[j];
      else c.n_leave = (j + 1 < n) ? c.nsrc - g->chunks[j + 1].n_reuse : c.nsrc;
      c.leave_off = off;
      off += c.n_leave;
    }
  }
  if (C < 1) C = 1;
  g->cache_rows = C;
  g->cache_policy = far_first ? HT_CACHE_FARTHEST : HT_CACHE_ADJACENT;
  g->single_leave = far_first && g->v_load == n_distinct;

  // ---- arenas
  const size_t vr = (size_t)std::max<int64_t>(g->v_load, 1);
  const size_t ep = (size_t)std::max<int64_t>(Ep, 1);
  const size_t n_reused = (size_t)std::max<int64_t>(g->v_ori - g->v_load, 1);
  {
    DevBlock& b = g->blk_chunks;
    b.add<int32_t>(vo); b.add<int32_t>(vo); b.add<int64_t>(vo + n); b.add<int32_t>(n_reused);
    for (int k = 0; k < 4; ++k) b.add<int32_t>(vr);
    for (int k = 0; k < 3; ++k) b.add<int32_t>(ep);
    if (g->merged) b.add<int64_t>(vo + n);
    HT_TRY(b.alloc(ctx));
    b.take(g->slot, vo);
    b.take(g->gslot, vo);
    b.take(g->sptr, vo + n);
    b.take(g->reuse, n_reused);
    b.take(g->load, vr);
    b.take(g->load_slot, vr);
    b.take(g->leave, vr);
    b.take(g->leave_slot, vr);
    b.take(g->col_local, ep);
    b.take(g->col_slot, ep);
    b.take(g->sdst, ep);
    if (g->merged) b.take(g->usptr, vo + n);
  }

  // ---- pass 2 temporaries
  const int64_t nwC = ceil_div64(C, 64);
  const int64_t nwmax = std::max(nw, nwC);
  DevBlock tmp2;
  DevArr<int32_t> cnt_tmp, vslot, freelist, mflag;
  DevArr<int64_t> pref, mrank, mpos;
  DevArr<uint64_t> freebm;
  const size_t mnnz = (size_t)std::max<int64_t>(g->max_nnz, 1);
  tmp2.add<int32_t>(nwmax); tmp2.add<int64_t>(nwmax + 1); tmp2.add<int32_t>((size_t)V); tmp2.add<int32_t>((size_t)C);
  tmp2.add<uint64_t>(nwC);
  if (g->merged) { tmp2.add<int32_t>(mnnz); tmp2.add<int64_t>(mnnz + 1); tmp2.add<int64_t>(mnnz + 1); }
  HT_TRY(tmp2.alloc(ctx));
  tmp2.take(cnt_tmp, nwmax);
  tmp2.take(pref, nwmax + 1);
  tmp2.take(vslot, (size_t)V);
  tmp2.take(freelist, (size_t)C);
  tmp2.take(freebm, nwC);
  if (g->merged) {
    tmp2.take(mflag, mnnz);
    tmp2.take(mrank, mnnz + 1);
    tmp2.take(mpos, mnnz + 1);
  }
  HT_HIP(ctx, hipMemsetAsync(vslot.p, 0xFF, (size_t)V * 4, st));
  // every position free: all ones, the last word cut to C bits (its value travels from pinned memory)
  HT_HIP(ctx, hipMemsetAsync(freebm.p, 0xFF, nwC * 8, st));
  if (C % 64) {
    hpin[4] = (int64_t)((~0ull) >> (64 - (C % 64)));
    HT_HIP(ctx, hipMemcpyAsync(freebm.p + (nwC - 1), &hpin[4], 8, hipMemcpyHostToDevice, st));
  }
  ItemTmp itmp;
  HT_TRY(itmp.alloc(ctx, std::max<int64_t>(std::max(g->max_ndst, g->max_nsrc), 1)));
  itmp.totals = hpin;
  const char* ord_env = getenv("HT_ITEM_ORDER");
  const bool order_items = !(ord_env && atoi(ord_env) == 0);
  int seg_fwd = HT_SEG, seg_bwd = HT_SEG / 2;   // measured best at cfg2; the variables are for experiments
  if (const char* v = getenv("HT_SEG_FWD")) seg_fwd = std::max(64, atoi(v));
  if (const char* v = getenv("HT_SEG_BWD")) seg_bwd = std::max(64, atoi(v));
  // One block for the work-item lists of all chunks and both directions.  A row of len entries makes
  // ceil(len / seg) items and is a cut row when that is more than one, so rows + entries / seg bounds the items
  // and entries / seg the cut rows; the lists take 20 bytes per item and 12 per cut row.
  {
    size_t cap = 0;
    for (int j = 0; j < n; ++j) {
      const ChunkMeta& c = g->chunks[j];
      const size_t ent = (size_t)(g->merged ? c.nu : c.nnz);
      const size_t rows[2] = {(size_t)(c.dst1 - c.dst0), (size_t)c.nsrc};
      const size_t seg[2] = {(size_t)seg_fwd, (size_t)seg_bwd};
      for (int d = 0; d < 2; ++d) cap += DevBlock::pad(20 * (rows[d] + ent / seg[d] + 1) + 12 * (ent / seg[d] + 1));
    }
    HT_TRY(g->items_mem.alloc(ctx, cap));
    itmp.arena = g->items_mem.p;
    itmp.arena_cap = cap;
  }
  // prev: the previous chunk's set (adjacent reuse), or the resident rows, kept up to date in bmB (schedule-aware)
  prev = bmB.p;
  HT_HIP(ctx, hipMemsetAsync(prev, 0, nw * 8, st));
  for (int j = 0; j < n; ++j) {
    ChunkMeta& c = g->chunks[j];
    int32_t* nbr_j = g->nbr.p + c.nbr_off;
    int32_t* slot_j = g->slot.p + c.nbr_off;
    int32_t* gslot_j = g->gslot.p + c.nbr_off;
    int64_t* sptr_j = g->sptr.p + c.sptr_off;
    // unique sorted sources and local indices
    HT_TRY(chunk_bm(j, (far_first || !(j & 1)) ? bmA.p : bmB.p, &cur));
    HT_TRY(ht_bitmap_prefix(ctx, cur, nw, cnt_tmp.p, pref.p));
    HT_TRY(ht_bitmap_expand(ctx, cur, nw, pref.p, nbr_j));
    if (c.nnz > 0) {
      k_remap<<<nblk(c.nnz), TB, 0, st>>>(g->col.p + c.e0, c.nnz, cur, pref.p, g->col_local.p + c.e0);
      HT_LAUNCH_CHECK(ctx);
    }
    // reuse / load / leave(previous chunk)
    k_bm_op<<<nblk(nw), TB, 0, st>>>(cur, prev, nw, 0, bmT.p);
    HT_LAUNCH_CHECK(ctx);
    HT_TRY(ht_bitmap_prefix(ctx, bmT.p, nw, cnt_tmp.p, pref.p));
    HT_TRY(ht_bitmap_expand(ctx, bmT.p, nw, pref.p, g->reuse.p + c.reuse_off));
    k_bm_op<<<nblk(nw), TB, 0, st>>>(cur, prev, nw, 1, bmT.p);
    HT_LAUNCH_CHECK(ctx);
    HT_TRY(ht_bitmap_prefix(ctx, bmT.p, nw, cnt_tmp.p, pref.p));
    HT_TRY(ht_bitmap_expand(ctx, bmT.p, nw, pref.p, g->load.p + c.load_off));
    if (j > 0) {
      ChunkMeta& pc = g->chunks[j - 1];
      if (far_first) {
        HT_HIP(ctx, hipMemcpyAsync(bmT.p, Ebm.p + (size_t)j * nw, nw * 8, hipMemcpyDeviceToDevice, st));
      } else {
        k_bm_op<<<nblk(nw), TB, 0, st>>>(prev, cur, nw, 1, bmT.p);
        HT_LAUNCH_CHECK(ctx);
      }
      HT_TRY(ht_bitmap_prefix(ctx, bmT.p, nw, cnt_tmp.p, pref.p));
      HT_TRY(ht_bitmap_expand(ctx, bmT.p, nw, pref.p, g->leave.p + pc.leave_off));
      if (pc.n_leave > 0) {
        k_evict<<<nblk(pc.n_leave), TB, 0, st>>>(g->leave.p + pc.leave_off, pc.n_leave, vslot.p,
                                                 (uint32_t*)freebm.p, g->leave_slot.p + pc.leave_off);
        HT_LAUNCH_CHECK(ctx);
      }
    }
    // positions: loaded rows take the lowest free positions
    if (c.n_load > 0) {
      HT_TRY(ht_bitmap_prefix(ctx, freebm.p, nwC, cnt_tmp.p, pref.p));
      HT_TRY(ht_bitmap_expand(ctx, freebm.p, nwC, pref.p, freelist.p));
      k_assign<<<nblk(c.n_load), TB, 0, st>>>(g->load.p + c.load_off, c.n_load, freelist.p, vslot.p,
                                              (uint32_t*)freebm.p, g->load_slot.p + c.load_off);
      HT_LAUNCH_CHECK(ctx);
    }
    if (c.nsrc > 0) {
      k_lookup_slots<<<nblk(c.nsrc), TB, 0, st>>>(nbr_j, c.nsrc, vslot.p, prev, slot_j, gslot_j);
      HT_LAUNCH_CHECK(ctx);
    }
    if (c.nnz > 0) {
      k_map_i32<<<nblk(c.nnz), TB, 0, st>>>(g->col_local.p + c.e0, c.nnz, slot_j, g->col_slot.p + c.e0);
      HT_LAUNCH_CHECK(ctx);
    }
    // the same edges grouped by local source, destinations ascending inside a source
    uint64_t* csr_sorted = nullptr;
    HT_HIP(ctx, hipMemsetAsync(sptr_j, 0, (c.nsrc + 1) * 8, st));
    if (c.nnz > 0) {
      k_csr_keys<<<nblk(c.nnz), TB, 0, st>>>(g->indptr.p, c.dst0, c.dst1, c.e0, c.nnz, g->col_local.p + c.e0,
                                             keysA.p);
      HT_LAUNCH_CHECK(ctx);
      uint64_t* sorted = nullptr;
      HT_TRY(ht_radix_sort_u64(ctx, keysA.p, keysB.p, c.nnz, 32, 32 + bits_for(c.nsrc), &sorted));
      k_low_bits<<<nblk(c.nnz), TB, 0, st>>>(sorted, c.nnz, 0xFFFFFFFFull, g->sdst.p + c.e0);
      HT_LAUNCH_CHECK(ctx);
      k_boundaries<<<nblk(c.nnz), TB, 0, st>>>(sorted, c.nnz, 32, c.nsrc, sptr_j);
      HT_LAUNCH_CHECK(ctx);
      csr_sorted = sorted;
    }
    // work items of both directions
    // forward items are ordered by buffer-independent source id; backward ones by local destination
    if (!g->merged) {
      HT_TRY(build_items(ctx, itmp, g->indptr.p + c.dst0, c.e0, c.dst1 - c.dst0, g->col.p + c.e0, V, keysA.p, keysB.p,
                         order_items, seg_fwd, &c.fwd));
      HT_TRY(build_items(ctx, itmp, sptr_j, 0, c.nsrc, g->sdst.p + c.e0, c.dst1 - c.dst0, keysA.p, keysB.p, order_items,
                         seg_bwd, &c.bwd));
    } else {
      int64_t* usptr_j = g->usptr.p + c.sptr_off;
      HT_HIP(ctx, hipMemsetAsync(usptr_j, 0, (c.nsrc + 1) * 8, st));
      if (c.nu > 0) {
        // buffer positions of the distinct forward pairs
        k_gather_i32_at<<<nblk(c.nu), TB, 0, st>>>(upos.p + c.ue0, c.e0, c.nu, g->col_slot.p + c.e0, g->ucol_slot.p + c.ue0);
        HT_LAUNCH_CHECK(ctx);
        // distinct (source, destination) pairs of the by-source order; csr_sorted holds the sorted keys
        uint64_t* other = csr_sorted == keysA.p ? keysB.p : keysA.p;
        k_dup_flags_u64<<<nblk(c.nnz), TB, 0, st>>>(csr_sorted, c.nnz, mflag.p);
        HT_LAUNCH_CHECK(ctx);
        HT_TRY(ht_scan_i32(ctx, mflag.p, mrank.p, c.nnz, false));
        k_flag_positions<<<nblk(c.nnz), TB, 0, st>>>(mflag.p, mrank.p, c.nnz, mpos.p);
        HT_LAUNCH_CHECK(ctx);
        k_set_i64<<<1, 1, 0, st>>>(mpos.p + c.nu, c.nnz);
        HT_LAUNCH_CHECK(ctx);
        k_merge_bwd<<<nblk(c.nu), TB, 0, st>>>(mpos.p, c.nu, csr_sorted, g->s.p + c.dst0, g->usdst.p + c.ue0,
                                               g->uw_bwd.p + c.ue0, g->umult_bwd.p + c.ue0, other);
        HT_LAUNCH_CHECK(ctx);
        k_boundaries<<<nblk(c.nu), TB, 0, st>>>(other, c.nu, 32, c.nsrc, usptr_j);
        HT_LAUNCH_CHECK(ctx);
      }
      HT_TRY(build_items(ctx, itmp, g->uindptr.p + c.dst0, c.ue0, c.dst1 - c.dst0, g->ucol.p + c.ue0, V, keysA.p, keysB.p,
                         order_items, seg_fwd, &c.fwd));
      HT_TRY(build_items(ctx, itmp, usptr_j, 0, c.nsrc, g->usdst.p + c.ue0, c.dst1 - c.dst0, keysA.p, keysB.p,
                         order_items, seg_bwd, &c.bwd));
    }
    g->max_fpart = std::max(g->max_fpart, c.fwd.n_part);
    g->max_bpart = std::max(g->max_bpart, c.bwd.n_part);
    if (far_first) {   // prev = resident rows: minus what was released before this chunk, plus this chunk's
      k_bm_clear<<<nblk(nw), TB, 0, st>>>(prev, Ebm.p + (size_t)j * nw, nw);
      HT_LAUNCH_CHECK(ctx);
      k_bm_or<<<nblk(nw), TB, 0, st>>>(prev, cur, nw);
      HT_LAUNCH_CHECK(ctx);
    } else {
      prev = cur;
    }
  }
  // what is still buffered leaves at the end of a pass
  if (n > 0) {
    ChunkMeta& lc = g->chunks[n - 1];
    if (far_first) {
      if (lc.n_leave > 0) {
        HT_TRY(ht_bitmap_prefix(ctx, prev, nw, cnt_tmp.p, pref.p));
        HT_TRY(ht_bitmap_expand(ctx, prev, nw, pref.p, g->leave.p + lc.leave_off));
        k_map_i32<<<nblk(lc.n_leave), TB, 0, st>>>(g->leave.p + lc.leave_off, lc.n_leave, vslot.p,
                                                   g->leave_slot.p + lc.leave_off);
        HT_LAUNCH_CHECK(ctx);
      }
    } else if (lc.nsrc > 0) {
      HT_HIP(ctx, hipMemcpyAsync(g->leave.p + lc.leave_off, g->nbr.p + lc.nbr_off, lc.nsrc * 4,
                                 hipMemcpyDeviceToDevice, st));
      HT_HIP(ctx, hipMemcpyAsync(g->leave_slot.p + lc.leave_off, g->slot.p + lc.nbr_off, lc.nsrc * 4,
                                 hipMemcpyDeviceToDevice, st));
    }
  }
  HT_HIP(ctx, hipStreamSynchronize(st));
  return HT_OK;
}

template <typename T>
int d2h(ht_ctx* ctx, T* dst, const T* src, int64_t n) {
  if (!dst || n <= 0) return HT_OK;
  HT_HIP(ctx, hipMemcpy(dst, src, (size_t)n * sizeof(T), hipMemcpyDeviceToHost));
  return HT_OK;
}

}  // namespace

int64_t ht_graph::hbm_bytes() const {
  int64_t b = indptr.bytes() + col.bytes() + s.bytes() + nbr.bytes() + col_local.bytes() + col_slot.bytes() +
              sptr.bytes() + sdst.bytes() + slot.bytes() + gslot.bytes() + reuse.bytes() + load.bytes() +
              load_slot.bytes() + leave.bytes() + leave_slot.bytes() + uindptr.bytes() + ucol.bytes() +
              ucol_slot.bytes() + uw_fwd.bytes() + umult.bytes() + usdst.bytes() + uw_bwd.bytes() + umult_bwd.bytes() + usptr.bytes();
  for (const ChunkMeta& c : chunks) b += c.fwd.blob.bytes() + c.bwd.blob.bytes();
  return b;
}

extern "C" {

int ht_partition(ht_ctx* ctx, int64_t V, int64_t E, const int32_t* src, const int32_t* dst, int32_t n_chunks,
                 const ht_part_opts* opts, ht_graph** out) {
  if (!ctx) return HT_EINVAL;
  if (!out) return ht_set_err(ctx, HT_EINVAL, "ht_partition: out is null");
  *out = nullptr;
  if (V <= 0 || V >= ((int64_t)1 << 31)) return ht_set_err(ctx, HT_EINVAL, "ht_partition: V must be in [1, 2^31)");
  if (E < 0 || (E > 0 && (!src || !dst))) return ht_set_err(ctx, HT_EINVAL, "ht_partition: bad edge list");
  if (n_chunks < 1) return ht_set_err(ctx, HT_EINVAL, "ht_partition: n_chunks must be >= 1");
  if (opts && (opts->reorder_chunks < 0 || opts->reorder_chunks > 1 || opts->balance_mode < 0 || opts->balance_mode > 1 || opts->ptr_loc < 0 || opts->ptr_loc > 1 ||
               opts->cache_rows < -1 || opts->cache_policy < 0 || opts->cache_policy > 1))
    return ht_set_err(ctx, HT_EINVAL, "ht_partition: bad options");
  HT_HIP(ctx, hipSetDevice(ctx->device));
  auto t0 = std::chrono::steady_clock::now();
  static std::atomic<uint64_t> next_serial{1};
  ht_graph* g = new (std::nothrow) ht_graph();
  if (g) g->serial = next_serial.fetch_add(1);
  if (!g) return ht_set_err(ctx, HT_ENOMEM, "ht_partition: host allocation failed");
  int rc = partition_impl(ctx, V, E, src, dst, n_chunks, opts, g);
  if (rc != HT_OK) {
    (void)hipStreamSynchronize(ctx->stream);
    delete g;
    return rc;
  }
  g->partition_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  *out = g;
  return HT_OK;
}

int ht_graph_destroy(ht_graph* g) {
  if (!g) return HT_EINVAL;
  if (g->ctx) (void)hipStreamSynchronize(g->ctx->stream);
  delete g;
  return HT_OK;
}

int ht_graph_info_get(const ht_graph* g, ht_graph_info* out) {
  if (!g || !out) return HT_EINVAL;
  out->V = g->V;
  out->E_stored = g->Ep;
  out->n_chunks = g->n;
  out->reserved = 0;
  out->v_ori = g->v_ori;
  out->v_ru = g->v_ru;
  out->v_load = g->v_load;
  out->alpha = g->V > 0 ? (double)g->v_ori / (double)g->V : 0.0;
  out->max_nsrc = g->max_nsrc;
  out->max_ndst = g->max_ndst;
  out->max_nnz = g->max_nnz;
  out->cache_rows = g->cache_rows;
  out->hbm_bytes = g->hbm_bytes();
  out->partition_ms = g->partition_ms;
  return HT_OK;
}

int ht_graph_chunk_info(const ht_graph* g, int32_t j, ht_chunk_info* out) {
  if (!g || !out || j < 0 || j >= g->n) return HT_EINVAL;
  const ChunkMeta& c = g->chunks[j];
  out->dst_begin = c.dst0;
  out->dst_end = c.dst1;
  out->nnz = c.nnz;
  out->n_src = c.nsrc;
  out->n_reuse = c.n_reuse;
  out->n_load = c.n_load;
  out->n_leave = c.n_leave;
  return HT_OK;
}

int ht_graph_export_chunk(const ht_graph* g, int32_t j, ht_chunk_host* out) {
  if (!g || !out || j < 0 || j >= g->n) return HT_EINVAL;
  ht_ctx* ctx = g->ctx;
  const ChunkMeta& c = g->chunks[j];
  HT_HIP(ctx, hipStreamSynchronize(ctx->stream));
  const int64_t nd = c.dst1 - c.dst0;
  if (out->indptr) {
    HT_TRY(d2h(ctx, out->indptr, g->indptr.p + c.dst0, nd + 1));
    for (int64_t i = 0; i <= nd; ++i) out->indptr[i] -= c.e0;
  }
  HT_TRY(d2h(ctx, out->col, g->col.p + c.e0, c.nnz));
  HT_TRY(d2h(ctx, out->nbr, g->nbr.p + c.nbr_off, c.nsrc));
  HT_TRY(d2h(ctx, out->col_local, g->col_local.p + c.e0, c.nnz));
  HT_TRY(d2h(ctx, out->sptr, g->sptr.p + c.sptr_off, c.nsrc + 1));
  HT_TRY(d2h(ctx, out->sdst, g->sdst.p + c.e0, c.nnz));
  HT_TRY(d2h(ctx, out->reuse, g->reuse.p + c.reuse_off, c.n_reuse));
  HT_TRY(d2h(ctx, out->load, g->load.p + c.load_off, c.n_load));
  HT_TRY(d2h(ctx, out->slot, g->slot.p + c.nbr_off, c.nsrc));
  HT_TRY(d2h(ctx, out->leave, g->leave.p + c.leave_off, c.n_leave));
  return HT_OK;
}

int ht_graph_export_csc(const ht_graph* g, int64_t* indptr, int32_t* col, float* s, int64_t* bounds) {
  if (!g) return HT_EINVAL;
  ht_ctx* ctx = g->ctx;
  HT_HIP(ctx, hipStreamSynchronize(ctx->stream));
  HT_TRY(d2h(ctx, indptr, g->indptr.p, g->V + 1));
  HT_TRY(d2h(ctx, col, g->col.p, g->Ep));
  HT_TRY(d2h(ctx, s, g->s.p, g->V));
  if (bounds)
    for (int j = 0; j <= g->n; ++j) bounds[j] = g->bounds[j];
  return HT_OK;
}

int ht_graph_chunk_order(const ht_graph* g, int32_t* order) {
  if (!g || !order) return HT_EINVAL;
  for (int j = 0; j < g->n; ++j) order[j] = g->order[j];
  return HT_OK;
}

// Alg. 4 on neighbour bitmaps: one |V|-bit map per subgraph and one per batch union; every greedy
// step is one launch that counts the common members of all candidates with the current union.
int ht_graph_reorganize(ht_ctx* ctx, const ht_graph* g, int32_t m, int32_t* layout, int64_t* before, int64_t* after) {
  if (!ctx) return HT_EINVAL;
  if (!g || !layout) return ht_set_err(ctx, HT_EINVAL, "ht_graph_reorganize: null argument");
  if (g->ctx != ctx) return ht_set_err(ctx, HT_ESTATE, "graph belongs to another context");
  if (m < 1 || g->n % m != 0)
    return ht_set_err(ctx, HT_EINVAL, "ht_graph_reorganize: %d chunks do not split into %d partitions", g->n, m);
  for (int j = 0; j < g->n; ++j)
    if (g->order[j] != j)
      return ht_set_err(ctx, HT_ESTATE, "ht_graph_reorganize: the graph's chunks must be in vertex-id order (reorder_chunks = 0)");
  const int n = g->n / m, mn = g->n;
  const int64_t nw = ceil_div64(g->V, 64);
  hipStream_t st = ctx->stream;
  DevArr<uint64_t> bms, U;
  HT_TRY(bms.alloc(ctx, (size_t)mn * nw));
  HT_TRY(U.alloc(ctx, (size_t)n * nw));
  DevArr<uint8_t> seen;
  HT_TRY(seen.alloc(ctx, (size_t)nw * 64));
  HT_HIP(ctx, hipMemsetAsync(seen.p, 0, (size_t)nw * 64, st));
  for (int c = 0; c < mn; ++c) {
    const ChunkMeta& ch = g->chunks[c];
    HT_TRY(mark_sources(ctx, st, g->col.p + ch.e0, ch.nnz, seen.p, nw, bms.p + (size_t)c * nw));
  }
  DevArr<unsigned long long> cnt;
  HT_TRY(cnt.alloc(ctx, (size_t)2 * n));
  std::vector<unsigned long long> hcnt((size_t)2 * n);
  const unsigned gx = (unsigned)std::min<int64_t>(ceil_div64(nw, TB), 64);
  // hcnt[k] = |cand_k ^ with| for the ncand bitmaps that start at cand
  auto common = [&](const uint64_t* cand, int ncand, const uint64_t* with) -> int {
    HT_HIP(ctx, hipMemsetAsync(cnt.p, 0, (size_t)ncand * 8, st));
    k_overlap<<<dim3(gx, ncand), TB, 0, st>>>(cand, nw, with, cnt.p);
    HT_LAUNCH_CHECK(ctx);
    HT_HIP(ctx, hipMemcpyAsync(hcnt.data(), cnt.p, (size_t)ncand * 8, hipMemcpyDeviceToHost, st));
    HT_HIP(ctx, hipStreamSynchronize(st));
    return HT_OK;
  };
  // V_ori, V_+p2p, V_+ru (Sec. 5.3) of a layout; uses U for the batch unions
  auto volumes = [&](const std::vector<int32_t>& lay, int64_t* out) -> int {
    HT_HIP(ctx, hipMemsetAsync(U.p, 0, (size_t)n * nw * 8, st));
    for (int j = 0; j < n; ++j)
      for (int i = 0; i < m; ++i) {
        k_bm_or<<<nblk(nw), TB, 0, st>>>(U.p + (size_t)j * nw, bms.p + (size_t)(i * n + lay[i * n + j]) * nw, nw);
        HT_LAUNCH_CHECK(ctx);
      }
    HT_HIP(ctx, hipMemsetAsync(cnt.p, 0, (size_t)2 * n * 8, st));
    for (int j = 0; j < n; ++j) {   // slot j: |U_j|; slot n + j: |U_j ^ U_{j-1}|
      k_overlap<<<dim3(gx, 1), TB, 0, st>>>(U.p + (size_t)j * nw, nw, U.p + (size_t)j * nw, cnt.p + j);
      HT_LAUNCH_CHECK(ctx);
      if (j > 0) {
        k_overlap<<<dim3(gx, 1), TB, 0, st>>>(U.p + (size_t)j * nw, nw, U.p + (size_t)(j - 1) * nw, cnt.p + n + j);
        HT_LAUNCH_CHECK(ctx);
      }
    }
    HT_HIP(ctx, hipMemcpyAsync(hcnt.data(), cnt.p, (size_t)2 * n * 8, hipMemcpyDeviceToHost, st));
    HT_HIP(ctx, hipStreamSynchronize(st));
    out[0] = g->v_ori;
    out[1] = out[2] = 0;
    for (int j = 0; j < n; ++j) {
      out[1] += (int64_t)hcnt[j];
      out[2] += (int64_t)hcnt[j] - (j > 0 ? (int64_t)hcnt[n + j] : 0);
    }
    return HT_OK;
  };
  std::vector<int32_t> lay((size_t)mn);
  for (int c = 0; c < mn; ++c) lay[c] = c % n;
  if (before) HT_TRY(volumes(lay, before));
  // ---- phase 1: the batches start as partition 0's subgraphs; every other partition hands each batch, in
  // batch order, its unassigned subgraph with the most neighbours in common with the batch's union so far
  std::vector<int32_t> Gt((size_t)mn);
  for (int j = 0; j < n; ++j) Gt[j] = j;
  HT_HIP(ctx, hipMemcpyAsync(U.p, bms.p, (size_t)n * nw * 8, hipMemcpyDeviceToDevice, st));
  for (int i = 1; i < m; ++i) {
    std::vector<char> taken(n, 0);
    for (int j = 0; j < n; ++j) {
      HT_TRY(common(bms.p + (size_t)i * n * nw, n, U.p + (size_t)j * nw));
      int best = -1;
      for (int k = 0; k < n; ++k)
        if (!taken[k] && (best < 0 || hcnt[k] > hcnt[best])) best = k;
      Gt[(size_t)i * n + j] = best;
      taken[best] = 1;
      k_bm_or<<<nblk(nw), TB, 0, st>>>(U.p + (size_t)j * nw, bms.p + (size_t)(i * n + best) * nw, nw);
      HT_LAUNCH_CHECK(ctx);
    }
  }
  // ---- phase 2: batch 0 first, then always the unplaced batch whose union shares the most with the last one
  std::vector<int32_t> at(n, 0);
  std::vector<char> placed(n, 0);
  if (n > 0) placed[0] = 1;
  for (int j = 1; j < n; ++j) {
    HT_TRY(common(U.p, n, U.p + (size_t)at[j - 1] * nw));
    int best = -1;
    for (int k = 0; k < n; ++k)
      if (!placed[k] && (best < 0 || hcnt[k] > hcnt[best])) best = k;
    at[j] = best;
    placed[best] = 1;
  }
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) lay[(size_t)i * n + j] = Gt[(size_t)i * n + at[j]];
  if (after) HT_TRY(volumes(lay, after));
  for (int c = 0; c < mn; ++c) layout[c] = lay[c];
  HT_HIP(ctx, hipStreamSynchronize(st));
  return HT_OK;
}

}  // extern "C"

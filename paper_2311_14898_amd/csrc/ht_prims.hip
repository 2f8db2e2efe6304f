// Device-wide primitives for the integer (preprocessing) part: exclusive scan,
// stable LSD radix sort of 64-bit keys, bitmap rank / expand.  Wave64 ballot,
// popcount and shuffle scans do the in-wave work.
#include "ht_internal.h"

namespace {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

__device__ __forceinline__ int64_t wave_incl_scan_i64(int64_t x, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int64_t y = __shfl_up(x, o, 64);
    if (lane >= o) x += y;
  }
  return x;
}

// Exclusive scan of one value per thread across a 256-thread block.
// Returns the exclusive prefix; *total gets the block sum (valid in all threads).
__device__ __forceinline__ int64_t block_excl_scan_i64(int64_t x, int64_t* total) {
  __shared__ int64_t wsum[SCAN_THREADS / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t inc = wave_incl_scan_i64(x, lane);
  __syncthreads();  // protect wsum against a previous use
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int64_t off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < SCAN_THREADS / 64; ++w) {
    if (w < wave) off += wsum[w];
    tot += wsum[w];
  }
  *total = tot;
  return off + inc - x;
}

template <typename Tin>
__global__ void __launch_bounds__(SCAN_THREADS) k_scan_reduce(const Tin* __restrict__ in, int64_t n,
                                                             int64_t* __restrict__ block_sums) {
  const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
  int64_t s = 0;
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    int64_t idx = base + i;
    if (idx < n) s += (int64_t)in[idx];
  }
  int64_t tot;
  block_excl_scan_i64(s, &tot);
  if (threadIdx.x == 0) block_sums[blockIdx.x] = tot;
}

// block_offsets may be null (single block).  out may alias in when Tin is int64.
// RAW_SUMS: block_offsets holds the blocks' own sums, not their prefix; a block adds up the sums
// before it by itself (a few thousand values at most), which saves the launch that scans them.
template <typename Tin, bool RAW_SUMS>
__global__ void __launch_bounds__(SCAN_THREADS) k_scan_apply(const Tin* in, int64_t n,
                                                            const int64_t* __restrict__ block_offsets,
                                                            int64_t* out, int want_total) {
  const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
  int64_t before = 0;
  if (RAW_SUMS) {
    int64_t part = 0;
    for (int64_t i = threadIdx.x; i < (int64_t)blockIdx.x; i += SCAN_THREADS) part += block_offsets[i];
    block_excl_scan_i64(part, &before);
  } else if (block_offsets) {
    before = block_offsets[blockIdx.x];
  }
  int64_t v[SCAN_ITEMS];
  int64_t s = 0;
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    int64_t idx = base + i;
    v[i] = idx < n ? (int64_t)in[idx] : 0;
    s += v[i];
  }
  int64_t tot;
  int64_t off = block_excl_scan_i64(s, &tot) + before;
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    int64_t idx = base + i;
    if (idx < n) out[idx] = off;
    off += v[i];
  }
  if (want_total && blockIdx.x == gridDim.x - 1 && threadIdx.x == SCAN_THREADS - 1) out[n] = off;
}

// One block walks the whole input tile by tile with a running carry: one launch for short inputs
// (bitmap word counts, per-row item counts of a chunk).  out may alias in when Tin is int64.
template <typename Tin>
__global__ void __launch_bounds__(SCAN_THREADS) k_scan_one_block(const Tin* in, int64_t n, int64_t* out,
                                                                int want_total) {
  int64_t carry = 0;
  for (int64_t t0 = 0; t0 < n; t0 += SCAN_TILE) {
    const int64_t base = t0 + (int64_t)threadIdx.x * SCAN_ITEMS;
    int64_t v[SCAN_ITEMS];
    int64_t s = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
      int64_t idx = base + i;
      v[i] = idx < n ? (int64_t)in[idx] : 0;
      s += v[i];
    }
    int64_t tot;
    int64_t off = block_excl_scan_i64(s, &tot) + carry;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
      int64_t idx = base + i;
      if (idx < n) out[idx] = off;
      off += v[i];
    }
    carry += tot;
  }
  if (want_total && threadIdx.x == 0) out[n] = carry;
}

constexpr int64_t SCAN_ONE_BLOCK_MAX = 16 * SCAN_TILE;   // up to here one block is faster than two launches
constexpr int64_t SCAN_RAW_SUMS_MAX = 4096;              // blocks whose sums each block adds up by itself

// Block sums of every level live back to back in one scratch slot of the context (the level of n elements
// needs ceil(n / SCAN_TILE) sums, the next one a tile-th of that, ...): no allocation, hence no
// implicit device synchronisation, per call.  ws points at this level's sums.
template <typename Tin>
int scan_level(ht_ctx* ctx, const Tin* in, int64_t* out, int64_t n, bool want_total, int64_t* ws) {
  const int64_t nb = ceil_div64(n, SCAN_TILE);
  const int wt = want_total ? 1 : 0;
  if (n <= SCAN_ONE_BLOCK_MAX) {
    k_scan_one_block<Tin><<<1, SCAN_THREADS, 0, ctx->stream>>>(in, n, out, wt);
    HT_LAUNCH_CHECK(ctx);
    return HT_OK;
  }
  k_scan_reduce<Tin><<<(unsigned)nb, SCAN_THREADS, 0, ctx->stream>>>(in, n, ws);
  HT_LAUNCH_CHECK(ctx);
  if (nb <= SCAN_RAW_SUMS_MAX) {
    k_scan_apply<Tin, true><<<(unsigned)nb, SCAN_THREADS, 0, ctx->stream>>>(in, n, ws, out, wt);
    HT_LAUNCH_CHECK(ctx);
    return HT_OK;
  }
  HT_TRY(scan_level<int64_t>(ctx, ws, ws, nb, false, ws + nb));
  k_scan_apply<Tin, false><<<(unsigned)nb, SCAN_THREADS, 0, ctx->stream>>>(in, n, ws, out, wt);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

template <typename Tin>
int scan_impl(ht_ctx* ctx, const Tin* in, int64_t* out, int64_t n, bool want_total) {
  if (n < 0) return ht_set_err(ctx, HT_EINVAL, "scan: negative length");
  if (n == 0) {
    if (want_total) HT_HIP(ctx, hipMemsetAsync(out, 0, sizeof(int64_t), ctx->stream));
    return HT_OK;
  }
  size_t sums = 0;
  for (int64_t m = ceil_div64(n, SCAN_TILE); m > 1; m = ceil_div64(m, SCAN_TILE)) sums += (size_t)m;
  int64_t* ws = nullptr;
  if (sums > 0) HT_TRY(ht_scratch(ctx, HT_S_SCAN, sums * sizeof(int64_t), (void**)&ws));
  return scan_level<Tin>(ctx, in, out, n, want_total, ws);
}

// ------------------------------------------------------------------ radix sort
constexpr int RS_THREADS = 256;
constexpr int RS_WAVES = RS_THREADS / 64;
constexpr int RS_ROUNDS = 16;
constexpr int RS_TILE = RS_THREADS * RS_ROUNDS;  // keys per block
constexpr int RS_BINS = 256;

__global__ void __launch_bounds__(RS_THREADS) k_rs_hist(const uint64_t* __restrict__ keys, int64_t n, int shift,
                                                       uint32_t mask, int32_t* __restrict__ table,
                                                       int64_t nblocks) {
  __shared__ uint32_t h[RS_BINS];
  h[threadIdx.x] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * RS_TILE;
#pragma unroll 4
  for (int i = threadIdx.x; i < RS_TILE; i += RS_THREADS) {
    int64_t idx = base + i;
    if (idx < n) atomicAdd(&h[(uint32_t)(keys[idx] >> shift) & mask], 1u);
  }
  __syncthreads();
  table[(int64_t)threadIdx.x * nblocks + blockIdx.x] = (int32_t)h[threadIdx.x];
}

// Stable scatter.  Key order inside a block is (wave, round, lane) = index
// order.  A lane's rank among equal digits: earlier waves' counts, earlier
// rounds of its own wave, lower lanes of its own round (ballot match).
// The block first puts its keys into digit order in LDS and then writes them out in that order, so that
// consecutive lanes store consecutive keys of one digit's run (a lane storing its own key straight to its
// final place touches a 128-byte line of the output from up to 16 different store instructions).
__global__ void __launch_bounds__(RS_THREADS) k_rs_scatter(const uint64_t* __restrict__ in,
                                                          uint64_t* __restrict__ out, int64_t n, int shift,
                                                          uint32_t mask, const int64_t* __restrict__ offs,
                                                          int64_t nblocks) {
  __shared__ uint32_t cnt[RS_WAVES][RS_BINS];
  __shared__ int64_t goff[RS_BINS];     // where the block's run of a digit starts in the output, minus lstart
  __shared__ uint32_t lstart[RS_BINS];  // where it starts in the block's tile
  __shared__ uint32_t wtot[RS_WAVES];
  __shared__ uint64_t tile[RS_TILE];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < RS_WAVES * RS_BINS; i += RS_THREADS) (&cnt[0][0])[i] = 0;
  __syncthreads();

  uint64_t key[RS_ROUNDS];
  uint32_t rank[RS_ROUNDS];
  const int64_t base = (int64_t)blockIdx.x * RS_TILE + (int64_t)wave * (64 * RS_ROUNDS);
  const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
  for (int r = 0; r < RS_ROUNDS; ++r) {
    const int64_t idx = base + r * 64 + lane;
    const bool valid = idx < n;
    key[r] = valid ? in[idx] : 0ull;
    const uint32_t dg = (uint32_t)(key[r] >> shift) & mask;
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const bool bit = (dg >> b) & 1u;
      const uint64_t bal = __ballot(bit);
      peers &= bit ? bal : ~bal;
    }
    const uint32_t before = valid ? cnt[wave][dg] : 0u;
    __builtin_amdgcn_wave_barrier();
    const uint32_t lower = (uint32_t)__popcll(peers & lt);
    if (valid && lower == 0) cnt[wave][dg] = before + (uint32_t)__popcll(peers);
    __builtin_amdgcn_wave_barrier();
    rank[r] = before + lower;
  }
  __syncthreads();
  {
    const int dgt = threadIdx.x;  // one digit per thread
    uint32_t run = 0;
#pragma unroll
    for (int w = 0; w < RS_WAVES; ++w) {
      uint32_t c = cnt[w][dgt];
      cnt[w][dgt] = run;
      run += c;
    }
    // exclusive prefix of the digit totals over the block's 256 digits
    uint32_t inc = run;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t y = __shfl_up(inc, o, 64);
      if (lane >= o) inc += y;
    }
    if (lane == 63) wtot[wave] = inc;
    __syncthreads();
    uint32_t off = 0;
#pragma unroll
    for (int w = 0; w < RS_WAVES; ++w)
      if (w < wave) off += wtot[w];
    const uint32_t ls = off + inc - run;
    lstart[dgt] = ls;
    goff[dgt] = offs[(int64_t)dgt * nblocks + blockIdx.x] - (int64_t)ls;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < RS_ROUNDS; ++r) {
    const int64_t idx = base + r * 64 + lane;
    if (idx < n) {
      const uint32_t dg = (uint32_t)(key[r] >> shift) & mask;
      tile[lstart[dg] + cnt[wave][dg] + rank[r]] = key[r];
    }
  }
  __syncthreads();
  const int64_t left = n - (int64_t)blockIdx.x * RS_TILE;
  const int here = left < RS_TILE ? (int)left : RS_TILE;
#pragma unroll 4
  for (int i = threadIdx.x; i < here; i += RS_THREADS) {
    const uint64_t k = tile[i];
    const uint32_t dg = (uint32_t)(k >> shift) & mask;
    out[goff[dg] + i] = k;
  }
}

// ------------------------------------------------------------------ bitmaps
__global__ void k_popc(const uint64_t* __restrict__ bm, int64_t nw, int32_t* __restrict__ cnt) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nw) cnt[i] = __popcll(bm[i]);
}

__global__ void k_bm_expand(const uint64_t* __restrict__ bm, int64_t nw, const int64_t* __restrict__ pref,
                            int32_t* __restrict__ out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nw) return;
  uint64_t w = bm[i];
  int64_t p = pref[i];
  const int32_t base = (int32_t)(i * 64);
  while (w) {
    int b = __ffsll((unsigned long long)w) - 1;
    out[p++] = base + b;
    w &= w - 1;
  }
}

}  // namespace

int ht_scan_i32(ht_ctx* ctx, const int32_t* in, int64_t* out, int64_t n, bool want_total) {
  return scan_impl<int32_t>(ctx, in, out, n, want_total);
}
int ht_scan_i64(ht_ctx* ctx, const int64_t* in, int64_t* out, int64_t n, bool want_total) {
  return scan_impl<int64_t>(ctx, in, out, n, want_total);
}

int ht_radix_sort_u64(ht_ctx* ctx, uint64_t* keys, uint64_t* tmp, int64_t n, int bit_lo, int bit_hi,
                      uint64_t** sorted) {
  *sorted = keys;
  if (n <= 1 || bit_hi <= bit_lo) return HT_OK;
  const int64_t nblocks = ceil_div64(n, RS_TILE);
  // per-block digit counts and their offsets, in a scratch slot of the context (no allocation per call)
  const size_t cells = (size_t)(RS_BINS * nblocks);
  char* rs = nullptr;
  HT_TRY(ht_scratch(ctx, HT_S_RSORT, cells * 12 + 16, (void**)&rs));
  struct { int64_t* p; } offs{(int64_t*)rs};
  struct { int32_t* p; } table{(int32_t*)(rs + cells * 8)};
  uint64_t* a = keys;
  uint64_t* b = tmp;
  for (int shift = bit_lo; shift < bit_hi; shift += 8) {
    const int bits = (bit_hi - shift) < 8 ? (bit_hi - shift) : 8;
    const uint32_t mask = (1u << bits) - 1u;
    k_rs_hist<<<(unsigned)nblocks, RS_THREADS, 0, ctx->stream>>>(a, n, shift, mask, table.p, nblocks);
    HT_LAUNCH_CHECK(ctx);
    HT_TRY(ht_scan_i32(ctx, table.p, offs.p, RS_BINS * nblocks, false));
    k_rs_scatter<<<(unsigned)nblocks, RS_THREADS, 0, ctx->stream>>>(a, b, n, shift, mask, offs.p, nblocks);
    HT_LAUNCH_CHECK(ctx);
    uint64_t* t = a;
    a = b;
    b = t;
  }
  *sorted = a;
  return HT_OK;
}

int ht_bitmap_prefix(ht_ctx* ctx, const uint64_t* bm, int64_t nw, int32_t* cnt_tmp, int64_t* pref) {
  if (nw > 0) {
    k_popc<<<(unsigned)ceil_div64(nw, 256), 256, 0, ctx->stream>>>(bm, nw, cnt_tmp);
    HT_LAUNCH_CHECK(ctx);
  }
  return ht_scan_i32(ctx, cnt_tmp, pref, nw, true);
}

int ht_bitmap_expand(ht_ctx* ctx, const uint64_t* bm, int64_t nw, const int64_t* pref, int32_t* out) {
  if (nw <= 0) return HT_OK;
  k_bm_expand<<<(unsigned)ceil_div64(nw, 256), 256, 0, ctx->stream>>>(bm, nw, pref, out);
  HT_LAUNCH_CHECK(ctx);
  return HT_OK;
}

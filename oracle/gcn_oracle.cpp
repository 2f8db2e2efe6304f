// CPU oracle for partition-based full-graph GCN training.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
// the hot path computes.  It is called by the tests, by the smoke check and by
// the benchmark's CPU-baseline leg; the product library never links, loads or
// calls it, and it shares no code with the HIP path.
//
// What it follows (paper sections, not listings):
//   * GCN layer, Eq. 2:  h'_v = sigma( W (x) sum_{u in N(v)} d_uv h_u ), with
//     the aggregate taken first and the linear + ReLU update after it.
//   * Backward of UPDATE, Sec. 2.3:  grad W = a^T (ReLU'(aW) * grad h'), with
//     ReLU' = 1 for positive input and 0 otherwise (so 0 at 0).
//   * Backward of AGGREGATE, Sec. 4.1: a source sums gradient along its
//     out-edges; replicas in different chunks sum.
//   * Chunks, Sec. 4.1 / 4.3: a chunk is a set of destinations with all their
//     in-edges; N_j is its in-neighbour set.
//   * Dedup sets and volumes, Sec. 5.1 / 5.3: reuse set N_j ^ N_{j-1}, load set
//     N_j \ N_{j-1}, V_ori and V_+ru (one GPU, so the inter-GPU term is void);
//     V_ori, V_+p2p, V_+ru for m partitions of n subgraphs and the partition
//     reorganisation of Alg. 4 (a planning step: sets only, no second GPU).
//   * Epoch, Alg. 1: forward over layers, loss, backward, parameter update.
//   * GAT layer, Eq. 3: attention coefficients from a^l [W h_v || W h_u], LeakyReLU,
//     neighbour-oriented softmax, weighted sum; its backward by the chain rule.
//
// Readings where the paper is silent (normalisation degree, loss, optimiser,
// boundary rule, canonical orders) are the ones listed in the design notes of
// this repository; every one is restated at the function that uses it.
//
// Arithmetic is fp64 throughout.  Parallel loops run over independent output
// rows only, so results do not depend on the thread count.
//
// Pins (see tests, "not gpu"): dense brute force on tiny graphs, finite
// differences of the loss, all-ones features on regular graphs, ln C loss at
// zero weights, partitioned == unpartitioned, the paper's printed transfer
// counts and buffer example, brute-force set arithmetic; for the GAT layer a
// dense statement of Eq. 3 on tiny multigraphs, autograd through it, finite
// differences, the neighbour mean at zero attention parameters.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <iterator>
#include <set>
#include <vector>

extern "C" {

// ---------------------------------------------------------------------------
// Integer part
// ---------------------------------------------------------------------------

// Edge list (u -> v) to CSC by destination.  One self-loop per vertex is added
// when add_self_loops != 0.  Duplicate edges are kept.  Inside a destination
// the sources ascend (equal sources adjacent).  Returns E' = number of stored
// entries; indptr has V+1 entries, col must hold E (+V) entries.
int64_t orc_csc_build(int64_t V, int64_t E, const int32_t* src, const int32_t* dst,
                      int add_self_loops, int64_t* indptr, int32_t* col) {
  std::vector<std::pair<int32_t, int32_t>> e;  // (dst, src)
  e.reserve((size_t)E + (add_self_loops ? (size_t)V : 0));
  for (int64_t i = 0; i < E; ++i) e.emplace_back(dst[i], src[i]);
  if (add_self_loops)
    for (int64_t v = 0; v < V; ++v) e.emplace_back((int32_t)v, (int32_t)v);
  std::sort(e.begin(), e.end());
  for (int64_t v = 0; v <= V; ++v) indptr[v] = 0;
  for (auto& p : e) indptr[p.first + 1]++;
  for (int64_t v = 0; v < V; ++v) indptr[v + 1] += indptr[v];
  for (size_t i = 0; i < e.size(); ++i) col[i] = e[i].second;
  return (int64_t)e.size();
}

// Chunk boundaries over contiguous destination IDs, b[0]=0, b[n]=V.
// mode 0 ("computation-balanced", the range rule of Sec. 4.1 read as balancing
// stored in-edges): b[j] = min{ v : indptr[v] >= ceil(j*E'/n) }.
// mode 1 (equal vertices): b[j] = floor(j*V/n).  Empty chunks are legal.
void orc_chunk_bounds(int64_t V, const int64_t* indptr, int n, int mode, int64_t* b) {
  const int64_t Ep = indptr[V];
  b[0] = 0;
  b[n] = V;
  for (int j = 1; j < n; ++j) {
    if (mode == 1) {
      b[j] = (int64_t)(((__int128)j * V) / n);
    } else {
      __int128 num = (__int128)j * Ep;
      int64_t target = (int64_t)((num + n - 1) / n);
      int64_t v = 0;
      while (v < V && indptr[v] < target) ++v;
      b[j] = v;
    }
  }
}

// |N_j| for the chunk of destinations [b0, b1).
int64_t orc_chunk_nsrc(const int64_t* indptr, const int32_t* col, int64_t b0, int64_t b1) {
  std::vector<int32_t> s(col + indptr[b0], col + indptr[b1]);
  std::sort(s.begin(), s.end());
  return (int64_t)(std::unique(s.begin(), s.end()) - s.begin());
}

// Dedup remap of one chunk.
//   N         ascending unique sources of the chunk's edges           [|N_j|]
//   col_local position of each edge's source in N, edges in CSC order [E'_j]
//   sptr/sdst the same edges by local source: for local source i the
//             entries sdst[sptr[i] .. sptr[i+1]) are local destinations
//             (v - b0), ascending, equal ones adjacent                [|N_j|+1],[E'_j]
void orc_chunk_dedup(const int64_t* indptr, const int32_t* col, int64_t b0, int64_t b1,
                     int32_t* N, int32_t* col_local, int64_t* sptr, int32_t* sdst) {
  const int64_t e0 = indptr[b0], e1 = indptr[b1];
  std::vector<int32_t> s(col + e0, col + e1);
  std::sort(s.begin(), s.end());
  s.erase(std::unique(s.begin(), s.end()), s.end());
  const int64_t ns = (int64_t)s.size();
  for (int64_t i = 0; i < ns; ++i) N[i] = s[i];
  for (int64_t e = e0; e < e1; ++e)
    col_local[e - e0] = (int32_t)(std::lower_bound(s.begin(), s.end(), col[e]) - s.begin());
  std::vector<std::pair<int32_t, int32_t>> t;  // (local source, local destination)
  t.reserve((size_t)(e1 - e0));
  for (int64_t v = b0; v < b1; ++v)
    for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e)
      t.emplace_back(col_local[e - e0], (int32_t)(v - b0));
  std::sort(t.begin(), t.end());
  for (int64_t i = 0; i <= ns; ++i) sptr[i] = 0;
  for (auto& p : t) sptr[p.first + 1]++;
  for (int64_t i = 0; i < ns; ++i) sptr[i + 1] += sptr[i];
  for (size_t i = 0; i < t.size(); ++i) sdst[i] = t[i].second;
}

// Reuse / load split between adjacently scheduled chunks (Sec. 5.1, step 2):
// R = cur ^ prev, Ld = cur \ prev, both ascending.  Inputs ascending unique.
void orc_reuse_split(const int32_t* prev, int64_t n_prev, const int32_t* cur, int64_t n_cur,
                     int32_t* R, int32_t* Ld, int64_t* nR, int64_t* nLd) {
  int32_t* r_end = std::set_intersection(cur, cur + n_cur, prev, prev + n_prev, R);
  int32_t* l_end = std::set_difference(cur, cur + n_cur, prev, prev + n_prev, Ld);
  *nR = r_end - R;
  *nLd = l_end - Ld;
}

// Host-GPU transfer volumes in rows for one GPU (Sec. 5.3 with m = 1):
// V_ori = sum_j |N_j|;  V_+ru = |N_0| + sum_{j>=1} |N_j \ N_{j-1}|.
void orc_volumes(int64_t V, const int64_t* indptr, const int32_t* col, int n, const int64_t* b,
                 int64_t* v_ori, int64_t* v_ru) {
  (void)V;
  std::vector<int32_t> prev, cur, tmp;
  int64_t ori = 0, ru = 0;
  for (int j = 0; j < n; ++j) {
    cur.assign(col + indptr[b[j]], col + indptr[b[j + 1]]);
    std::sort(cur.begin(), cur.end());
    cur.erase(std::unique(cur.begin(), cur.end()), cur.end());
    ori += (int64_t)cur.size();
    tmp.clear();
    std::set_difference(cur.begin(), cur.end(), prev.begin(), prev.end(), std::back_inserter(tmp));
    ru += (int64_t)tmp.size();
    prev.swap(cur);
  }
  *v_ori = ori;
  *v_ru = ru;
}

// Schedule order of the chunks of one partition by the greedy of Alg. 4, phase 2
// (one GPU, so a batch is one chunk): the first chunk stays first; then, step by
// step, the unplaced chunk whose neighbour set shares the most vertices with the
// chunk placed last comes next.  Ties go to the smallest chunk id (the paper
// does not say).  order[j] = id of the chunk scheduled at position j.
void orc_chunk_order(const int64_t* indptr, const int32_t* col, int n, const int64_t* b, int32_t* order) {
  std::vector<std::vector<int32_t>> N(n);
  for (int j = 0; j < n; ++j) {
    N[j].assign(col + indptr[b[j]], col + indptr[b[j + 1]]);
    std::sort(N[j].begin(), N[j].end());
    N[j].erase(std::unique(N[j].begin(), N[j].end()), N[j].end());
  }
  std::vector<char> placed(n, 0);
  if (n > 0) {
    order[0] = 0;
    placed[0] = 1;
  }
  std::vector<int32_t> tmp;
  for (int j = 1; j < n; ++j) {
    const std::vector<int32_t>& last = N[order[j - 1]];
    int best = -1;
    int64_t best_ov = -1;
    for (int k = 0; k < n; ++k) {
      if (placed[k]) continue;
      tmp.clear();
      std::set_intersection(N[k].begin(), N[k].end(), last.begin(), last.end(), std::back_inserter(tmp));
      if ((int64_t)tmp.size() > best_ov) {
        best_ov = (int64_t)tmp.size();
        best = k;
      }
    }
    order[j] = best;
    placed[best] = 1;
  }
}

// Communication volumes of Sec. 5.3 for m partitions of n subgraphs each, in rows per pass.
// Subgraph k of partition i is the destination range [b[i*n+k], b[i*n+k+1]); layout[i*n+j] names the
// subgraph of partition i that runs in batch j (the m subgraphs of a batch run at the same time, one
// per GPU).  With N_ij the in-neighbour set of that subgraph and U_j the union of N_ij over i:
//   out[0] = V_ori  = sum over i, j of |N_ij|          (every subgraph fetches its own neighbours)
//   out[1] = V_+p2p = sum over j of |U_j|              (a batch fetches each vertex once)
//   out[2] = V_+ru  = |U_0| + sum over j >= 1 of |U_j minus U_{j-1}|   (and keeps what the last batch had)
void orc_volumes_mn(const int64_t* indptr, const int32_t* col, int m, int n, const int64_t* b, const int32_t* layout,
                    int64_t* out) {
  int64_t ori = 0, p2p = 0, ru = 0;
  std::set<int32_t> prev;
  for (int j = 0; j < n; ++j) {
    std::set<int32_t> U;
    for (int i = 0; i < m; ++i) {
      const int c = i * n + layout[i * n + j];
      std::set<int32_t> N(col + indptr[b[c]], col + indptr[b[c + 1]]);
      ori += (int64_t)N.size();
      U.insert(N.begin(), N.end());
    }
    p2p += (int64_t)U.size();
    for (int32_t v : U)
      if (j == 0 || !prev.count(v)) ++ru;
    prev.swap(U);
  }
  out[0] = ori;
  out[1] = p2p;
  out[2] = ru;
}

// Partition reorganisation, Alg. 4, both phases, for m partitions of n subgraphs (same indexing as
// orc_volumes_mn).  layout[i*n+j] = subgraph of partition i that ends up in batch j.
//   Phase 1 (which subgraphs share a batch): the batches start as the subgraphs of partition 0 in
//   their given order, U_j = N_0j.  Partitions 1 .. m-1 are taken in turn; for each, batch after
//   batch (j = 0 .. n-1) receives the not yet assigned subgraph k of that partition with the largest
//   |N_ik ^ U_j|, and U_j grows by N_ik.
//   Phase 2 (in which order the batches run): batch 0 stays first; then, step by step, the unplaced
//   batch whose union shares the most vertices with the union of the batch placed last comes next.
//   Every partition's subgraphs follow their batch, partition 0 included (the listing's inner loop
//   starts at 1, which would leave partition 0 out of step with its batch).
// Ties go to the smallest index in both phases (the paper does not say).
void orc_reorganize(const int64_t* indptr, const int32_t* col, int m, int n, const int64_t* b, int32_t* layout) {
  auto nbrs = [&](int c) {
    std::vector<int32_t> N(col + indptr[b[c]], col + indptr[b[c + 1]]);
    std::sort(N.begin(), N.end());
    N.erase(std::unique(N.begin(), N.end()), N.end());
    return N;
  };
  auto common = [](const std::vector<int32_t>& x, const std::vector<int32_t>& y) {
    std::vector<int32_t> t;
    std::set_intersection(x.begin(), x.end(), y.begin(), y.end(), std::back_inserter(t));
    return (int64_t)t.size();
  };
  // phase 1
  std::vector<std::vector<int32_t>> Gt(m, std::vector<int32_t>(n));   // Gt[i][j]: subgraph of partition i in batch j
  std::vector<std::vector<int32_t>> U(n);
  for (int j = 0; j < n; ++j) {
    Gt[0][j] = j;
    U[j] = nbrs(j);
  }
  for (int i = 1; i < m; ++i) {
    std::vector<char> taken(n, 0);
    for (int j = 0; j < n; ++j) {
      int best = -1;
      int64_t best_ov = -1;
      for (int k = 0; k < n; ++k) {
        if (taken[k]) continue;
        const int64_t ov = common(nbrs(i * n + k), U[j]);
        if (ov > best_ov) {
          best_ov = ov;
          best = k;
        }
      }
      Gt[i][j] = best;
      taken[best] = 1;
      const std::vector<int32_t> Nk = nbrs(i * n + best);
      std::vector<int32_t> t;
      std::set_union(U[j].begin(), U[j].end(), Nk.begin(), Nk.end(), std::back_inserter(t));
      U[j].swap(t);
    }
  }
  // phase 2
  std::vector<int32_t> at(n, 0);   // at[j]: the phase-1 batch that runs at position j
  std::vector<char> placed(n, 0);
  if (n > 0) placed[0] = 1;
  for (int j = 1; j < n; ++j) {
    int best = -1;
    int64_t best_ov = -1;
    for (int k = 0; k < n; ++k) {
      if (placed[k]) continue;
      const int64_t ov = common(U[k], U[at[j - 1]]);
      if (ov > best_ov) {
        best_ov = ov;
        best = k;
      }
    }
    at[j] = best;
    placed[best] = 1;
  }
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) layout[i * n + j] = Gt[i][at[j]];
}

// Row-buffer schedule: which neighbour rows are reused, loaded and released at
// every chunk, for a buffer of C rows (C >= max_j |N_j|), chunks taken in the
// given order (order[j] = chunk id at position j).
//   policy 0  adjacent reuse (Sec. 5.1, step 2): after a chunk every row the
//             next chunk does not need is released, whatever C is.
//   policy 1  a row is released right after the last chunk that needs it;
//             a row with a later use is released only when room is needed,
//             and then the rows whose next use lies farthest ahead go first
//             (equal next use: smaller id first).  With the whole schedule
//             known in advance this is the paging rule that loads the fewest
//             rows (Belady); the paper's Sec. 5.3 formula is policy 0.
// Per position j: reuse_j = N_j ^ resident, load_j = N_j \ resident (both
// ascending), leave_j = rows released after chunk j (ascending; after the last
// chunk everything still resident).  Lists are written back to back into
// reuse / load / leave (each must hold sum_j |N_j| entries), counts into n_*.
void orc_cache_schedule(const int64_t* indptr, const int32_t* col, int n, const int64_t* b, const int32_t* order,
                        int64_t C, int policy, int64_t* n_reuse, int64_t* n_load, int64_t* n_leave, int32_t* reuse,
                        int32_t* load, int32_t* leave) {
  std::vector<std::vector<int32_t>> N(n);
  for (int j = 0; j < n; ++j) {
    const int id = order[j];
    N[j].assign(col + indptr[b[id]], col + indptr[b[id + 1]]);
    std::sort(N[j].begin(), N[j].end());
    N[j].erase(std::unique(N[j].begin(), N[j].end()), N[j].end());
  }
  // next use of u strictly after position j: first k > j with u in N_k, else n
  auto next_use = [&](int32_t u, int j) {
    for (int k = j + 1; k < n; ++k)
      if (std::binary_search(N[k].begin(), N[k].end(), u)) return k;
    return n;
  };
  std::set<int32_t> resident;
  int64_t ro = 0, lo = 0, vo = 0;
  for (int j = 0; j < n; ++j) {
    // room for N_j: release rows that are resident, not needed now, farthest next use first
    if (j > 0) {
      std::vector<int32_t> out;
      if (policy == 0) {
        for (int32_t u : resident)
          if (!std::binary_search(N[j].begin(), N[j].end(), u)) out.push_back(u);
      } else {
        for (int32_t u : resident)
          if (next_use(u, j - 1) == n) out.push_back(u);      // not needed at position j or later
        for (int32_t u : out) resident.erase(u);
        std::set<int32_t> uni(resident);
        uni.insert(N[j].begin(), N[j].end());
        int64_t over = (int64_t)uni.size() - C;
        if (over > 0) {
          std::vector<std::pair<int, int32_t>> cand;   // (-next use, id): ascending order = farthest first, then smaller id
          for (int32_t u : resident)
            if (!std::binary_search(N[j].begin(), N[j].end(), u)) cand.push_back({-next_use(u, j), u});
          std::sort(cand.begin(), cand.end());
          for (int64_t k = 0; k < over; ++k) out.push_back(cand[k].second);
        }
        std::sort(out.begin(), out.end());
      }
      n_leave[j - 1] = (int64_t)out.size();
      for (int32_t u : out) {
        leave[vo++] = u;
        resident.erase(u);
      }
    }
    int64_t nr = 0, nl = 0;
    for (int32_t u : N[j]) {
      if (resident.count(u)) {
        reuse[ro++] = u;
        ++nr;
      } else {
        load[lo++] = u;
        ++nl;
      }
    }
    n_reuse[j] = nr;
    n_load[j] = nl;
    resident.insert(N[j].begin(), N[j].end());
  }
  if (n > 0) {
    n_leave[n - 1] = (int64_t)resident.size();
    for (int32_t u : resident) leave[vo++] = u;
  }
}

// ---------------------------------------------------------------------------
// Float part (fp64)
// ---------------------------------------------------------------------------

// s_v = 1/sqrt(D_v), D_v = number of stored in-edges of v (self-loop and
// multiplicity included).  One D on both sides of the symmetric normalisation.
void orc_norm(int64_t V, const int64_t* indptr, double* s) {
  for (int64_t v = 0; v < V; ++v) {
    int64_t D = indptr[v + 1] - indptr[v];
    s[v] = D > 0 ? 1.0 / std::sqrt((double)D) : 0.0;
  }
}

// AGGREGATE of Eq. 2:  a[v] = s_v * sum_{e in in(v)} s_{u_e} h[u_e],  rows v in [v0, v1).
void orc_aggregate(const int64_t* indptr, const int32_t* col, const double* s, int64_t v0,
                   int64_t v1, int64_t d, const double* h, double* a) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t v = v0; v < v1; ++v) {
    double* av = a + v * d;
    for (int64_t k = 0; k < d; ++k) av[k] = 0.0;
    for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
      const int64_t u = col[e];
      const double w = s[u];
      const double* hu = h + u * d;
      for (int64_t k = 0; k < d; ++k) av[k] += w * hu[k];
    }
    for (int64_t k = 0; k < d; ++k) av[k] *= s[v];
  }
}

// Backward of AGGREGATE:  g[u] = s_u * sum_{(u->v)} s_v x[v]  over all stored edges.
// Written as a loop over destinations scattering into sources (serial, plain).
void orc_aggregate_T(int64_t V, const int64_t* indptr, const int32_t* col, const double* s,
                     int64_t d, const double* x, double* g) {
  for (int64_t i = 0; i < V * d; ++i) g[i] = 0.0;
  for (int64_t v = 0; v < V; ++v)
    for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
      const int64_t u = col[e];
      const double w = s[v];
      for (int64_t k = 0; k < d; ++k) g[u * d + k] += w * x[v * d + k];
    }
  for (int64_t u = 0; u < V; ++u)
    for (int64_t k = 0; k < d; ++k) g[u * d + k] *= s[u];
}

// C[M x N] = A[M x K] * B[K x N]
void orc_matmul(int64_t M, int64_t K, int64_t N, const double* A, const double* B, double* C) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i) {
    for (int64_t j = 0; j < N; ++j) C[i * N + j] = 0.0;
    for (int64_t k = 0; k < K; ++k) {
      const double aik = A[i * K + k];
      for (int64_t j = 0; j < N; ++j) C[i * N + j] += aik * B[k * N + j];
    }
  }
}

// C[K x N] = A[M x K]^T * B[M x N]   (parallel over the K output rows)
void orc_matmul_tn(int64_t M, int64_t K, int64_t N, const double* A, const double* B, double* C) {
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < K; ++k) {
    for (int64_t j = 0; j < N; ++j) C[k * N + j] = 0.0;
    for (int64_t i = 0; i < M; ++i) {
      const double aik = A[i * K + k];
      for (int64_t j = 0; j < N; ++j) C[k * N + j] += aik * B[i * N + j];
    }
  }
}

// C[M x K] = A[M x N] * B[K x N]^T
void orc_matmul_nt(int64_t M, int64_t N, int64_t K, const double* A, const double* B, double* C) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i)
    for (int64_t k = 0; k < K; ++k) {
      double acc = 0.0;
      for (int64_t j = 0; j < N; ++j) acc += A[i * N + j] * B[k * N + j];
      C[i * K + k] = acc;
    }
}

// Softmax cross-entropy, mean over labelled vertices (label >= 0).
// grad[v] = (softmax(logits_v) - onehot(y_v)) / |T| for labelled v, else 0.
double orc_softmax_ce(int64_t V, int64_t C, const double* logits, const int32_t* labels,
                      double* grad) {
  int64_t T = 0;
  for (int64_t v = 0; v < V; ++v) T += labels[v] >= 0;
  double loss = 0.0;
  for (int64_t v = 0; v < V; ++v) {
    double* gv = grad ? grad + v * C : nullptr;
    if (labels[v] < 0) {
      if (gv) for (int64_t c = 0; c < C; ++c) gv[c] = 0.0;
      continue;
    }
    const double* x = logits + v * C;
    double m = x[0];
    for (int64_t c = 1; c < C; ++c) m = std::max(m, x[c]);
    double z = 0.0;
    for (int64_t c = 0; c < C; ++c) z += std::exp(x[c] - m);
    const double lse = m + std::log(z);
    loss += lse - x[labels[v]];
    if (gv)
      for (int64_t c = 0; c < C; ++c)
        gv[c] = (std::exp(x[c] - lse) - (c == labels[v] ? 1.0 : 0.0)) / (double)T;
  }
  return T > 0 ? loss / (double)T : 0.0;
}

// One training epoch of an L-layer GCN (Alg. 1 without the partitioning, which
// does not change the result): forward, loss, backward, SGD step.
//   dims[L+1]; X fp32 [V x dims[0]]; W fp32, the L matrices [dims[l] x dims[l+1]]
//   back to back; labels int32 (-1 = unlabelled).
// Outputs (each array may be null to skip it), per layer l = 0..L-1:
//   a[l]  [V x dims[l]]    aggregate output a^l
//   z[l]  [V x dims[l+1]]  pre-activation a^l W^l
//   h[l]  [V x dims[l+1]]  h^{l+1} = ReLU(z^l), identity on the last layer
//   gh[l] [V x dims[l+1]]  gradient of the loss w.r.t. h^{l+1}
//   ga[l] [V x dims[l]]    gradient w.r.t. a^l
//   gW    concatenated like W;  W_new = W - lr * gW;  *loss.
// ReLU'(z) = [z > 0] (Sec. 2.3: 1 for positive inputs and 0 otherwise).
int orc_gcn_epoch(int64_t V, const int64_t* indptr, const int32_t* col, int L,
                  const int32_t* dims, const float* X, const float* W, const int32_t* labels,
                  double lr, double** a_out, double** z_out, double** h_out,
                  double** gh_out, double** ga_out, double* gW_out, double* W_new,
                  double* loss_out) {
  std::vector<double> s(V);
  orc_norm(V, indptr, s.data());
  std::vector<std::vector<double>> h(L + 1), a(L), z(L), Wd(L);
  std::vector<int64_t> woff(L + 1, 0);
  for (int l = 0; l < L; ++l) woff[l + 1] = woff[l] + (int64_t)dims[l] * dims[l + 1];
  h[0].assign(X, X + V * (int64_t)dims[0]);
  for (int l = 0; l < L; ++l) Wd[l].assign(W + woff[l], W + woff[l + 1]);

  for (int l = 0; l < L; ++l) {
    const int64_t di = dims[l], dn = dims[l + 1];
    a[l].resize(V * di);
    z[l].resize(V * dn);
    h[l + 1].resize(V * dn);
    orc_aggregate(indptr, col, s.data(), 0, V, di, h[l].data(), a[l].data());
    orc_matmul(V, di, dn, a[l].data(), Wd[l].data(), z[l].data());
    for (int64_t i = 0; i < V * dn; ++i)
      h[l + 1][i] = (l < L - 1) ? std::max(z[l][i], 0.0) : z[l][i];
  }
  std::vector<double> gh(V * (int64_t)dims[L]);
  const double loss = orc_softmax_ce(V, dims[L], h[L].data(), labels, gh.data());
  if (loss_out) *loss_out = loss;

  for (int l = L - 1; l >= 0; --l) {
    const int64_t di = dims[l], dn = dims[l + 1];
    if (gh_out && gh_out[l]) std::memcpy(gh_out[l], gh.data(), sizeof(double) * V * dn);
    std::vector<double> gz(V * dn);
    for (int64_t i = 0; i < V * dn; ++i)
      gz[i] = (l < L - 1) ? (z[l][i] > 0.0 ? gh[i] : 0.0) : gh[i];
    std::vector<double> gW(di * dn);
    orc_matmul_tn(V, di, dn, a[l].data(), gz.data(), gW.data());
    std::vector<double> ga(V * di);
    orc_matmul_nt(V, dn, di, gz.data(), Wd[l].data(), ga.data());
    if (ga_out && ga_out[l]) std::memcpy(ga_out[l], ga.data(), sizeof(double) * V * di);
    if (gW_out) std::memcpy(gW_out + woff[l], gW.data(), sizeof(double) * di * dn);
    if (W_new)
      for (int64_t i = 0; i < di * dn; ++i) W_new[woff[l] + i] = Wd[l][i] - lr * gW[i];
    if (l > 0) {
      gh.assign(V * di, 0.0);
      orc_aggregate_T(V, indptr, col, s.data(), di, ga.data(), gh.data());
    }
  }
  for (int l = 0; l < L; ++l) {
    if (a_out && a_out[l]) std::memcpy(a_out[l], a[l].data(), sizeof(double) * a[l].size());
    if (z_out && z_out[l]) std::memcpy(z_out[l], z[l].data(), sizeof(double) * z[l].size());
    if (h_out && h_out[l]) std::memcpy(h_out[l], h[l + 1].data(), sizeof(double) * h[l + 1].size());
  }
  return 0;
}

// The same layer step done chunk by chunk through the dedup structures
// (Sec. 4.1, 5.1): forward reads the rows of N_j by local index; backward
// sums each chunk's source gradients into the full gradient buffer.  Used to
// pin "partitioned == unpartitioned" and to tie the integer part to the float
// part.  b[n+1] are chunk boundaries.
void orc_layer_fwd_chunked(int64_t V, const int64_t* indptr, const int32_t* col, int n,
                           const int64_t* b, int64_t d, const double* h, double* a) {
  std::vector<double> s(V);
  orc_norm(V, indptr, s.data());
  for (int j = 0; j < n; ++j) {
    const int64_t b0 = b[j], b1 = b[j + 1], e0 = indptr[b0], ne = indptr[b1] - e0;
    const int64_t ns = orc_chunk_nsrc(indptr, col, b0, b1);
    std::vector<int32_t> N(ns), cl(ne), sdst(ne);
    std::vector<int64_t> sptr(ns + 1);
    orc_chunk_dedup(indptr, col, b0, b1, N.data(), cl.data(), sptr.data(), sdst.data());
    std::vector<double> buf(ns * d);  // the chunk's neighbour rows, one per unique source
    for (int64_t i = 0; i < ns; ++i)
      for (int64_t k = 0; k < d; ++k) buf[i * d + k] = s[N[i]] * h[(int64_t)N[i] * d + k];
    for (int64_t v = b0; v < b1; ++v) {
      for (int64_t k = 0; k < d; ++k) a[v * d + k] = 0.0;
      for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e)
        for (int64_t k = 0; k < d; ++k) a[v * d + k] += buf[(int64_t)cl[e - e0] * d + k];
      for (int64_t k = 0; k < d; ++k) a[v * d + k] *= s[v];
    }
  }
}

void orc_layer_bwd_chunked(int64_t V, const int64_t* indptr, const int32_t* col, int n,
                           const int64_t* b, int64_t d, const double* ga, double* gh) {
  std::vector<double> s(V);
  orc_norm(V, indptr, s.data());
  for (int64_t i = 0; i < V * d; ++i) gh[i] = 0.0;
  for (int j = 0; j < n; ++j) {
    const int64_t b0 = b[j], b1 = b[j + 1], ne = indptr[b1] - indptr[b0];
    const int64_t ns = orc_chunk_nsrc(indptr, col, b0, b1);
    std::vector<int32_t> N(ns), cl(ne), sdst(ne);
    std::vector<int64_t> sptr(ns + 1);
    orc_chunk_dedup(indptr, col, b0, b1, N.data(), cl.data(), sptr.data(), sdst.data());
    for (int64_t i = 0; i < ns; ++i) {
      const int64_t u = N[i];
      for (int64_t k = 0; k < d; ++k) {
        double acc = 0.0;
        for (int64_t t = sptr[i]; t < sptr[i + 1]; ++t) {
          const int64_t v = b0 + sdst[t];
          acc += s[v] * ga[v * d + k];
        }
        gh[u * d + k] += s[u] * acc;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// GAT layer (Eq. 3), one attention head
// ---------------------------------------------------------------------------
// For every stored edge e = (u -> v) of the CSC (multi-edges each count, the
// self-loop is an edge like any other):
//   t = H W                                   parameterised representations
//   y_e = a_dst . t_v + a_src . t_u           a^l applied to [W h_v || W h_u]
//   x_e = LeakyReLU(y_e)                      slope for y_e <= 0, 1 for y_e > 0
//   alpha_e = exp(x_e) / sum_{e' in in(v)} exp(x_e')    neighbour-oriented softmax
//   z_v = sum_{e in in(v)} alpha_e t_u ;  h'_v = ReLU(z_v) (or z_v)
// Readings: the rows that are summed are the parameterised ones (W h_u), as
// in the attention model the equation cites (the printed sum shows h_u); the
// first half of a^l multiplies the destination's half of the concatenation; the
// softmax subtracts the row maximum (same value, no overflow).
// A vertex with no in-edge (only possible without self-loops) gets z_v = 0.
void orc_gat_fwd(int64_t V, const int64_t* indptr, const int32_t* col, int64_t d_in, int64_t d_out, const double* H,
                 const double* W, const double* a_dst, const double* a_src, double slope, int relu, double* T,
                 double* alpha, double* Z, double* out) {
  orc_matmul(V, d_in, d_out, H, W, T);
  std::vector<double> p(V), q(V);
  for (int64_t v = 0; v < V; ++v) {
    double sp = 0.0, sq = 0.0;
    for (int64_t k = 0; k < d_out; ++k) {
      sp += a_dst[k] * T[v * d_out + k];
      sq += a_src[k] * T[v * d_out + k];
    }
    p[v] = sp;
    q[v] = sq;
  }
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t v = 0; v < V; ++v) {
    const int64_t e0 = indptr[v], e1 = indptr[v + 1];
    double m = -1e300;
    for (int64_t e = e0; e < e1; ++e) {
      const double y = p[v] + q[col[e]];
      const double x = y > 0.0 ? y : slope * y;
      alpha[e] = x;
      if (x > m) m = x;
    }
    double sum = 0.0;
    for (int64_t e = e0; e < e1; ++e) {
      alpha[e] = std::exp(alpha[e] - m);
      sum += alpha[e];
    }
    for (int64_t k = 0; k < d_out; ++k) Z[v * d_out + k] = 0.0;
    for (int64_t e = e0; e < e1; ++e) {
      alpha[e] /= sum;
      const double* tu = T + (int64_t)col[e] * d_out;
      for (int64_t k = 0; k < d_out; ++k) Z[v * d_out + k] += alpha[e] * tu[k];
    }
    for (int64_t k = 0; k < d_out; ++k) {
      const double z = Z[v * d_out + k];
      out[v * d_out + k] = (relu && !(z > 0.0)) ? 0.0 : z;
    }
  }
}

// Chain rule through the layer above, edge by edge.  dOut = grad h'.
//   dz = dOut * [z > 0]
//   d alpha_e = dz_v . t_u ;  dt_u += alpha_e dz_v
//   softmax:   dx_e = alpha_e (d alpha_e - sum_{e'} alpha_e' d alpha_e')
//   LeakyReLU: dy_e = dx_e * (1 if y_e > 0 else slope)
//   dp_v += dy_e ; dq_u += dy_e ;  dt_v += dp_v a_dst ; dt_u += dq_u a_src
//   da_dst = sum_v dp_v t_v ; da_src = sum_u dq_u t_u ; dW = H^T dt ; dH = dt W^T
// Two sweeps so that every loop runs over independent rows: destinations first
// (d alpha, dy_e, dp_v), then sources over their out-edges in edge order
// (dt_u, dq_u); the out-edge lists come from a counting sort of the edge ids.
void orc_gat_bwd(int64_t V, const int64_t* indptr, const int32_t* col, int64_t d_in, int64_t d_out, const double* H,
                 const double* W, const double* a_dst, const double* a_src, double slope, int relu, const double* T,
                 const double* alpha, const double* Z, const double* dOut,
                 double* dH, double* dW, double* da_dst, double* da_src) {
  const int64_t E = indptr[V];
  std::vector<double> p(V), q(V), dp(V, 0.0), dq(V, 0.0), dT((size_t)V * d_out, 0.0), dy((size_t)E);
  for (int64_t v = 0; v < V; ++v) {
    double sp = 0.0, sq = 0.0;
    for (int64_t k = 0; k < d_out; ++k) {
      sp += a_dst[k] * T[v * d_out + k];
      sq += a_src[k] * T[v * d_out + k];
    }
    p[v] = sp;
    q[v] = sq;
  }
  auto dz_at = [&](int64_t v, int64_t k) { return (relu && !(Z[v * d_out + k] > 0.0)) ? 0.0 : dOut[v * d_out + k]; };
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t v = 0; v < V; ++v) {
    const int64_t e0 = indptr[v], e1 = indptr[v + 1];
    double S = 0.0;
    for (int64_t e = e0; e < e1; ++e) {
      const int64_t u = col[e];
      double dot = 0.0;
      for (int64_t k = 0; k < d_out; ++k) dot += dz_at(v, k) * T[u * d_out + k];
      dy[e] = dot;                       // d alpha_e for now
      S += alpha[e] * dot;
    }
    double acc = 0.0;
    for (int64_t e = e0; e < e1; ++e) {
      const double dx = alpha[e] * (dy[e] - S);
      const double y = p[v] + q[col[e]];
      dy[e] = dx * (y > 0.0 ? 1.0 : slope);
      acc += dy[e];
    }
    dp[v] = acc;
  }
  // out-edges of every source, ascending edge id
  std::vector<int64_t> optr(V + 1, 0), oedge((size_t)E);
  std::vector<int32_t> dst_of((size_t)E);
  for (int64_t v = 0; v < V; ++v)
    for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
      dst_of[e] = (int32_t)v;
      optr[col[e] + 1]++;
    }
  for (int64_t u = 0; u < V; ++u) optr[u + 1] += optr[u];
  {
    std::vector<int64_t> pos(optr.begin(), optr.end() - 1);
    for (int64_t e = 0; e < E; ++e) oedge[pos[col[e]]++] = e;
  }
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t u = 0; u < V; ++u) {
    double acc = 0.0;
    for (int64_t i = optr[u]; i < optr[u + 1]; ++i) {
      const int64_t e = oedge[i], v = dst_of[e];
      for (int64_t k = 0; k < d_out; ++k) dT[u * d_out + k] += alpha[e] * dz_at(v, k);
      acc += dy[e];
    }
    dq[u] = acc;
  }
  for (int64_t k = 0; k < d_out; ++k) da_dst[k] = da_src[k] = 0.0;
  for (int64_t v = 0; v < V; ++v)
    for (int64_t k = 0; k < d_out; ++k) {
      dT[v * d_out + k] += dp[v] * a_dst[k] + dq[v] * a_src[k];
      da_dst[k] += dp[v] * T[v * d_out + k];
      da_src[k] += dq[v] * T[v * d_out + k];
    }
  orc_matmul_tn(V, d_in, d_out, H, dT.data(), dW);
  if (dH) orc_matmul_nt(V, d_out, d_in, dT.data(), W, dH);
}

}  // extern "C"

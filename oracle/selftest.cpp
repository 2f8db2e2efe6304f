// Sanitizer run of the CPU oracle (test infrastructure): every entry point once on small random
// inputs, in one translation unit with the oracle so that AddressSanitizer and
// UndefinedBehaviorSanitizer see all of it.  Built and run by tests/test_oracle_sanitized.py:
//   g++ -O1 -g -fopenmp -fsanitize=address,undefined -fno-sanitize-recover=all -static-libasan oracle/selftest.cpp
// The results are only checked for being finite and for a few invariants; parity pins live in tests/.
#include "gcn_oracle.cpp"

#include <cstdio>
#include <cstdlib>

namespace {
uint64_t state = 88172645463325252ull;
uint64_t rnd() { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return state; }
double rnd_unit() { return (double)(rnd() >> 11) / 9007199254740992.0 - 0.5; }
void need(bool ok, const char* what) {
  if (!ok) {
    std::fprintf(stderr, "selftest: %s\n", what);
    std::exit(1);
  }
}
bool finite_all(const std::vector<double>& x) {
  for (double v : x)
    if (!std::isfinite(v)) return false;
  return true;
}
}  // namespace

int main() {
  for (int self_loops = 0; self_loops < 2; ++self_loops) {
    const int64_t V = 61, E = 420;
    std::vector<int32_t> src(E), dst(E);
    for (int64_t i = 0; i < E; ++i) {
      src[i] = (int32_t)(rnd() % V);
      dst[i] = (int32_t)(i % 7 == 0 ? 3 : rnd() % V);       // a hub destination, repeated pairs
    }
    std::vector<int64_t> indptr(V + 1);
    std::vector<int32_t> col(E + V);
    const int64_t Ep = orc_csc_build(V, E, src.data(), dst.data(), self_loops, indptr.data(), col.data());
    need(Ep == E + (self_loops ? V : 0) && indptr[V] == Ep, "stored edge count");
    col.resize(Ep > 0 ? Ep : 1);

    for (int mode = 0; mode < 2; ++mode) {
      for (int n : {1, 5, 70}) {
        std::vector<int64_t> b(n + 1);
        orc_chunk_bounds(V, indptr.data(), n, mode, b.data());
        need(b[0] == 0 && b[n] == V, "chunk bounds tile the vertices");
        int64_t v_ori = 0, v_ru = 0, max_nsrc = 1, total = 0;
        orc_volumes(V, indptr.data(), col.data(), n, b.data(), &v_ori, &v_ru);
        std::vector<int32_t> prev;
        for (int j = 0; j < n; ++j) {
          const int64_t ns = orc_chunk_nsrc(indptr.data(), col.data(), b[j], b[j + 1]);
          const int64_t ne = indptr[b[j + 1]] - indptr[b[j]];
          std::vector<int32_t> N(ns ? ns : 1), cl(ne ? ne : 1), sd(ne ? ne : 1), R(ns ? ns : 1), Ld(ns ? ns : 1);
          std::vector<int64_t> sptr(ns + 1);
          orc_chunk_dedup(indptr.data(), col.data(), b[j], b[j + 1], N.data(), cl.data(), sptr.data(), sd.data());
          int64_t nR = 0, nLd = 0;
          orc_reuse_split(prev.data(), (int64_t)prev.size(), N.data(), ns, R.data(), Ld.data(), &nR, &nLd);
          need(nR + nLd == ns && sptr[ns] == ne, "dedup / reuse split sizes");
          prev.assign(N.begin(), N.begin() + ns);
          max_nsrc = std::max(max_nsrc, ns);
          total += ns;
        }
        need(total == v_ori && v_ru <= v_ori, "volumes");
        std::vector<int32_t> order(n);
        orc_chunk_order(indptr.data(), col.data(), n, b.data(), order.data());
        for (int policy = 0; policy < 2; ++policy)
          for (int64_t C : {max_nsrc, max_nsrc + 7, (int64_t)V}) {
            std::vector<int64_t> nr(n), nl(n), nv(n);
            std::vector<int32_t> ru(total + 1), ld(total + 1), lv(total + 1);
            orc_cache_schedule(indptr.data(), col.data(), n, b.data(), order.data(), C, policy, nr.data(), nl.data(),
                               nv.data(), ru.data(), ld.data(), lv.data());
            int64_t loads = 0, leaves = 0;
            for (int j = 0; j < n; ++j) { loads += nl[j]; leaves += nv[j]; }
            need(loads == leaves, "every loaded row leaves");
          }
        // the same chunks read as m partitions of n / m subgraphs: reorganisation and volumes
        for (int m : {1, 2, 3})
          if (n % m == 0) {
            const int nn = n / m;
            std::vector<int32_t> lay(n), ident(n);
            for (int c = 0; c < n; ++c) ident[c] = c % nn;
            orc_reorganize(indptr.data(), col.data(), m, nn, b.data(), lay.data());
            int64_t v0[3], v1[3];
            orc_volumes_mn(indptr.data(), col.data(), m, nn, b.data(), ident.data(), v0);
            orc_volumes_mn(indptr.data(), col.data(), m, nn, b.data(), lay.data(), v1);
            need(v0[0] == v1[0] && v0[0] == v_ori && v1[1] <= v1[0] && v1[2] <= v1[1], "volumes of m partitions");
          }
        // one layer step chunk by chunk, both directions
        const int64_t d = 9;
        std::vector<double> h(V * d), a(V * d), ga(V * d), gh(V * d);
        for (double& x : h) x = rnd_unit();
        for (double& x : ga) x = rnd_unit();
        orc_layer_fwd_chunked(V, indptr.data(), col.data(), n, b.data(), d, h.data(), a.data());
        orc_layer_bwd_chunked(V, indptr.data(), col.data(), n, b.data(), d, ga.data(), gh.data());
        need(finite_all(a) && finite_all(gh), "chunked layer step is finite");
      }
    }

    // whole GCN epoch
    const int L = 3;
    const int32_t dims[L + 1] = {11, 8, 6, 4};
    std::vector<float> X(V * dims[0]), W;
    for (float& x : X) x = (float)rnd_unit();
    for (int l = 0; l < L; ++l)
      for (int i = 0; i < dims[l] * dims[l + 1]; ++i) W.push_back((float)rnd_unit());
    std::vector<int32_t> labels(V);
    for (int64_t v = 0; v < V; ++v) labels[v] = v % 5 == 0 ? -1 : (int32_t)(rnd() % dims[L]);
    std::vector<std::vector<double>> a(L), z(L), h(L), gh(L), ga(L);
    std::vector<double*> ap(L), zp(L), hp(L), ghp(L), gap(L);
    for (int l = 0; l < L; ++l) {
      a[l].resize(V * dims[l]); z[l].resize(V * dims[l + 1]); h[l].resize(V * dims[l + 1]);
      gh[l].resize(V * dims[l + 1]); ga[l].resize(V * dims[l]);
      ap[l] = a[l].data(); zp[l] = z[l].data(); hp[l] = h[l].data(); ghp[l] = gh[l].data(); gap[l] = ga[l].data();
    }
    std::vector<double> gW(W.size()), Wn(W.size());
    double loss = 0.0;
    need(orc_gcn_epoch(V, indptr.data(), col.data(), L, dims, X.data(), W.data(), labels.data(), 0.01, ap.data(),
                       zp.data(), hp.data(), ghp.data(), gap.data(), gW.data(), Wn.data(), &loss) == 0,
         "gcn epoch");
    need(std::isfinite(loss) && finite_all(gW) && finite_all(Wn), "gcn epoch is finite");
    // and without the optional outputs
    need(orc_gcn_epoch(V, indptr.data(), col.data(), L, dims, X.data(), W.data(), labels.data(), 0.01, nullptr,
                       nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == 0,
         "gcn epoch without outputs");

    // GAT layer forward and backward
    const int64_t di = 7, dn = 5;
    std::vector<double> H(V * di), Wg(di * dn), ad(dn), as(dn), T(V * dn), alpha(Ep ? Ep : 1), Z(V * dn), out(V * dn),
        dOut(V * dn), dH(V * di), dW(di * dn), dad(dn), das(dn);
    for (double& x : H) x = rnd_unit();
    for (double& x : Wg) x = rnd_unit();
    for (double& x : ad) x = rnd_unit();
    for (double& x : as) x = rnd_unit();
    for (double& x : dOut) x = rnd_unit();
    for (int relu = 0; relu < 2; ++relu) {
      orc_gat_fwd(V, indptr.data(), col.data(), di, dn, H.data(), Wg.data(), ad.data(), as.data(), 0.2, relu, T.data(),
                  alpha.data(), Z.data(), out.data());
      orc_gat_bwd(V, indptr.data(), col.data(), di, dn, H.data(), Wg.data(), ad.data(), as.data(), 0.2, relu, T.data(),
                  alpha.data(), Z.data(), dOut.data(), dH.data(), dW.data(), dad.data(), das.data());
      need(finite_all(out) && finite_all(dH) && finite_all(dW) && finite_all(dad) && finite_all(das), "GAT layer is finite");
    }
  }
  std::puts("oracle selftest: ok");
  return 0;
}

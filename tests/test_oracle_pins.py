"""Pins of the CPU oracle against things other than itself.

Every check here compares oracle/ with something the paper or the mathematics
fixes: dense matrices and torch autograd on tiny graphs, finite differences,
closed forms on regular graphs, the paper's printed worked examples, brute
force Python sets, scipy's sparse routines.  None of them needs a GPU.
"""
import math
import os

import numpy as np
import pytest
import scipy.sparse as sp
import torch

from oracle import oracle as orc
from paper_2311_14898_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if ":" in line:
                k, v = line.split(":")
                out[k.strip()] = [int(x) for x in v.split()]
            else:
                rows.append(line.split())
    return out, rows


def _tiny_graph(V, E, seed):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, V, size=E).astype(np.int32)
    dst = rng.integers(0, V, size=E).astype(np.int32)
    keep = src != dst
    src, dst = src[keep], dst[keep]
    # force a few duplicate edges so multiplicity is exercised
    src = np.concatenate([src, src[:3]])
    dst = np.concatenate([dst, dst[:3]])
    return src, dst


def _dense_norm_adj(V, src, dst):
    """D^-1/2 (A + I) D^-1/2 as a dense fp64 matrix, multiplicities kept."""
    At = np.zeros((V, V))
    np.add.at(At, (dst, src), 1.0)      # row = destination, column = source
    At += np.eye(V)
    D = At.sum(axis=1)
    s = 1.0 / np.sqrt(D)
    return s[:, None] * At * s[None, :]


# ------------------------------------------------------------------ integer part

def test_csc_build_against_scipy_and_order():
    V = 40
    src, dst = _tiny_graph(V, 300, 0)
    indptr, col = orc.csc_build(V, src, dst, add_self_loops=True)
    assert indptr[0] == 0 and indptr[-1] == len(src) + V == len(col)
    # multiplicity matrix equals scipy's duplicate-summing COO -> dense
    ref = sp.coo_matrix((np.ones(len(src)), (dst, src)), shape=(V, V)).toarray() + np.eye(V)
    got = np.zeros((V, V))
    for v in range(V):
        seg = col[indptr[v]:indptr[v + 1]]
        assert np.all(np.diff(seg) >= 0), "sources ascend inside a destination"
        np.add.at(got[v], seg, 1.0)
    assert np.array_equal(got, ref)
    # without self loops
    indptr2, col2 = orc.csc_build(V, src, dst, add_self_loops=False)
    assert indptr2[-1] == len(src)


def test_chunk_bounds_properties_and_closed_form():
    # k-regular ring-like graph: every vertex has exactly k in-edges + self loop
    V, k, n = 120, 3, 7
    src = np.concatenate([(np.arange(V) + o) % V for o in range(1, k + 1)]).astype(np.int32)
    dst = np.tile(np.arange(V), k).astype(np.int32)
    indptr, col = orc.csc_build(V, src, dst)
    b = orc.chunk_bounds(indptr, n, mode=0)
    assert b[0] == 0 and b[-1] == V and np.all(np.diff(b) >= 0)
    assert np.array_equal(b, [math.ceil(j * V / n) for j in range(n + 1)])   # closed form on a regular graph
    b1 = orc.chunk_bounds(indptr, n, mode=1)
    assert np.array_equal(b1, [(j * V) // n for j in range(n + 1)])
    # n = 1 is the whole graph; chunk nnz sum to E'
    assert np.array_equal(orc.chunk_bounds(indptr, 1), [0, V])
    assert sum(indptr[b[j + 1]] - indptr[b[j]] for j in range(n)) == indptr[-1]
    # skewed graph: definition checked by brute force
    src, dst = _tiny_graph(50, 400, 3)
    dst = (dst // 3).astype(np.int32)            # pile edges on low destinations
    keep = src != dst
    indptr, col = orc.csc_build(50, src[keep], dst[keep])
    Ep = int(indptr[-1])
    for n in (2, 3, 5, 64):
        b = orc.chunk_bounds(indptr, n)
        for j in range(1, n):
            target = -(-j * Ep // n)
            cand = [v for v in range(50) if indptr[v] >= target]
            assert b[j] == (cand[0] if cand else 50)


def test_dedup_against_python_sets():
    V = 45
    src, dst = _tiny_graph(V, 260, 5)
    indptr, col = orc.csc_build(V, src, dst)
    b = orc.chunk_bounds(indptr, 4)
    prev = set()
    v_ori = v_ru = 0
    for j in range(4):
        b0, b1 = int(b[j]), int(b[j + 1])
        r = orc.chunk_dedup(indptr, col, b0, b1)
        edges = [(int(col[e]), v) for v in range(b0, b1) for e in range(indptr[v], indptr[v + 1])]
        Nset = sorted({u for u, _ in edges})
        assert r["N"].tolist() == Nset
        assert [Nset[i] for i in r["col_local"]] == [u for u, _ in edges]
        # CSR by source holds the same multiset of edges, rows ascending in destination
        back = []
        for i in range(len(Nset)):
            seg = r["sdst"][r["sptr"][i]:r["sptr"][i + 1]]
            assert np.all(np.diff(seg) >= 0)
            back += [(Nset[i], b0 + int(t)) for t in seg]
        assert sorted(back) == sorted(edges)
        R, Ld = orc.reuse_split(np.array(sorted(prev), dtype=np.int32), r["N"])
        assert R.tolist() == sorted(set(Nset) & prev)
        assert Ld.tolist() == sorted(set(Nset) - prev)
        v_ori += len(Nset)
        v_ru += len(set(Nset) - prev)
        prev = set(Nset)
    assert orc.volumes(indptr, col, b) == (v_ori, v_ru)
    # with a self-loop on every vertex each vertex is a source somewhere
    assert V <= v_ru <= v_ori


def test_paper_transfer_count_example():
    g, _ = _golden("dedup_transfer_counts.txt")
    u0, u1 = g["union0"], g["union1"]
    assert len(u0) + len(u1) == g["transfers_after_union"][0]
    R, Ld = orc.reuse_split(np.array(u0, dtype=np.int32), np.array(u1, dtype=np.int32))
    assert len(u0) + len(Ld) == g["transfers_after_reuse"][0]
    # the same through the volume routine: a graph whose two chunks have exactly these source sets
    src = np.array(u0 + u1, dtype=np.int32)
    dst = np.array([8] * len(u0) + [9] * len(u1), dtype=np.int32)
    indptr, col = orc.csc_build(10, src, dst, add_self_loops=False)
    vo, vr = orc.volumes(indptr, col, np.array([0, 9, 10]))
    assert (vo, vr) == (g["transfers_after_union"][0], g["transfers_after_reuse"][0])


def test_paper_inplace_buffer_example_sets():
    g, _ = _golden("inplace_buffer_example.txt")
    R, Ld = orc.reuse_split(np.array(g["prev"], dtype=np.int32), np.array(g["next"], dtype=np.int32))
    assert R.tolist() == g["reused"] and Ld.tolist() == g["loaded"]
    assert sorted(set(g["prev"]) - set(g["next"])) == g["discarded"]
    assert len(g["loaded"]) <= len(g["discarded"])      # loads fit in freed positions


def test_table7_reduction_definition():
    _, rows = _golden("table7_duplication.txt")
    for name, vori, inter, intra, pct in rows:
        vori, inter, intra, pct = map(float, (vori, inter, intra, pct))
        assert abs(100.0 * (inter + intra) / vori - pct) < 0.06, name


# ------------------------------------------------------------------ float part

def _torch_dense_epoch(V, src, dst, dims, X, Ws, y, lr):
    """Dense fp64 forward with torch autograd for every gradient."""
    Ahat = torch.tensor(_dense_norm_adj(V, src, dst))
    Wt = [torch.tensor(np.asarray(w, dtype=np.float64), requires_grad=True) for w in Ws]
    h = torch.tensor(np.asarray(X, dtype=np.float64), requires_grad=True)
    keep = {"a": [], "h": []}
    L = len(dims) - 1
    for l in range(L):
        a = Ahat @ h
        a.retain_grad()
        z = a @ Wt[l]
        h = torch.relu(z) if l < L - 1 else z
        h.retain_grad()
        keep["a"].append(a)
        keep["h"].append(h)
    yt = torch.tensor(np.asarray(y), dtype=torch.int64)
    m = yt >= 0
    loss = torch.nn.functional.cross_entropy(h[m], yt[m], reduction="mean")
    loss.backward()
    return loss.item(), keep, Wt


@pytest.mark.parametrize("V,E,dims,seed", [(30, 150, [5, 7, 3], 0), (50, 400, [6, 4, 5, 3], 1)])
def test_epoch_against_dense_autograd(V, E, dims, seed):
    src, dst = _tiny_graph(V, E, seed)
    rng = np.random.default_rng(seed + 10)
    X = rng.standard_normal((V, dims[0])).astype(np.float32)
    Ws = [w.numpy() for w in inputs.glorot_weights(dims, seed=seed + 4)]
    y = rng.integers(0, dims[-1], size=V).astype(np.int32)
    y[::7] = -1                               # some unlabelled vertices
    indptr, col = orc.csc_build(V, src, dst)
    out = orc.gcn_epoch(indptr, col, dims, X, Ws, y, lr=0.05)
    loss, keep, Wt = _torch_dense_epoch(V, src, dst, dims, X, Ws, y, 0.05)
    assert abs(out["loss"] - loss) < 1e-12
    L = len(dims) - 1
    for l in range(L):
        np.testing.assert_allclose(out["a"][l], keep["a"][l].detach().numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(out["h"][l], keep["h"][l].detach().numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(out["gh"][l], keep["h"][l].grad.numpy(), rtol=0, atol=1e-13)
        np.testing.assert_allclose(out["ga"][l], keep["a"][l].grad.numpy(), rtol=0, atol=1e-13)
        np.testing.assert_allclose(out["gW"][l], Wt[l].grad.numpy(), rtol=0, atol=1e-13)
        np.testing.assert_allclose(out["W_new"][l], np.float64(Ws[l]) - 0.05 * Wt[l].grad.numpy(), rtol=0, atol=1e-13)


def test_finite_differences_of_loss():
    V, dims = 24, [4, 5, 3]
    src, dst = _tiny_graph(V, 100, 7)
    rng = np.random.default_rng(3)
    X = rng.standard_normal((V, dims[0])).astype(np.float32)
    Ws = [w.numpy().copy() for w in inputs.glorot_weights(dims, seed=11)]
    y = rng.integers(0, dims[-1], size=V).astype(np.int32)
    indptr, col = orc.csc_build(V, src, dst)
    base = orc.gcn_epoch(indptr, col, dims, X, Ws, y)
    # stay away from ReLU kinks so the central difference is valid
    assert np.abs(base["z"][0]).min() > 1e-3
    h = 1e-3     # weights are fp32 inputs: perturbations must be representable
    for l in range(2):
        for (i, j) in [(0, 0), (1, 2), (dims[l] - 1, dims[l + 1] - 1)]:
            Wp = [w.copy() for w in Ws]
            Wm = [w.copy() for w in Ws]
            Wp[l][i, j] += h
            Wm[l][i, j] -= h
            dp = float(np.float64(Wp[l][i, j]) - np.float64(Wm[l][i, j]))
            fp = orc.gcn_epoch(indptr, col, dims, X, Wp, y, want=())["loss"]
            fm = orc.gcn_epoch(indptr, col, dims, X, Wm, y, want=())["loss"]
            fd = (fp - fm) / dp
            assert abs(fd - base["gW"][l][i, j]) < 2e-6 * max(1.0, abs(fd)), (l, i, j)


def test_all_ones_gives_normalised_degree_sums_and_regular_graph_gives_one():
    V = 37
    src, dst = _tiny_graph(V, 200, 2)
    indptr, col = orc.csc_build(V, src, dst)
    a = orc.aggregate(indptr, col, np.ones((V, 3)))
    Ahat = _dense_norm_adj(V, src, dst)
    np.testing.assert_allclose(a, np.repeat(Ahat.sum(axis=1)[:, None], 3, axis=1), atol=1e-13)
    # k-regular (in-degree = out-degree = k): every D_v = k+1, so the sum is exactly 1
    V, k = 64, 5
    src = np.concatenate([(np.arange(V) + o) % V for o in range(1, k + 1)]).astype(np.int32)
    dst = np.tile(np.arange(V), k).astype(np.int32)
    indptr, col = orc.csc_build(V, src, dst)
    np.testing.assert_allclose(orc.aggregate(indptr, col, np.ones((V, 2))), 1.0, atol=1e-14)
    np.testing.assert_allclose(orc.aggregate_T(indptr, col, np.ones((V, 2))), 1.0, atol=1e-14)


def test_uniform_logits_loss_is_ln_C():
    V, dims = 20, [3, 4, 8]
    src, dst = _tiny_graph(V, 60, 4)
    indptr, col = orc.csc_build(V, src, dst)
    X = np.random.default_rng(0).standard_normal((V, 3)).astype(np.float32)
    Ws = [np.zeros((3, 4), np.float32), np.zeros((4, 8), np.float32)]
    y = np.arange(V, dtype=np.int32) % 8
    out = orc.gcn_epoch(indptr, col, dims, X, Ws, y)
    assert abs(out["loss"] - math.log(8)) < 1e-15
    loss, g = orc.softmax_ce(np.zeros((V, 8)), y)
    assert abs(loss - 2.0794415416798357) < 1e-15
    assert abs(g.sum()) < 1e-15 and abs(g[0, 0] - (1 / 8 - 1) / V) < 1e-16


def test_aggregate_against_scipy_on_cfg1_shape():
    w = inputs.WORKLOADS["cfg1"]
    src, dst = inputs.rmat_edges(w.V, w.E, w.graph_seed)
    src, dst = src.numpy(), dst.numpy()
    indptr, col = orc.csc_build(w.V, src, dst)
    X = inputs.features(w.V, 16).numpy().astype(np.float64)
    A = sp.coo_matrix((np.ones(len(src)), (dst, src)), shape=(w.V, w.V)).tocsr() + sp.identity(w.V, format="csr")
    D = np.asarray(A.sum(axis=1)).ravel()
    s = 1.0 / np.sqrt(D)
    ref = s[:, None] * (A @ (s[:, None] * X))
    np.testing.assert_allclose(orc.aggregate(indptr, col, X), ref, rtol=0, atol=1e-12)
    refT = s[:, None] * (A.T @ (s[:, None] * X))
    np.testing.assert_allclose(orc.aggregate_T(indptr, col, X), refT, rtol=0, atol=1e-12)
    np.testing.assert_allclose(orc.norm(indptr), s, rtol=0, atol=0)


def test_matmuls_against_numpy():
    rng = np.random.default_rng(1)
    A, B = rng.standard_normal((33, 7)), rng.standard_normal((7, 5))
    np.testing.assert_allclose(orc.matmul(A, B), A @ B, atol=1e-13)
    G = rng.standard_normal((33, 5))
    np.testing.assert_allclose(orc.matmul_tn(A, G), A.T @ G, atol=1e-13)
    np.testing.assert_allclose(orc.matmul_nt(G, B), G @ B.T, atol=1e-13)


@pytest.mark.parametrize("n,mode", [(1, 0), (4, 0), (7, 1), (64, 0)])
def test_partitioned_equals_unpartitioned(n, mode):
    V = 300
    src, dst = inputs.rmat_edges(V, 3000, seed=5)
    indptr, col = orc.csc_build(V, src.numpy(), dst.numpy())
    b = orc.chunk_bounds(indptr, n, mode)
    rng = np.random.default_rng(n)
    h = rng.standard_normal((V, 6))
    np.testing.assert_allclose(orc.layer_fwd_chunked(indptr, col, b, h), orc.aggregate(indptr, col, h), atol=1e-12)
    np.testing.assert_allclose(orc.layer_bwd_chunked(indptr, col, b, h), orc.aggregate_T(indptr, col, h), atol=1e-12)


def test_planted_mistakes_are_caught():
    """The pins above are sharp: a transposed operand or a dropped self-loop shows."""
    V = 30
    src, dst = _tiny_graph(V, 150, 0)
    indptr, col = orc.csc_build(V, src, dst)
    h = np.random.default_rng(0).standard_normal((V, 4))
    Ahat = _dense_norm_adj(V, src, dst)
    good = orc.aggregate(indptr, col, h)
    assert np.abs(good - Ahat @ h).max() < 1e-12
    assert np.abs(good - Ahat.T @ h).max() > 1e-3                 # transposed adjacency differs
    indptr_n, col_n = orc.csc_build(V, src, dst, add_self_loops=False)
    assert np.abs(orc.aggregate(indptr_n, col_n, h) - Ahat @ h).max() > 1e-3


def test_chunk_order_greedy_against_python_sets():
    # Alg. 4 phase 2 with one partition: max overlap with the chunk placed last, ties to the smallest id
    V = 60
    src, dst = _tiny_graph(V, 500, 11)
    indptr, col = orc.csc_build(V, src, dst)
    for n in (1, 2, 5, 9):
        b = orc.chunk_bounds(indptr, n)
        sets = [set(col[indptr[b[j]]:indptr[b[j + 1]]].tolist()) for j in range(n)]
        order = [0]
        left = list(range(1, n))
        while left:
            last = sets[order[-1]]
            k = max(left, key=lambda c: (len(sets[c] & last), -c))
            order.append(k)
            left.remove(k)
        assert orc.chunk_order(indptr, col, b).tolist() == order
    # a hand-made case: chunk 2 shares more with chunk 0 than chunk 1 does, so it is scheduled second
    src = np.array([0, 1, 2, 3, 7, 8, 0, 1, 2], dtype=np.int32)
    dst = np.array([10, 10, 10, 10, 11, 11, 12, 12, 12], dtype=np.int32)
    indptr, col = orc.csc_build(13, src, dst, add_self_loops=False)
    assert orc.chunk_order(indptr, col, np.array([0, 11, 12, 13])).tolist() == [0, 2, 1]


# ------------------------------------------------------------------ m partitions: volumes and Alg. 4

def _graph_of_sets(sets, V):
    """A graph in which subgraph c is one destination vertex (id V + c) whose in-neighbours are sets[c]; no self-loops.
    Returns CSC and the boundaries that make every such destination a subgraph of its own."""
    src = np.array([u for c, S in enumerate(sets) for u in sorted(S)], dtype=np.int32)
    dst = np.array([V + c for c, S in enumerate(sets) for _ in S], dtype=np.int32)
    indptr, col = orc.csc_build(V + len(sets), src, dst, add_self_loops=False)
    b = np.array([0] + [V + c + 1 for c in range(len(sets))], dtype=np.int64)     # subgraph 0 also holds the source-only ids
    return indptr, col, b


def _py_volumes(sets, m, n, layout):
    ori = sum(len(S) for S in sets)
    U = [set().union(*[sets[i * n + layout[i * n + j]] for i in range(m)]) for j in range(n)]
    p2p = sum(len(u) for u in U)
    ru = len(U[0]) + sum(len(U[j] - U[j - 1]) for j in range(1, n))
    return ori, p2p, ru


def _py_reorganize(sets, m, n):
    """Alg. 4 with Python sets; ties to the smallest index."""
    Gt = [[0] * n for _ in range(m)]
    U = []
    for j in range(n):
        Gt[0][j] = j
        U.append(set(sets[j]))
    for i in range(1, m):
        K = list(range(n))
        for j in range(n):
            k = max(K, key=lambda a: (len(sets[i * n + a] & U[j]), -a))
            Gt[i][j] = k
            U[j] |= sets[i * n + k]
            K.remove(k)
    at = [0]
    K = list(range(1, n))
    while K:
        k = max(K, key=lambda a: (len(U[a] & U[at[-1]]), -a))
        at.append(k)
        K.remove(k)
    return [Gt[i][at[j]] for i in range(m) for j in range(n)]


def test_volumes_mn_paper_example():
    # Sec. 5.1: 19 transfers without deduplication, 11 once a batch fetches each vertex once, 8 with reuse
    # between the two batches.  The text prints the two batch unions; the six subgraph sets below are one
    # choice with those unions and 19 members in all (three partitions, two batches).
    g, _ = _golden("dedup_transfer_counts.txt")
    sets = [{0, 1, 2, 3}, {2, 3, 4},        # partition 0: batch 0, batch 1
            {2, 3, 4, 7}, {4, 5, 6},        # partition 1
            {0, 4, 7}, {3, 6}]              # partition 2
    assert sorted(set().union(sets[0], sets[2], sets[4])) == g["union0"]
    assert sorted(set().union(sets[1], sets[3], sets[5])) == g["union1"]
    indptr, col, b = _graph_of_sets(sets, 8)
    assert orc.volumes_mn(indptr, col, b, 3, 2) == (g["transfers_before"][0], g["transfers_after_union"][0],
                                                    g["transfers_after_reuse"][0])


def test_reorganize_against_python_sets():
    rng = np.random.default_rng(5)
    for m, n in ((1, 1), (1, 5), (2, 2), (2, 6), (3, 4), (4, 5)):
        for trial in range(4):
            V = 40
            sets = [set(rng.choice(V, size=int(rng.integers(1, 15)), replace=False).tolist()) for _ in range(m * n)]
            indptr, col, b = _graph_of_sets(sets, V)
            lay = orc.reorganize(indptr, col, b, m, n)
            assert lay.tolist() == _py_reorganize(sets, m, n)
            for i in range(m):
                assert sorted(lay[i * n:(i + 1) * n].tolist()) == list(range(n))      # a permutation per partition
            ident = list(range(n)) * m
            for layout in (ident, lay.tolist()):
                vo, vp, vr = orc.volumes_mn(indptr, col, b, m, n, layout)
                assert (vo, vp, vr) == _py_volumes(sets, m, n, layout)
                assert vo >= vp >= vr >= len(set().union(*sets))
            if m == 1:      # one partition: the batch order is the chunk order, and no inter-GPU term
                assert lay.tolist() == orc.chunk_order(indptr, col, b).tolist()
                vo, vp, vr = orc.volumes_mn(indptr, col, b, 1, n)
                assert vo == vp and (vo, vr) == orc.volumes(indptr, col, b)


def test_reorganize_recovers_a_planted_matching():
    # every partition holds the same n disjoint neighbour sets in its own shuffled order: phase 1 must put equal
    # sets into the same batch, after which a batch fetches |S_j| rows instead of m |S_j|
    rng = np.random.default_rng(9)
    m, n, per = 4, 6, 5
    S = [set(range(j * per, (j + 1) * per)) for j in range(n)]
    perms = [list(range(n))] + [rng.permutation(n).tolist() for _ in range(m - 1)]
    sets = [S[perms[i][k]] for i in range(m) for k in range(n)]
    indptr, col, b = _graph_of_sets(sets, n * per)
    lay = orc.reorganize(indptr, col, b, m, n)
    for i in range(m):
        for j in range(n):
            assert perms[i][lay[i * n + j]] == j       # batch j holds S_j of every partition (phase 2: all ties)
    before = orc.volumes_mn(indptr, col, b, m, n)
    after = orc.volumes_mn(indptr, col, b, m, n, lay)
    assert after == (m * n * per, n * per, n * per) and before[0] == after[0] and before[1] > after[1]


def test_reorganize_hand_made_case():
    # two partitions, three subgraphs each.  Phase 1: batch 0 = {0,1,2} takes {1,2,3} (2 common) over {0,9} (1) and
    # {7,8}; batch 1 = {4,5} takes {0,9} (tie at 0 common: smaller index) and batch 2 = {7,8,9} gets {7,8}.
    # Phase 2: unions {0,1,2,3}, {0,4,5,9}, {7,8,9}: after batch 0 comes batch 1 (1 common against 0), then batch 2.
    sets = [{0, 1, 2}, {4, 5}, {7, 8, 9},
            {0, 9}, {7, 8}, {1, 2, 3}]
    indptr, col, b = _graph_of_sets(sets, 10)
    assert orc.reorganize(indptr, col, b, 2, 3).tolist() == [0, 1, 2, 2, 0, 1]
    assert orc.volumes_mn(indptr, col, b, 2, 3) == (15, 14, 12)      # unions {0,1,2,9}, {4,5,7,8}, {1,2,3,7,8,9}: 4 + 4 + 4 loaded
    assert orc.volumes_mn(indptr, col, b, 2, 3, [0, 1, 2, 2, 0, 1]) == (15, 11, 9)


# ------------------------------------------------------------------ row-buffer schedules

def _tiny_chunks(rng, V, n, per):
    """A graph whose chunk j (destination j) has the given random source set; returns CSC, bounds."""
    src, dst = [], []
    for j in range(n):
        for u in rng.choice(V, size=per, replace=False):
            src.append(u)
            dst.append(j)
    src, dst = np.array(src, np.int32), np.array(dst, np.int32)
    indptr, col = orc.csc_build(max(V, n), src, dst, add_self_loops=False)
    b = np.array(list(range(n)) + [max(V, n)], dtype=np.int64)      # chunk j = destination j (the last one takes the rest)
    return indptr, col, b


def test_cache_schedule_adjacent_policy_is_the_reuse_split():
    rng = np.random.default_rng(0)
    indptr, col, b = _tiny_chunks(rng, 30, 6, 9)
    order = np.arange(6, dtype=np.int32)
    sch = orc.cache_schedule(indptr, col, b, order, 9, 0)
    N = [np.unique(col[indptr[b[j]]:indptr[b[j + 1]]]) for j in range(6)]
    prev = np.zeros(0, np.int32)
    for j in range(6):
        R, Ld = orc.reuse_split(prev, N[j])
        assert np.array_equal(sch[j]["reuse"], R) and np.array_equal(sch[j]["load"], Ld)
        nxt = N[j + 1] if j + 1 < 6 else np.zeros(0, np.int32)
        assert np.array_equal(sch[j]["leave"], np.setdiff1d(N[j], nxt))
        prev = N[j]


def _min_loads_brute_force(N, C):
    """Fewest row loads over every way of releasing rows (depth-first over release choices)."""
    import itertools
    n = len(N)
    best = [10 ** 9]

    def go(j, resident, loads):
        if loads >= best[0]:
            return
        if j == n:
            best[0] = loads
            return
        need = set(N[j])
        loads += len(need - resident)
        uni = resident | need
        over = len(uni) - C
        if over <= 0:
            go(j + 1, uni, loads)
            return
        cand = sorted(resident - need)
        for out in itertools.combinations(cand, over):
            go(j + 1, uni - set(out), loads)

    go(0, set(), 0)
    return best[0]


def test_cache_schedule_farthest_next_use_loads_the_fewest_rows():
    rng = np.random.default_rng(1)
    for trial in range(12):
        V, n, per = 9, 6, 4
        indptr, col, b = _tiny_chunks(rng, V, n, per)
        N = [sorted(set(col[indptr[b[j]]:indptr[b[j + 1]]].tolist())) for j in range(n)]
        for C in (4, 5, 6):
            sch = orc.cache_schedule(indptr, col, b, np.arange(n, dtype=np.int32), C, 1)
            loads = sum(len(s["load"]) for s in sch)
            assert loads == _min_loads_brute_force(N, C), (trial, C)
            # never more rows than the buffer holds; every needed row is there; released rows really leave
            resident = set()
            for j, s in enumerate(sch):
                assert set(s["reuse"]) <= resident and not (set(s["load"]) & resident)
                assert sorted(set(s["reuse"]) | set(s["load"])) == N[j]
                resident |= set(s["load"])
                assert len(resident) <= C
                assert set(s["leave"]) <= resident
                if j + 1 < n:
                    assert not (set(s["leave"]) & set(N[j + 1]))
                resident -= set(s["leave"])
                # nothing stays beyond its last use
                later = set().union(*N[j + 1:]) if j + 1 < n else set()
                assert resident <= later
            assert not resident
            # the adjacent policy never loads fewer
            adj = orc.cache_schedule(indptr, col, b, np.arange(n, dtype=np.int32), C, 0)
            assert loads <= sum(len(s["load"]) for s in adj)


def test_cache_schedule_large_buffer_loads_every_row_once_and_tie_break():
    rng = np.random.default_rng(2)
    indptr, col, b = _tiny_chunks(rng, 20, 5, 6)
    N = [np.unique(col[indptr[b[j]]:indptr[b[j + 1]]]) for j in range(5)]
    union = np.unique(np.concatenate(N))
    sch = orc.cache_schedule(indptr, col, b, np.arange(5, dtype=np.int32), len(union), 1)
    assert sum(len(s["load"]) for s in sch) == len(union)
    last = {int(u): max(j for j in range(5) if u in N[j]) for u in union}        # room for all: a row leaves after its last use
    for j in range(5):
        assert sch[j]["leave"].tolist() == sorted(u for u, k in last.items() if k == j)
    # hand-made: chunks {0,1,2}, {3,4,5}, {0,1,2} with C = 4: rows 0,1,2 all have next use 2; one may stay: the
    # two smallest ids go first among equals; 3,4,5 are never needed again and leave after their chunk
    src = np.array([0, 1, 2, 3, 4, 5, 0, 1, 2], np.int32)
    dst = np.array([0, 0, 0, 1, 1, 1, 2, 2, 2], np.int32)
    indptr, col = orc.csc_build(6, src, dst, add_self_loops=False)
    b = np.array([0, 1, 2, 6], dtype=np.int64)
    sch = orc.cache_schedule(indptr, col, b, np.arange(3, dtype=np.int32), 4, 1)
    assert sch[0]["leave"].tolist() == [0, 1] and sch[1]["leave"].tolist() == [3, 4, 5] and sch[2]["reuse"].tolist() == [2]
    assert sch[2]["load"].tolist() == [0, 1] and sch[2]["leave"].tolist() == [0, 1, 2]

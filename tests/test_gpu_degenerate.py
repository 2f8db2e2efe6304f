"""Degenerate graphs through the float paths: no self-loops (vertices without in-edges, D_v = 0),
isolated vertices, more chunks than vertices (empty chunks), a graph without any edge, one vertex.
GCN layer and epoch in both stage orders, and the GAT layer, against the oracle."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2311_14898_amd import binding as B
from tests.util import assert_close, assert_close_grad

pytestmark = pytest.mark.gpu
DEV = B.HT_LOC_DEVICE


@pytest.fixture(scope="module")
def ctx():
    c = B.ht_ctx_create(0)
    yield c
    B.ht_ctx_destroy(c)


def graphs():
    rng = np.random.default_rng(0)
    V = 70
    src = rng.integers(0, 40, 300).astype(np.int32)          # vertices 40..69 never a source
    dst = rng.integers(10, 50, 300).astype(np.int32)         # vertices 0..9 and 50..69 without in-edges
    yield "no-self-loops", V, src, dst, 3, False
    yield "more-chunks-than-vertices", 5, np.array([0, 1, 2, 2], np.int32), np.array([1, 2, 3, 3], np.int32), 9, True
    yield "no-edges", 6, np.zeros(0, np.int32), np.zeros(0, np.int32), 2, True
    yield "no-edges-no-loops", 6, np.zeros(0, np.int32), np.zeros(0, np.int32), 2, False
    yield "one-vertex", 1, np.zeros(0, np.int32), np.zeros(0, np.int32), 1, True


def _mat(x, loc=DEV):
    return B.to_matrix(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)), loc)


@pytest.mark.parametrize("case", list(graphs()), ids=lambda c: c[0])
def test_gcn_layer_and_epoch(ctx, case):
    _, V, src, dst, n, loops = case
    g = B.ht_partition(ctx, V, torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda(), n, add_self_loops=loops)
    indptr, col = orc.csc_build(V, src, dst, add_self_loops=loops)
    rng = np.random.default_rng(1)
    dims = [12, 9, 4]
    X = rng.standard_normal((V, dims[0])).astype(np.float32)
    Ws = [(rng.standard_normal((dims[l], dims[l + 1])) / 3).astype(np.float32) for l in range(2)]
    y = rng.integers(0, dims[-1], V).astype(np.int32)
    ref = orc.gcn_epoch(indptr, col, dims, X, Ws, y, lr=0.5)
    try:
        for loc in (DEV, B.HT_LOC_HOST_PINNED):
            for order in (B.HT_ORDER_AGG_FIRST, B.HT_ORDER_UPDATE_FIRST):
                Wd = [torch.from_numpy(w).cuda() for w in Ws]
                res = dict(res_h=B.HT_RES_HOST, res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST) if loc != DEV else {}
                loss, _ = B.ht_epoch(ctx, g, dims, Wd, 0.5, _mat(X, loc), torch.from_numpy(y).cuda(), order=order, **res)
                assert abs(loss - ref["loss"]) <= 1e-4 * abs(ref["loss"])
                for l in range(2):
                    # rows without in-edges are exactly zero; ReLU ties at 0 do not matter for zero rows
                    assert_close(B.ht_epoch_buffer(ctx, B.HT_BUF_H, l + 1).numpy(), ref["h"][l], f"h^{l + 1}")
                    assert_close_grad(Wd[l].cpu().numpy(), ref["W_new"][l], f"W^{l}")
    finally:
        B.ht_graph_destroy(g)


@pytest.mark.parametrize("case", list(graphs()), ids=lambda c: c[0])
def test_gat_layer(ctx, case):
    _, V, src, dst, n, loops = case
    g = B.ht_partition(ctx, V, torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda(), n, add_self_loops=loops)
    indptr, col = orc.csc_build(V, src, dst, add_self_loops=loops)
    rng = np.random.default_rng(2)
    d_in, d_out = 10, 6
    H = rng.standard_normal((V, d_in)).astype(np.float32)
    W = (rng.standard_normal((d_in, d_out)) / 3).astype(np.float32)
    a_dst, a_src = rng.standard_normal(d_out).astype(np.float32), rng.standard_normal(d_out).astype(np.float32)
    dh = rng.standard_normal((V, d_out)).astype(np.float32)
    f = orc.gat_layer_fwd(indptr, col, H, W, a_dst, a_src, relu=False)
    b = orc.gat_layer_bwd(indptr, col, H, W, a_dst, a_src, f, dh, relu=False)
    try:
        Hd, Wd = _mat(H), torch.from_numpy(W).cuda()
        ad, as_ = torch.from_numpy(a_dst).cuda(), torch.from_numpy(a_src).cuda()
        H_out = B.alloc_matrix(V, d_out, DEV, zero=False)
        B.ht_gat_layer_fwd(ctx, g, d_in, d_out, B.HT_ACT_NONE, Hd, Wd, ad, as_, H_out)
        assert_close(H_out.cpu().numpy()[:, :d_out], f["h"], "h_out")       # vertices without in-edges: zero rows
        dW = torch.empty(d_in, d_out, device="cuda")
        dad, das = torch.empty(d_out, device="cuda"), torch.empty(d_out, device="cuda")
        dH_in = B.alloc_matrix(V, d_in, DEV)
        B.ht_gat_layer_bwd(ctx, g, d_in, d_out, B.HT_ACT_NONE, Hd, Wd, ad, as_, H_out, _mat(dh), dW, dad, das, dH_in=dH_in)
        assert_close_grad(dW.cpu().numpy(), b["dW"], "dW")
        # the two halves of a^l as one vector: on a graph whose scores all have one sign the destination
        # half's gradient is exactly 0 (the softmax does not see p_v), and a relative error needs a scale
        assert_close_grad(np.concatenate([dad.cpu().numpy(), das.cpu().numpy()]), np.concatenate([b["da_dst"], b["da_src"]]), "da")
        assert_close_grad(dH_in.cpu().numpy()[:, :d_in], b["dH"], "dH_in")
    finally:
        B.ht_graph_destroy(g)

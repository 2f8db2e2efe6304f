"""ht_gat_layer_fwd / ht_gat_layer_bwd (Eq. 3, one head) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2311_14898_amd import binding as B
from paper_2311_14898_amd import inputs
from tests.util import assert_close, assert_close_grad, hub_graph

pytestmark = pytest.mark.gpu
DEV = B.HT_LOC_DEVICE


@pytest.fixture(scope="module")
def ctx():
    c = B.ht_ctx_create(0)
    yield c
    B.ht_ctx_destroy(c)


class Case:
    def __init__(self, ctx, V, src, dst, n):
        self.V, self.src, self.dst = V, src, dst
        self.g = B.ht_partition(ctx, V, src.cuda(), dst.cuda(), n)
        self.indptr, self.col = orc.csc_build(V, src.numpy(), dst.numpy(), True)


@pytest.fixture(scope="module")
def cases(ctx):
    out = {}
    V = 9_000
    src, dst = inputs.rmat_edges(V, 150_000, seed=4)
    out["rmat"] = Case(ctx, V, src, dst, 5)                      # few repeated pairs: canonical arrays
    k = torch.arange(0, src.numel(), 3)
    out["multi"] = Case(ctx, V, torch.cat([src, src[k], src[k]]), torch.cat([dst, dst[k], dst[k]]), 4)   # merged entries
    Vh = 15_013
    s, d = hub_graph(Vh, 120_000, hub_in=2500, hub_out=2000, seed=2)
    out["hub"] = Case(ctx, Vh, s, d, 3)                          # rows and sources cut into several items
    yield out
    for c in out.values():
        B.ht_graph_destroy(c.g)


def _mat(x):
    return B.to_matrix(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)), DEV)


def _run(ctx, case, d_in, d_out, relu, seed, want_dhin=True, slope=0.2, host=()):
    """host: which of the layer's tensors live in pinned host memory ("H_in", "H_out", "dH_out", "dH_in")."""
    def loc(name):
        return B.HT_LOC_HOST_PINNED if name in host else DEV

    def mat(x, name):
        return B.to_matrix(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)), loc(name))

    rng = np.random.default_rng(seed)
    V = case.V
    H = rng.standard_normal((V, d_in)).astype(np.float32)
    W = (rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)).astype(np.float32)
    a_dst = (rng.standard_normal(d_out) / np.sqrt(d_out)).astype(np.float32)
    a_src = (rng.standard_normal(d_out) / np.sqrt(d_out)).astype(np.float32)
    dh = rng.standard_normal((V, d_out)).astype(np.float32)
    act = B.HT_ACT_RELU if relu else B.HT_ACT_NONE
    f = orc.gat_layer_fwd(case.indptr, case.col, H, W, a_dst, a_src, slope=slope, relu=relu)
    Hd, Wd = mat(H, "H_in"), torch.from_numpy(W).cuda()
    ad, as_ = torch.from_numpy(a_dst).cuda(), torch.from_numpy(a_src).cuda()
    H_out = B.alloc_matrix(V, d_out, loc("H_out"), zero=False)
    B.ht_gat_layer_fwd(ctx, case.g, d_in, d_out, act, Hd, Wd, ad, as_, H_out, slope=slope)
    assert_close(H_out.cpu().numpy()[:, :d_out], f["h"], "h_out")
    # backward from the oracle's own forward result, so both sides mask the same elements
    b = orc.gat_layer_bwd(case.indptr, case.col, H, W, a_dst, a_src, f, dh, slope=slope, relu=relu, want_dH=want_dhin)
    dW = torch.empty(d_in, d_out, device="cuda")
    dad, das = torch.empty(d_out, device="cuda"), torch.empty(d_out, device="cuda")
    dH_in = B.alloc_matrix(V, d_in, loc("dH_in")) if want_dhin else None
    if want_dhin:       # the input gradient is added to what the tensor holds
        base = np.random.default_rng(seed + 1).standard_normal((V, d_in)).astype(np.float32) if host else None
        if base is not None:
            dH_in[:, :d_in] = torch.from_numpy(base)
    B.ht_gat_layer_bwd(ctx, case.g, d_in, d_out, act, Hd, Wd, ad, as_, mat(f["h"], "H_out"), mat(dh, "dH_out"), dW, dad, das,
                       dH_in=dH_in, slope=slope)
    assert_close_grad(dW.cpu().numpy(), b["dW"], "dW")
    assert_close_grad(dad.cpu().numpy(), b["da_dst"], "da_dst")
    assert_close_grad(das.cpu().numpy(), b["da_src"], "da_src")
    if want_dhin:
        got = dH_in.cpu().numpy()[:, :d_in].astype(np.float64)
        assert_close_grad(got - (base if host else 0.0), b["dH"], "dH_in")
    return H_out, dW


@pytest.mark.parametrize("d_in,d_out", [(16, 8), (64, 32), (100, 41), (30, 100), (130, 256), (48, 300), (24, 520)])
def test_gat_widths(ctx, cases, d_in, d_out):
    _run(ctx, cases["rmat"], d_in, d_out, True, seed=d_in + d_out)


@pytest.mark.parametrize("name", ["multi", "hub"])
@pytest.mark.parametrize("relu", [True, False])
def test_gat_multigraph_and_hubs(ctx, cases, name, relu):
    _run(ctx, cases[name], 72, 40, relu, seed=7)


def test_gat_no_input_gradient_and_other_slope(ctx, cases):
    _run(ctx, cases["multi"], 32, 64, True, seed=9, want_dhin=False, slope=0.05)


def test_gat_partition_options(ctx):
    # the layer does not care how the graph was chunked or scheduled
    V = 7_001
    src, dst = inputs.rmat_edges(V, 90_000, seed=11)
    for kw in (dict(reorder_chunks=True), dict(balance_mode=1, cache_rows=-1), dict(add_self_loops=False)):
        c = Case.__new__(Case)
        c.V = V
        c.g = B.ht_partition(ctx, V, src.cuda(), dst.cuda(), 7, **kw)
        c.indptr, c.col = orc.csc_build(V, src.numpy(), dst.numpy(), kw.get("add_self_loops", True))
        try:
            _run(ctx, c, 24, 36, True, seed=13)
        finally:
            B.ht_graph_destroy(c.g)


def test_gat_zero_attention_is_the_neighbour_mean(ctx, cases):
    c = cases["rmat"]
    rng = np.random.default_rng(3)
    H = rng.standard_normal((c.V, 24)).astype(np.float32)
    W = np.eye(24, dtype=np.float32)
    zero = torch.zeros(24, device="cuda")
    H_out = B.alloc_matrix(c.V, 24, DEV, zero=False)
    B.ht_gat_layer_fwd(ctx, c.g, 24, 24, B.HT_ACT_NONE, _mat(H), torch.from_numpy(W).cuda(), zero, zero, H_out)
    deg = np.diff(c.indptr)
    ref = np.add.reduceat(H.astype(np.float64)[c.col], c.indptr[:-1], axis=0) / deg[:, None]
    assert_close(H_out.cpu().numpy()[:, :24], ref, "mean")


ALL_HOST = ("H_in", "H_out", "dH_out", "dH_in")


@pytest.mark.parametrize("host", [("H_in",), ("H_out", "dH_out"), ("dH_in",), ALL_HOST], ids=lambda h: "+".join(h))
def test_gat_host_resident_tensors(ctx, cases, host):
    _run(ctx, cases["rmat"], 100, 41, True, seed=21, host=host)
    _run(ctx, cases["hub"], 30, 100, False, seed=22, host=host)


def test_gat_host_resident_small_blocks(cases):
    """Staged row blocks much smaller than the tensors: several rounds through both buffers of each staging pair."""
    import os
    os.environ["HT_LINK_BLOCK_ROWS"] = "700"
    try:
        c2 = B.ht_ctx_create(0)
    finally:
        del os.environ["HT_LINK_BLOCK_ROWS"]
    try:
        case = cases["multi"]
        twin = Case(c2, case.V, case.src, case.dst, 5)
        try:
            assert case.V > 4 * 700
            _run(c2, twin, 64, 32, True, seed=23, host=ALL_HOST)
            _run(c2, twin, 40, 130, True, seed=24, host=("H_in", "dH_in"))
        finally:
            B.ht_graph_destroy(twin.g)
    finally:
        B.ht_ctx_destroy(c2)


def test_gat_deterministic(ctx, cases):
    a = _run(ctx, cases["hub"], 40, 48, True, seed=5)
    b = _run(ctx, cases["hub"], 40, 48, True, seed=5)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_gat_epoch(ctx, cases):
    """Alg. 1 with two GAT layers against the oracle's layer functions composed in the same order."""
    c = cases["multi"]
    V, dims, lr = c.V, [40, 24, 7], 20.0         # a large step, so that the updated parameters expose the gradients
    rng = np.random.default_rng(12)
    X = rng.standard_normal((V, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[-1], V).astype(np.int32)
    y[rng.random(V) < 0.3] = -1
    Ws = [(rng.standard_normal((dims[l], dims[l + 1])) / np.sqrt(dims[l])).astype(np.float32) for l in range(2)]
    ad = [(rng.standard_normal(dims[l + 1]) / np.sqrt(dims[l + 1])).astype(np.float32) for l in range(2)]
    as_ = [(rng.standard_normal(dims[l + 1]) / np.sqrt(dims[l + 1])).astype(np.float32) for l in range(2)]
    # oracle
    f0 = orc.gat_layer_fwd(c.indptr, c.col, X, Ws[0], ad[0], as_[0], relu=True)
    f1 = orc.gat_layer_fwd(c.indptr, c.col, f0["h"], Ws[1], ad[1], as_[1], relu=False)
    assert np.abs(f0["z"]).min() > 1e-7        # same ReLU decisions on both sides
    loss_ref, g2 = orc.softmax_ce(f1["h"], y)
    b1 = orc.gat_layer_bwd(c.indptr, c.col, f0["h"], Ws[1], ad[1], as_[1], f1, g2, relu=False)
    b0 = orc.gat_layer_bwd(c.indptr, c.col, X, Ws[0], ad[0], as_[0], f0, b1["dH"], relu=True, want_dH=False)
    # device
    Wd = [torch.from_numpy(w).cuda() for w in Ws]
    add = [torch.from_numpy(a).cuda() for a in ad]
    asd = [torch.from_numpy(a).cuda() for a in as_]
    loss, st = B.ht_gat_epoch(ctx, c.g, dims, Wd, add, asd, lr, _mat(X), torch.from_numpy(y).cuda(), want_stats=True)
    assert abs(loss - loss_ref) <= 1e-4 * abs(loss_ref)
    for l, b in ((0, b0), (1, b1)):
        assert_close_grad(Wd[l].cpu().numpy(), Ws[l].astype(np.float64) - lr * b["dW"], f"W^{l} after the step")
        assert_close_grad(add[l].cpu().numpy(), ad[l].astype(np.float64) - lr * b["da_dst"], f"a_dst^{l} after the step")
        assert_close_grad(asd[l].cpu().numpy(), as_[l].astype(np.float64) - lr * b["da_src"], f"a_src^{l} after the step")
        assert np.abs(lr * b["dW"]).max() > 0.05 * np.abs(Ws[l]).max()      # the step is visible at the tolerance
    assert st.edges == len(c.col) * (2 + 4)     # 2 forward aggregations, 2 x 2 backward passes
    # small steps from the same start: the loss goes down
    Wd = [torch.from_numpy(w).cuda() for w in Ws]
    add = [torch.from_numpy(a).cuda() for a in ad]
    asd = [torch.from_numpy(a).cuda() for a in as_]
    losses = [B.ht_gat_epoch(ctx, c.g, dims, Wd, add, asd, 0.05, _mat(X), torch.from_numpy(y).cuda())[0] for _ in range(3)]
    assert losses[0] == loss and losses[2] < losses[1] < losses[0]
    # the same epoch with X, h^1 and its gradient in pinned host memory
    Wd = [torch.from_numpy(w).cuda() for w in Ws]
    add = [torch.from_numpy(a).cuda() for a in ad]
    asd = [torch.from_numpy(a).cuda() for a in as_]
    Xh = B.to_matrix(torch.from_numpy(X), B.HT_LOC_HOST_PINNED)
    loss_h, st = B.ht_gat_epoch(ctx, c.g, dims, Wd, add, asd, lr, Xh, torch.from_numpy(y).cuda(), want_stats=True,
                                res_h=B.HT_RES_HOST)
    assert abs(loss_h - loss_ref) <= 1e-4 * abs(loss_ref)
    for l, b in ((0, b0), (1, b1)):
        assert_close_grad(Wd[l].cpu().numpy(), Ws[l].astype(np.float64) - lr * b["dW"], f"W^{l} after the step (host)")
        assert_close_grad(add[l].cpu().numpy(), ad[l].astype(np.float64) - lr * b["da_dst"], f"a_dst^{l} after the step (host)")
    # link traffic, all in contiguous row ranges: X three times (t forward, t again and dW backward); h^1 out once and in
    # four times (t and dW of layer 1, forward and backward; as H_out of layer 0's backward); grad h^1 out and in once
    ld0, ld1 = B.pad_ld(dims[0], B.HT_LOC_HOST_PINNED), B.pad_ld(dims[1], B.HT_LOC_HOST_PINNED)
    assert st.bytes_h2d == 4 * V * (3 * ld0 + 5 * ld1) and st.bytes_d2h == 4 * V * 2 * ld1


def test_gat_errors(ctx, cases):
    c = cases["rmat"]
    W = torch.zeros(16, 8, device="cuda")
    v = torch.zeros(8, device="cuda")
    with pytest.raises(B.HongtuError):      # slope out of range
        B.ht_gat_layer_fwd(ctx, c.g, 16, 8, B.HT_ACT_NONE, B.alloc_matrix(c.V, 16, DEV), W, v, v,
                           B.alloc_matrix(c.V, 8, DEV), slope=2.0)
    with pytest.raises(B.HongtuError):      # wrong row count
        B.ht_gat_layer_fwd(ctx, c.g, 16, 8, B.HT_ACT_NONE, B.alloc_matrix(c.V - 1, 16, DEV), W, v, v,
                           B.alloc_matrix(c.V, 8, DEV))

"""The fused aggregate + update kernel (HT_FUSE_UPDATE=1: layers that keep no aggregate build a^l of 32 destination rows in
LDS and transform it there on the matrix cores, Sec. 4.2's recomputation case): the layer forward against the oracle at
several width pairs (ragged K and N, more than one LDS vector per lane, a hub row), bit-reproducible, and whole epochs
in the recomputation mode against the oracle's epoch."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2311_14898_amd import binding as B
from paper_2311_14898_amd import inputs
from tests.util import assert_close, assert_close_grad, hub_graph

pytestmark = pytest.mark.gpu


@pytest.fixture()
def fused_ctx(monkeypatch):
    monkeypatch.setenv("HT_FUSE_UPDATE", "1")
    ctx = B.ht_ctx_create(0)
    yield ctx
    B.ht_ctx_destroy(ctx)
    torch.cuda.synchronize()


@pytest.mark.parametrize("d_in,d_out,act", [(64, 32, B.HT_ACT_RELU), (602, 256, B.HT_ACT_RELU), (100, 47, B.HT_ACT_NONE),
                                           (257, 130, B.HT_ACT_RELU), (1021, 8, B.HT_ACT_NONE), (7, 300, B.HT_ACT_RELU)])
def test_fused_layer_forward(fused_ctx, d_in, d_out, act):
    ctx = fused_ctx
    V = 3000
    src, dst = hub_graph(V, 40_000, 5000, 300, seed=d_in)         # a destination with 5000 in-edges; repeated pairs
    indptr, col = orc.csc_build(V, src.numpy(), dst.numpy())
    rng = np.random.default_rng(d_in + d_out)
    H = rng.standard_normal((V, d_in)).astype(np.float32)
    W = (rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)).astype(np.float32)
    z_ref = orc.matmul(orc.aggregate(indptr, col, H), W)
    h_ref = np.maximum(z_ref, 0.0) if act == B.HT_ACT_RELU else z_ref
    g = B.ht_partition(ctx, V, src.cuda(), dst.cuda(), 5)
    try:
        Hd, Wd = B.to_matrix(torch.from_numpy(H)), torch.from_numpy(W).cuda()
        outs = []
        for _ in range(2):
            H_out = B.alloc_matrix(V, d_out)
            st = B.ht_layer_fwd(ctx, g, d_in, d_out, act, Hd, Wd, H_out, want_stats=True)      # no A_ckpt: nothing keeps a^l
            assert st.n_spmm_fwd == 5 and st.edges == len(col)
            outs.append(H_out[:, :d_out].cpu())
        assert_close(outs[0].numpy(), h_ref, f"h' {d_in}->{d_out}")
        assert torch.equal(outs[0], outs[1])
        # with a checkpoint asked for the separate kernels run: the same values to the tolerance
        H2, A2 = B.alloc_matrix(V, d_out), B.alloc_matrix(V, d_in)
        B.ht_layer_fwd(ctx, g, d_in, d_out, act, Hd, Wd, H2, A_ckpt=A2)
        assert_close(H2[:, :d_out].cpu().numpy(), h_ref, "separate kernels")
    finally:
        B.ht_graph_destroy(g)


def test_fused_epoch_in_recomputation_mode(fused_ctx):
    ctx = fused_ctx
    w = inputs.Workload("fused", 800, 24_000, [100, 130, 41], 5, graph_seed=39, lr=0.05)   # a seed whose pre-activations are clear of 0
    src, dst, X, y, Ws = inputs.make_inputs(w)
    indptr, col = orc.csc_build(w.V, src.numpy(), dst.numpy())
    ref = orc.gcn_epoch(indptr, col, w.dims, X.numpy(), [x.numpy() for x in Ws], y.numpy(), lr=w.lr)
    for l in range(w.n_layers - 1):
        z = np.abs(ref["z"][l])
        assert z.min() > 2e-6 * z.max(), "pick another graph seed: a pre-activation is within fp32 rounding of zero"
    g = B.ht_partition(ctx, w.V, src.cuda(), dst.cuda(), w.n_chunks)
    try:
        Wd = [x.clone().cuda() for x in Ws]
        loss, st = B.ht_epoch(ctx, g, w.dims, Wd, w.lr, B.to_matrix(X), y.cuda(), inter=B.HT_INTER_RECOMPUTE, want_stats=True)
        assert st.plan_inter == B.HT_INTER_RECOMPUTE
        assert abs(loss - ref["loss"]) <= 1e-4 * abs(ref["loss"])
        for l in range(w.n_layers):
            assert_close(B.ht_epoch_buffer(ctx, B.HT_BUF_H, l + 1).numpy(), ref["h"][l], f"h^{l + 1}")
            assert_close_grad(B.ht_epoch_buffer(ctx, B.HT_BUF_DW, l).numpy(), ref["gW"][l], f"grad W^{l}")
            assert_close_grad(Wd[l].cpu().numpy(), ref["W_new"][l], f"W^{l}")
    finally:
        B.ht_graph_destroy(g)

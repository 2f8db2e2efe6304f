"""The library's A/B switches (environment variables read when a context or a graph is created) each select a
different kernel variant, launch shape or copy path for the same mathematics: every setting must give the oracle's
epoch, in HBM and with host-resident vertex data."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2311_14898_amd import binding as B
from paper_2311_14898_amd import inputs
from tests.util import assert_close, assert_close_grad

pytestmark = pytest.mark.gpu

SETTINGS = [
    {"HT_AGG_VARIANT": "1"},                                 # one wave per item over the full row
    {"HT_SLABS_FWD": "1", "HT_SLABS_BWD": "1"},
    {"HT_SLABS_FWD": "2", "HT_SLABS_BWD": "8"},
    {"HT_SLABS_FWD": "8", "HT_SLABS_BWD": "2"},
    {"HT_AGG_UNROLL": "8"},
    {"HT_AGG_UNIFORM": "0"},
    {"HT_SLAB_ALIGN": "0"},
    {"HT_AGG_PHASES": "2"},
    {"HT_XCD_CONTIG": "1"},
    {"HT_MERGE_DUPS": "0"},
    {"HT_ITEM_ORDER": "0"},
    {"HT_SEG_FWD": "64", "HT_SEG_BWD": "256"},
    {"HT_LINK_MEMCPY": "1"},
    {"HT_LINK_MEMCPY": "1", "HT_NO_LINK_FENCE": "1"},
    {"HT_LINK_MEMCPY": "2"},
    {"HT_LINK_MEMCPY": "3"},
    {"HT_NO_LINK_FENCE": "1"},
    {"HT_LINK_BLOCKS": "16", "HT_GATHER_BLOCKS": "512"},
]


@pytest.fixture(scope="module")
def case():
    # widths that give the slab kernels several slabs (130 -> 33 vectors) and a ragged last one; duplicate edges
    # (the generator keeps them) so that merging has something to merge
    w = inputs.Workload("switches", 800, 24_000, [100, 130, 41], 5, graph_seed=39, lr=0.05)
    src, dst, X, y, Ws = inputs.make_inputs(w)
    indptr, col = orc.csc_build(w.V, src.numpy(), dst.numpy())
    ref = orc.gcn_epoch(indptr, col, w.dims, X.numpy(), [x.numpy() for x in Ws], y.numpy(), lr=w.lr)
    z = np.abs(ref["z"][0])
    assert z.min() > 2e-6 * z.max(), "pick another graph seed: a pre-activation is within fp32 rounding of zero"
    return w, src, dst, X, y, Ws, ref


@pytest.mark.parametrize("env", SETTINGS, ids=lambda e: ",".join(f"{k[3:]}={v}" for k, v in e.items()))
def test_switch(case, env, monkeypatch):
    w, src, dst, X, y, Ws, ref = case
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    ctx = B.ht_ctx_create(0)            # the context and the graph read the switches when they are made
    try:
        for host in (False, True):
            g = B.ht_partition(ctx, w.V, src.cuda(), dst.cuda(), w.n_chunks)
            try:
                Wd = [x.clone().cuda() for x in Ws]
                res = B.HT_RES_HOST if host else B.HT_RES_AUTO
                Xd = B.to_matrix(X, B.HT_LOC_HOST_PINNED if host else B.HT_LOC_DEVICE)
                loss, _ = B.ht_epoch(ctx, g, w.dims, Wd, w.lr, Xd, y.cuda(), res_h=res, res_a=res, res_g=res)
                assert abs(loss - ref["loss"]) <= 1e-4 * abs(ref["loss"])
                for l in range(w.n_layers):
                    assert_close(B.ht_epoch_buffer(ctx, B.HT_BUF_H, l + 1).numpy(), ref["h"][l], f"{env} host={host} h^{l + 1}")
                    assert_close_grad(B.ht_epoch_buffer(ctx, B.HT_BUF_GH, l + 1).numpy(), ref["gh"][l], f"{env} host={host} grad h^{l + 1}")
                    assert_close_grad(Wd[l].cpu().numpy(), ref["W_new"][l], f"{env} host={host} W^{l}")
            finally:
                B.ht_graph_destroy(g)
    finally:
        B.ht_ctx_destroy(ctx)
        torch.cuda.synchronize()

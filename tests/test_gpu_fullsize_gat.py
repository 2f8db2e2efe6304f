"""GAT layer parity at the benchmark's full size (config 2's graph and first layer: 232,965
vertices, 114.6 M edges, 602 -> 256, 8 chunks, all in HBM), in the launch configuration
`bench.py --model gat` runs.  The oracle computes the whole layer forward and backward in fp64
(about half a minute on the machine's host cores), so every output tensor is compared in full."""
import time

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2311_14898_amd import binding as B
from paper_2311_14898_amd import inputs
from tests import gat_ties
from tests.util import GRAD_ROW_FLOOR, assert_close, assert_close_grad, assert_in_interval

pytestmark = pytest.mark.gpu


def test_gat_layer_full_size():
    t0 = time.perf_counter()
    note = lambda m: print(f"[{time.perf_counter() - t0:6.1f}s] {m}", flush=True)
    w = inputs.WORKLOADS["cfg2"]
    V, d_in, d_out = w.V, w.dims[0], w.dims[1]
    src, dst = inputs.rmat_edges(V, w.E, w.graph_seed, device="cuda")
    X = inputs.features(V, d_in)
    W = inputs.glorot_weights(w.dims)[0]
    a_dst, a_src = [x[0] for x in inputs.attention_vectors(w.dims)]
    dh = torch.randn(V, d_out, generator=torch.Generator().manual_seed(9))
    ctx = B.ht_ctx_create(0)
    g = B.ht_partition(ctx, V, src, dst, w.n_chunks)
    try:
        Xd, Wd, ad, asd = B.to_matrix(X), W.cuda(), a_dst.cuda(), a_src.cuda()
        H_out = B.alloc_matrix(V, d_out, zero=False)
        B.ht_gat_layer_fwd(ctx, g, d_in, d_out, B.HT_ACT_RELU, Xd, Wd, ad, asd, H_out)
        h_dev = H_out.cpu().numpy()[:, :d_out]
        note("device forward done")
        indptr, col = orc.csc_build(V, src.cpu().numpy(), dst.cpu().numpy(), add_self_loops=True)
        f = orc.gat_layer_fwd(indptr, col, X.numpy(), W.numpy(), a_dst.numpy(), a_src.numpy(), relu=True)
        note("oracle forward done")
        assert_close(h_dev, f["h"], "h_out")
        Xn, Wn, adn, asn = X.numpy().astype(np.float64), W.numpy().astype(np.float64), a_dst.numpy().astype(np.float64), a_src.numpy().astype(np.float64)
        t, z = f["t"], f["z"]
        # ReLU: the backward pass masks by the sign of the pre-activation.  Of the 59.6 M a few lie within fp32
        # rounding of 0, where either decision is right.  The oracle's z alone says which (bound: the rounding of
        # t = H W and of the weighted sum, against the largest row of t a convex combination can meet); the
        # incoming gradient is set to 0 there, for both sides alike, so that those decisions carry no weight.
        e_t = gat_ties.EPS32 * np.sqrt(d_in) * np.sqrt((Xn * Xn) @ (Wn * Wn))
        err_z = 64.0 * (e_t + gat_ties.EPS32 * np.abs(t)).max(axis=0)
        near_zero = np.abs(z) <= err_z[None, :]
        n_und = int(near_zero.sum())
        assert n_und < 0.01 * z.size, n_und
        flips = (h_dev > 0) != (z > 0)
        assert not (flips & ~near_zero).any(), "a ReLU decision differs outside the rounding bound"
        dh_np = dh.numpy().copy()
        dh_np[near_zero] = 0.0
        note(f"{n_und} pre-activations within rounding of 0 ({int(flips.sum())} on the other side on the device)")
        dW = torch.empty(d_in, d_out, device="cuda")
        dad, das = torch.empty(d_out, device="cuda"), torch.empty(d_out, device="cuda")
        dH_in = B.alloc_matrix(V, d_in)
        st = B.ht_gat_layer_bwd(ctx, g, d_in, d_out, B.HT_ACT_RELU, Xd, Wd, ad, asd, H_out, B.to_matrix(torch.from_numpy(dh_np)),
                                dW, dad, das, dH_in=dH_in, want_stats=True)
        note("device backward done")
        assert st.n_spmm_bwd == 2 * w.n_chunks and st.edges == 2 * (w.E + V)
        b = orc.gat_layer_bwd(indptr, col, X.numpy(), W.numpy(), a_dst.numpy(), a_src.numpy(), f, dh_np, relu=True)
        note("oracle backward done")
        # LeakyReLU: the slope follows the sign of the score y_e = p_v + q_u.  The oracle's fp64 scores say
        # which of the 115 M edges lie within fp32 rounding of 0; for those either slope is right, and the
        # reference becomes an interval over both decisions (tests/gat_ties.py).
        p, q = t @ adn, t @ asn
        err_p = gat_ties.score_halves_error(Xn, Wn, adn, t)
        err_q = gat_ties.score_halves_error(Xn, Wn, asn, t)
        dst_of = np.repeat(np.arange(V, dtype=np.int32), np.diff(indptr))
        y = p[dst_of] + q[col]
        bound = err_p[dst_of] + err_q[col] + 4.0 * gat_ties.EPS32 * (np.abs(p)[dst_of] + np.abs(q)[col])
        ties = np.nonzero(np.abs(y) <= bound)[0]
        note(f"{len(ties)} scores within rounding of 0")
        assert len(ties) < 1e-3 * len(y)
        tv, tu = dst_of[ties].astype(np.int64), col[ties].astype(np.int64)
        dz = np.where(z > 0, dh_np, 0.0)
        dx = gat_ties.edge_dx(tv, tu, f["alpha"][ties], t, z, dz)
        delta = np.where(y[ties] > 0, dx * (0.2 - 1.0), dx * (1.0 - 0.2))       # what the other decision adds to dy_e
        del y, bound, dst_of
        sl = gat_ties.edge_flip_slack(tv, tu, delta, Xn, Wn, adn, asn, t)
        assert_in_interval(dW.cpu().numpy(), b["dW"], *sl["dW"], "dW")
        assert_in_interval(dad.cpu().numpy(), b["da_dst"], *sl["da_dst"], "da_dst")
        assert_in_interval(das.cpu().numpy(), b["da_src"], *sl["da_src"], "da_src")
        rows, lo, hi = sl["dH"]
        dH_dev = dH_in.cpu().numpy()[:, :d_in]
        free = np.ones(V, dtype=bool)
        free[rows] = False
        assert_close_grad(dH_dev[free], b["dH"][free], "dH_in (rows no tie touches)")
        if len(rows):
            scale = np.abs(b["dH"]).max()
            err = dH_dev[rows] - b["dH"][rows]
            assert (err <= hi + 1e-4 * scale).all() and (err >= lo - 1e-4 * scale).all(), "dH_in (rows of tie edges)"
            rn = np.linalg.norm(b["dH"][rows], axis=1)
            out = np.maximum(err - hi, 0.0) + np.minimum(err - lo, 0.0)
            assert (np.linalg.norm(out, axis=1) <= 1e-4 * np.maximum(rn, GRAD_ROW_FLOOR * np.median(np.linalg.norm(b["dH"], axis=1)))).all()
    finally:
        B.ht_graph_destroy(g)
        B.ht_ctx_destroy(ctx)

"""Parity at full size with host-resident vertex data (config 3: 2.45 M vertices, 61.9 M edges,
100-256-256-47, 16 chunks; h^l and grad h^l in pinned host memory, a^l in HBM), in the
configuration `bench.py --workload cfg3` runs: dedup gather through the in-place neighbour buffer,
checkpoint rows leaving through the output stream, gradient rows leaving by compaction, D2H and the
host-side add (or stored straight home with the keep-all buffer).

Each layer step is recomputed by the oracle in fp64 from that step's actual inputs (read back
from the device) on sampled rows, sources and weight-gradient columns.  ReLU decisions are read
from the device's own h^{l+1} (the fp32 decision), so ties need no special care here.
"""
import time

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2311_14898_amd import binding as B
from paper_2311_14898_amd import inputs
from tests.util import assert_close, assert_close_grad, assert_in_interval, relu_tie_slack

pytestmark = pytest.mark.gpu
N_SAMPLE = 160


@pytest.fixture(scope="module")
def data():
    w = inputs.WORKLOADS["cfg3"]
    src, dst = inputs.rmat_edges(w.V, w.E, w.graph_seed, device="cuda")
    d = {"w": w, "src_d": src, "dst_d": dst, "src": src.cpu().numpy(), "dst": dst.cpu().numpy(),
         "X": inputs.features(w.V, w.dims[0]), "y": inputs.labels(w.V, w.dims[-1]), "Ws": inputs.glorot_weights(w.dims)}
    deg = np.bincount(d["dst"], minlength=w.V)
    d["deg"] = deg
    d["s"] = orc.norm(np.concatenate([[0], np.cumsum(deg.astype(np.int64) + 1)]))
    # sampled destination rows (with their in-edges) and sampled sources (with their out-edges)
    rng = np.random.default_rng(5)
    hubs = np.argsort(deg)[-3:]
    d["rows"] = np.unique(np.concatenate([rng.integers(0, w.V, N_SAMPLE), hubs, [0, w.V - 1]]))
    keep = np.isin(d["dst"], d["rows"])
    d["csc_rows"] = orc.csc_build(w.V, d["src"][keep], d["dst"][keep], add_self_loops=True)
    d["us"] = np.unique(np.concatenate([rng.integers(0, w.V, 48), hubs[:2]]))
    out = np.isin(d["src"], d["us"])
    so, do = d["src"][out], d["dst"][out]
    d["out_nbrs"] = {int(u): np.concatenate([do[so == u], [u]]) for u in d["us"]}
    return d


@pytest.mark.parametrize("cache_rows", [0, -1], ids=["adjacent-reuse", "keep-all"])
def test_cfg3_host_resident_epoch(data, cache_rows):
    w, src, dst, s, deg = data["w"], data["src"], data["dst"], data["s"], data["deg"]
    V, dims, L = w.V, w.dims, w.n_layers
    X, y, Ws = data["X"].numpy(), data["y"].numpy(), [x.numpy() for x in data["Ws"]]
    t_start = time.perf_counter()

    def note(msg):
        print(f"[{time.perf_counter() - t_start:6.1f}s] {msg}", flush=True)

    ctx = B.ht_ctx_create(0)
    g = B.ht_partition(ctx, V, data["src_d"], data["dst_d"], w.n_chunks, cache_rows=cache_rows)
    try:
        Wd = [x.clone().cuda() for x in data["Ws"]]
        loss, st = B.ht_epoch(ctx, g, dims, Wd, w.lr, B.to_matrix(data["X"], B.HT_LOC_HOST_PINNED), data["y"].cuda(),
                              res_h=B.HT_RES_HOST, res_g=B.HT_RES_HOST, want_stats=True)
        info = B.ht_graph_info_get(g)
        # link traffic: neighbour rows per forward pass as the partition promised, plus contiguous ranges
        assert st.rows_loaded == info.v_load * L and st.rows_loaded + st.rows_reused == info.v_ori * L
        assert st.bytes_h2d_nodedup == 4 * sum(dims[:L]) * info.v_ori
        assert st.bytes_h2d >= 4 * sum(dims[:L]) * info.v_load and st.bytes_d2h > 0
        a_dev = [B.ht_epoch_buffer(ctx, B.HT_BUF_A, l).numpy() for l in range(L)]
        note(f"epoch done ({st.t_total_ms:.0f} ms), a^l read back")
        h_dev = [X] + [B.ht_epoch_buffer(ctx, B.HT_BUF_H, l + 1).numpy() for l in range(L)]
        gh_dev = [None] + [B.ht_epoch_buffer(ctx, B.HT_BUF_GH, l + 1).numpy() for l in range(L)]
        gW_dev = [B.ht_epoch_buffer(ctx, B.HT_BUF_DW, l).numpy() for l in range(L)]
        W_new = [x.cpu().numpy() for x in Wd]
        note("all buffers read back")
    finally:
        B.ht_graph_destroy(g)
        B.ht_ctx_destroy(ctx)

    rng = np.random.default_rng(6)
    rows, us = data["rows"], data["us"]
    indptr_s, col_s = data["csc_rows"]
    full = cache_rows == 0          # the second buffer policy re-checks what it changes: loads, leaving rows, the end results
    for l in range(L if full else 0):
        a_ref = orc.aggregate(indptr_s, col_s, h_dev[l], s=s)[rows]
        assert_close(a_dev[l][rows], a_ref, f"a^{l} rows")
        z_ref = orc.matmul(a_dev[l][rows], Ws[l])
        assert_close(h_dev[l + 1][rows], np.maximum(z_ref, 0.0) if l < L - 1 else z_ref, f"h^{l + 1} rows")
    note("forward rows checked")
    if full:
        # the same forward pass by an oracle run that shares only the seeded inputs with the device (its own CSC,
        # its own layer inputs); forward values do not depend on how a pre-activation within rounding of 0 is resolved
        indptr, col = orc.csc_build(V, src, dst)
        h = X
        rows_i = np.unique(np.random.default_rng(8).integers(0, V, 4096))
        for l in range(L):
            a = orc.aggregate(indptr, col, h)
            assert_close(a_dev[l][rows_i], a[rows_i], f"a^{l} rows, independent pass")
            z = orc.matmul(a, Ws[l])
            h = np.maximum(z, 0.0) if l < L - 1 else z
            assert_close(h_dev[l + 1][rows_i], h[rows_i], f"h^{l + 1} rows, independent pass")
        loss_ind, _ = orc.softmax_ce(h, y)
        assert abs(loss - loss_ind) <= 1e-4 * abs(loss_ind), (loss, loss_ind)
        del indptr, col, a, z, h
        note("independent forward pass checked")
    loss_ref, g_ref = orc.softmax_ce(h_dev[L], y)
    assert abs(loss - loss_ref) <= 1e-4 * abs(loss_ref)
    assert_close_grad(gh_dev[L][rows], g_ref[rows], "grad h^L rows")
    for l in range(L - 1, -1, -1):
        note(f"backward of layer {l}")
        gh = gh_dev[l + 1].astype(np.float64)
        dz = np.where(h_dev[l + 1] > 0.0, gh, 0.0) if l < L - 1 else gh
        cols = np.unique(rng.integers(0, dims[l + 1], 6))
        # (numpy's fp64 product here: the oracle's transposed product walks this tall operand column by column)
        gW_ref = a_dev[l].T.astype(np.float64) @ np.ascontiguousarray(dz[:, cols])
        assert (np.abs(gW_dev[l][:, cols] - gW_ref) <= 1e-4 * np.abs(gW_dev[l]).max()).all(), f"grad W^{l} columns"
        assert_close_grad(W_new[l], Ws[l].astype(np.float64) - w.lr * gW_dev[l].astype(np.float64), f"W^{l} step")
        if l > 0:
            scale = np.abs(gh_dev[l]).max()
            for u in us:
                vs = data["out_nbrs"][int(u)]
                da = orc.matmul_nt(dz[vs], Ws[l])
                ref = s[u] * (s[vs][:, None] * da).sum(axis=0)
                assert (np.abs(gh_dev[l][u] - ref) <= 1e-4 * scale).all(), (l, u)


def test_cfg3_whole_epoch_against_an_independent_oracle_epoch(data):
    """Alg. 1 end to end with h^l and grad h^l in pinned host memory (gather through the in-place buffer, gradient
    rows leaving over the link, host-side adds): loss, every weight gradient and every updated weight matrix against
    a whole fp64 oracle epoch that shares only the seeded inputs with the device (about a minute of host time).
    Pre-activations that fp32 cannot tell from 0 enter as an interval computed from the oracle's values alone."""
    w = data["w"]
    V, dims, L = w.V, w.dims, w.n_layers
    X, y, Ws = data["X"].numpy(), data["y"].numpy(), [x.numpy() for x in data["Ws"]]
    t_start = time.perf_counter()
    note = lambda msg: print(f"[{time.perf_counter() - t_start:6.1f}s] {msg}", flush=True)
    ctx = B.ht_ctx_create(0)
    g = B.ht_partition(ctx, V, data["src_d"], data["dst_d"], w.n_chunks)
    try:
        Wd = [x.clone().cuda() for x in data["Ws"]]
        loss, _ = B.ht_epoch(ctx, g, dims, Wd, w.lr, B.to_matrix(data["X"], B.HT_LOC_HOST_PINNED), data["y"].cuda(),
                             res_h=B.HT_RES_HOST, res_g=B.HT_RES_HOST)
        gW_dev = [B.ht_epoch_buffer(ctx, B.HT_BUF_DW, l).numpy() for l in range(L)]
        W_new = [x.cpu().numpy() for x in Wd]
    finally:
        B.ht_graph_destroy(g)
        B.ht_ctx_destroy(ctx)
    note("device epoch done")
    indptr, col = orc.csc_build(V, data["src"], data["dst"])
    ref = orc.gcn_epoch(indptr, col, dims, X, Ws, y, lr=w.lr, want=("a", "z", "gh"))
    note("oracle epoch done")
    assert abs(loss - ref["loss"]) <= 1e-4 * abs(ref["loss"]), (loss, ref["loss"])
    slack = relu_tie_slack(ref, indptr, col, Ws, dims)
    for l in range(L):
        lo, hi, ties = slack[l]
        note(f"layer {l}: {len(ties[0])} pre-activations within rounding of 0; they can move grad W^{l} by "
             f"{max(hi.max(), -lo.min()) / np.abs(ref['gW'][l]).max():.1e} of its largest entry")
        assert_in_interval(gW_dev[l], ref["gW"][l], lo, hi, f"grad W^{l}, independent epoch")
        assert_in_interval(W_new[l], ref["W_new"][l], -w.lr * hi, -w.lr * lo, f"W^{l} after the step, independent epoch")

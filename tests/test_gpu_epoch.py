"""ht_epoch against the CPU oracle: loss, every activation and gradient, updated weights."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2311_14898_amd import binding as B
from paper_2311_14898_amd import inputs
from tests.util import assert_close, assert_close_grad

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = B.ht_ctx_create(0)
    yield c
    B.ht_ctx_destroy(c)


def run_epoch(ctx, w, src, dst, X, y, Ws, n_chunks=None, x_loc=B.HT_LOC_DEVICE, cache_rows=0, reorder=False,
              update_first=(), cache_policy=0, **plan):
    """update_first: the layers expected to run update-first (they keep no aggregate checkpoint)."""
    g = B.ht_partition(ctx, w.V, src.cuda(), dst.cuda(), n_chunks or w.n_chunks, cache_rows=cache_rows,
                       reorder_chunks=reorder, cache_policy=cache_policy)
    try:
        Xd = B.to_matrix(X, x_loc)
        Wd = [x.clone().cuda() for x in Ws]
        loss, st = B.ht_epoch(ctx, g, w.dims, Wd, w.lr, Xd, y.cuda(), want_stats=True, **plan)
        L = w.n_layers
        out = {"loss": loss, "stats": st, "W_new": [x.cpu().numpy() for x in Wd],
               "a": [B.ht_epoch_buffer(ctx, B.HT_BUF_A, l).numpy() if l not in update_first else None
                     for l in range(L)],
               "h": [B.ht_epoch_buffer(ctx, B.HT_BUF_H, l + 1).numpy() for l in range(L)],
               "gh": [B.ht_epoch_buffer(ctx, B.HT_BUF_GH, l + 1).numpy() for l in range(L)],
               "gW": [B.ht_epoch_buffer(ctx, B.HT_BUF_DW, l).numpy() for l in range(L)]}
        return out
    finally:
        B.ht_graph_destroy(g)


def oracle_epoch(w, src, dst, X, y, Ws):
    indptr, col = orc.csc_build(w.V, src.numpy(), dst.numpy())
    return orc.gcn_epoch(indptr, col, w.dims, X.numpy(), [x.numpy() for x in Ws], y.numpy(), lr=w.lr)


def compare(out, ref, L):
    assert abs(out["loss"] - ref["loss"]) <= 1e-4 * abs(ref["loss"]), (out["loss"], ref["loss"])
    for l in range(L):
        if out["a"][l] is not None:
            assert_close(out["a"][l], ref["a"][l], f"a^{l}")
        assert_close(out["h"][l], ref["h"][l], f"h^{l + 1}")
        assert_close_grad(out["gh"][l], ref["gh"][l], f"grad h^{l + 1}")
        assert_close_grad(out["gW"][l], ref["gW"][l], f"grad W^{l}")
        assert_close_grad(out["W_new"][l], ref["W_new"][l], f"W^{l} after the step")


@pytest.fixture(scope="module")
def cfg1():
    w = inputs.WORKLOADS["cfg1"]
    src, dst, X, y, Ws = inputs.make_inputs(w)
    ref = oracle_epoch(w, src, dst, X, y, Ws)
    # the fp32 path and the fp64 oracle must take the same ReLU decisions
    for l in range(w.n_layers - 1):
        assert np.abs(ref["z"][l]).min() > 1e-6
    return w, src, dst, X, y, Ws, ref


def test_cfg1_all_in_hbm(ctx, cfg1):
    w, src, dst, X, y, Ws, ref = cfg1
    out = run_epoch(ctx, w, src, dst, X, y, Ws)
    compare(out, ref, w.n_layers)
    st = out["stats"]
    assert st.edges == (w.E + w.V) * (2 * w.n_layers - 1)      # L forward + (L-1) backward aggregations
    assert st.bytes_h2d == 0 and st.bytes_d2h == 0


def test_cfg1_hybrid_equals_mask_bitwise(ctx, cfg1):
    # Sec. 4.2: recomputing the update stage regenerates identical intermediates
    w, src, dst, X, y, Ws, ref = cfg1
    a = run_epoch(ctx, w, src, dst, X, y, Ws, inter=B.HT_INTER_MASK)
    b = run_epoch(ctx, w, src, dst, X, y, Ws, inter=B.HT_INTER_HYBRID)
    assert a["loss"] == b["loss"]
    for l in range(w.n_layers):
        assert np.array_equal(a["gW"][l], b["gW"][l]) and np.array_equal(a["W_new"][l], b["W_new"][l])
        assert np.array_equal(a["gh"][l], b["gh"][l])


def test_cfg1_host_resident_with_buffer(ctx, cfg1):
    # vertex data, checkpoints and gradients in pinned host memory: dedup gather through the
    # in-place buffer, D2H compaction and CPU-side accumulation
    w, src, dst, X, y, Ws, ref = cfg1
    out = run_epoch(ctx, w, src, dst, X, y, Ws, x_loc=B.HT_LOC_HOST_PINNED, res_h=B.HT_RES_HOST,
                    res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST)
    compare(out, ref, w.n_layers)
    st = out["stats"]
    assert st.rows_loaded + st.rows_reused > 0 and st.bytes_h2d > 0 and st.bytes_d2h > 0
    assert st.bytes_h2d_nodedup >= 4 * w.dims[0] * st.rows_loaded // w.n_layers


def test_cfg1_host_resident_keep_all_buffer(ctx, cfg1):
    # a buffer as large as the source set: every row crosses the link once per pass
    w, src, dst, X, y, Ws, ref = cfg1
    out = run_epoch(ctx, w, src, dst, X, y, Ws, x_loc=B.HT_LOC_HOST_PINNED, cache_rows=-1, res_h=B.HT_RES_HOST,
                    res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST)
    compare(out, ref, w.n_layers)
    st = out["stats"]
    assert st.rows_loaded == w.V * w.n_layers          # V rows per forward pass, not V_+ru
    out = run_epoch(ctx, w, src, dst, X, y, Ws, cache_rows=-1, gather_mode=B.HT_GATHER_BUFFER)
    compare(out, ref, w.n_layers)


def test_cfg1_host_resident_farthest_next_use_buffer(ctx, cfg1):
    # a buffer between the two extremes that releases rows only for room: same results, fewer rows over the link
    w, src, dst, X, y, Ws, ref = cfg1
    host = dict(x_loc=B.HT_LOC_HOST_PINNED, res_h=B.HT_RES_HOST, res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST)
    base = run_epoch(ctx, w, src, dst, X, y, Ws, n_chunks=8, **host)["stats"].rows_loaded
    last = base
    for rows in (0, 7000, 9000):
        out = run_epoch(ctx, w, src, dst, X, y, Ws, n_chunks=8, cache_rows=rows, cache_policy=B.HT_CACHE_FARTHEST,
                        **host)
        compare(out, ref, w.n_layers)
        assert out["stats"].rows_loaded <= last
        last = out["stats"].rows_loaded
    assert last < base
    compare(run_epoch(ctx, w, src, dst, X, y, Ws, n_chunks=8, cache_rows=7000, cache_policy=B.HT_CACHE_FARTHEST,
                      reorder=True, gather_mode=B.HT_GATHER_BUFFER), ref, w.n_layers)


def test_cfg1_buffer_mode_in_hbm_and_chunk_count_invariance(ctx, cfg1):
    w, src, dst, X, y, Ws, ref = cfg1
    out = run_epoch(ctx, w, src, dst, X, y, Ws, gather_mode=B.HT_GATHER_BUFFER)
    compare(out, ref, w.n_layers)
    for n in (1, 9):
        compare(run_epoch(ctx, w, src, dst, X, y, Ws, n_chunks=n), ref, w.n_layers)
    # reorganised schedule (Alg. 4 phase 2): same result, host-resident and in HBM
    compare(run_epoch(ctx, w, src, dst, X, y, Ws, n_chunks=9, reorder=True), ref, w.n_layers)
    compare(run_epoch(ctx, w, src, dst, X, y, Ws, n_chunks=9, reorder=True, x_loc=B.HT_LOC_HOST_PINNED,
                      res_h=B.HT_RES_HOST, res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST), ref, w.n_layers)


def test_cfg1_pure_recomputation(ctx, cfg1):
    # Fig. 5(b): no aggregate checkpoints; the backward pass gathers and aggregates again from h^l
    w, src, dst, X, y, Ws, ref = cfg1
    L = w.n_layers
    out = run_epoch(ctx, w, src, dst, X, y, Ws, inter=B.HT_INTER_RECOMPUTE, update_first=range(L))
    compare(out, ref, L)
    assert out["stats"].edges == (w.E + w.V) * (3 * L - 1)       # L forward, L recomputed, L-1 backward
    out = run_epoch(ctx, w, src, dst, X, y, Ws, inter=B.HT_INTER_RECOMPUTE, update_first=range(L),
                    x_loc=B.HT_LOC_HOST_PINNED, res_h=B.HT_RES_HOST, res_g=B.HT_RES_HOST)
    compare(out, ref, L)
    # the regenerated intermediates are the ones the hybrid caches: same bits
    a = run_epoch(ctx, w, src, dst, X, y, Ws, inter=B.HT_INTER_HYBRID)
    b = run_epoch(ctx, w, src, dst, X, y, Ws, inter=B.HT_INTER_RECOMPUTE, update_first=range(L))
    for l in range(L):
        assert np.array_equal(a["gW"][l], b["gW"][l]) and np.array_equal(a["gh"][l], b["gh"][l])


def test_input_aggregate_reused_across_epochs(ctx, cfg1):
    """a^0 = A_hat X does not depend on the parameters: epochs that take the cached copy give the same bits as
    epochs that aggregate layer 0 again, in HBM and with host-resident tensors, and skip that aggregation."""
    w, src, dst, X, y, Ws, ref = cfg1
    L = w.n_layers
    Ep = w.E + w.V
    for host in (False, True):
        loc = B.HT_LOC_HOST_PINNED if host else B.HT_LOC_DEVICE
        plan = dict(res_h=B.HT_RES_HOST, res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST) if host else {}
        g = B.ht_partition(ctx, w.V, src.cuda(), dst.cuda(), w.n_chunks)
        try:
            Xd, yd = B.to_matrix(X, loc), y.cuda()
            runs = {}
            for reuse in (False, True):
                Wd = [x.clone().cuda() for x in Ws]
                losses, edges = [], []
                for k in range(3):
                    loss, st = B.ht_epoch(ctx, g, w.dims, Wd, w.lr, Xd, yd, want_stats=True, reuse_input_aggregate=reuse,
                                          **plan)
                    losses.append(loss)
                    edges.append(st.edges)
                runs[reuse] = (losses, edges, [x.cpu().numpy() for x in Wd],
                               B.ht_epoch_buffer(ctx, B.HT_BUF_A, 0).numpy() if reuse else None)
            assert runs[True][0] == runs[False][0]
            for a, b in zip(runs[True][2], runs[False][2]):
                assert np.array_equal(a, b)
            assert_close(runs[True][3], ref["a"][0], "a^0 kept")
            # L forward and L - 1 backward aggregations; minus layer 0's when its aggregate is taken from an earlier
            # epoch (the epochs without the flag, same X and graph, left it behind)
            assert runs[False][1] == [Ep * (2 * L - 1)] * 3 and runs[True][1] == [Ep * (2 * L - 2)] * 3
            # another X (same values, new address): aggregated again
            X2 = B.to_matrix(X, loc)
            Wd = [x.clone().cuda() for x in Ws]
            _, st = B.ht_epoch(ctx, g, w.dims, Wd, w.lr, X2, yd, want_stats=True, reuse_input_aggregate=True, **plan)
            assert st.edges == Ep * (2 * L - 1)
            # with HT_ORDER_AUTO layer 0 keeps the printed order (its aggregate is what is reused), layer 1 runs
            # update-first: two epochs against two epochs of the oracle
            if not host:
                Wd = [x.clone().cuda() for x in Ws]
                for k in range(2):
                    _, st = B.ht_epoch(ctx, g, w.dims, Wd, w.lr, Xd, yd, want_stats=True, reuse_input_aggregate=True,
                                       order=B.HT_ORDER_AUTO)
                assert st.edges == Ep * (2 * L - 2)
                indptr, col = orc.csc_build(w.V, src.numpy(), dst.numpy())
                W2 = orc.gcn_epoch(indptr, col, w.dims, X.numpy(), ref["W_new"], y.numpy(), lr=w.lr)["W_new"]
                for l in range(L):
                    assert_close_grad(Wd[l].cpu().numpy(), W2[l], f"W^{l} after two epochs")
        finally:
            B.ht_graph_destroy(g)


def test_epoch_replayed_from_a_hip_graph(ctx, cfg1):
    """use_graph: the first epoch of a key runs eagerly, the second is captured and launched, later ones are
    replays.  Every epoch must give the bits of an eager epoch, with other work on the context (also work that
    reallocates the library's scratch memory) and synchronisations between the replays, and after a change of lr."""
    w, src, dst, X, y, Ws, ref = cfg1
    g = B.ht_partition(ctx, w.V, src.cuda(), dst.cuda(), w.n_chunks)
    try:
        Xd, yd = B.to_matrix(X), y.cuda()
        for order, reuse in ((B.HT_ORDER_AGG_FIRST, False), (B.HT_ORDER_AUTO, True)):
            lrs = [w.lr] * 6 + [0.5] * 4
            eager, Wd = [], [x.clone().cuda() for x in Ws]
            for lr in lrs:
                loss, _ = B.ht_epoch(ctx, g, w.dims, Wd, lr, Xd, yd, order=order, reuse_input_aggregate=reuse)
                eager.append((loss, [x.cpu().numpy().copy() for x in Wd]))
            Wd = [x.clone().cuda() for x in Ws]
            n_graph = B.ht_ctx_graph_launches(ctx)
            side_in = B.to_matrix(inputs.features(w.V, 24, seed=9))
            big_in = B.to_matrix(inputs.features(w.V, 200, seed=10))
            for k, lr in enumerate(lrs):
                loss, _ = B.ht_epoch(ctx, g, w.dims, Wd, lr, Xd, yd, order=order, reuse_input_aggregate=reuse, use_graph=True)
                assert loss == eager[k][0], (k, loss, eager[k][0])
                for a, b in zip(Wd, eager[k][1]):
                    assert np.array_equal(a.cpu().numpy(), b), f"epoch {k}"
                # other work between the epochs: a layer on the same context (it overwrites scratch memory), once
                # with rows so wide that scratch slots grow and move (k == 3: in the middle of the replays)
                d_in, h_in = (200, big_in) if k == 3 else (24, side_in)
                Wl = torch.ones(d_in, 16, device="cuda")
                B.ht_layer_fwd(ctx, g, d_in, 16, B.HT_ACT_RELU, h_in, Wl, B.alloc_matrix(w.V, 16), gather_mode=B.HT_GATHER_BUFFER)
                torch.cuda.synchronize()
            # eager, captured + launched, replays; after the scratch moved and after the new lr: eager, captured, replays
            assert B.ht_ctx_graph_launches(ctx) - n_graph >= 5, B.ht_ctx_graph_launches(ctx) - n_graph
    finally:
        B.ht_graph_destroy(g)


def test_epoch_falls_back_when_the_capture_breaks(ctx, cfg1, monkeypatch):
    """HT_GRAPH_DEBUG=3 makes the library issue, while it captures, one launch that the runtime rejects on the host
    (an impossible block size; nothing reaches the GPU): the capture is dropped, the epoch runs eagerly with the
    same result, and that key is not captured again."""
    w, src, dst, X, y, Ws, ref = cfg1
    g = B.ht_partition(ctx, w.V, src.cuda(), dst.cuda(), w.n_chunks)
    try:
        Xd, yd = B.to_matrix(X), y.cuda()
        runs = []
        for broken in (False, True):
            if broken:
                monkeypatch.setenv("HT_GRAPH_DEBUG", "3")
            Wd = [x.clone().cuda() for x in Ws]
            n0 = B.ht_ctx_graph_launches(ctx)
            losses = [B.ht_epoch(ctx, g, w.dims, Wd, 0.3, Xd, yd, use_graph=broken)[0] for _ in range(5)]
            runs.append((losses, [x.cpu().numpy() for x in Wd]))
            assert B.ht_ctx_graph_launches(ctx) == n0
        assert runs[0][0] == runs[1][0]
        for a, b in zip(runs[0][1], runs[1][1]):
            assert np.array_equal(a, b)
    finally:
        B.ht_graph_destroy(g)


def test_planner_prices_recomputation_against_the_host_side_cache(ctx, cfg1):
    """HT_INTER_AUTO under a byte budget that a^l does not fit (Sec. 4.2's trade-off, priced for this GPU)."""
    w, src, dst, X, y, Ws, ref = cfg1
    L = w.n_layers
    MB = 1 << 20
    # room for everything: a^l cached in HBM, ReLU' read from h^{l+1}
    st = run_epoch(ctx, w, src, dst, X, y, Ws, hbm_budget_bytes=64 * MB)["stats"]
    assert (st.plan_inter, st.plan_res_a, st.plan_res_h, st.plan_res_g) == (B.HT_INTER_MASK, B.HT_RES_HBM, B.HT_RES_HBM, B.HT_RES_HBM)
    # logits 0.64 MB, grad h 1.28 MB, h 1.28 MB fit, a^l (3.84 MB) does not; h^l in HBM: aggregating again costs no
    # link traffic at all, the host-side cache would cost 2 x 3.84 MB of it
    out = run_epoch(ctx, w, src, dst, X, y, Ws, hbm_budget_bytes=int(4.2 * MB), update_first=range(L))
    compare(out, ref, L)
    st = out["stats"]
    assert (st.plan_inter, st.plan_res_h, st.plan_res_g) == (B.HT_INTER_RECOMPUTE, B.HT_RES_HBM, B.HT_RES_HBM)
    assert st.bytes_h2d == 0 and st.bytes_d2h == 0 and st.edges == (w.E + w.V) * (3 * L - 1)
    # nothing fits and X is on the host: recomputation fetches the buffer schedule's rows once more (v_load per
    # layer) where the cache moves 2 V rows: it wins with a schedule that loads every row once, not with the
    # adjacent-reuse buffer of many small chunks
    host = dict(x_loc=B.HT_LOC_HOST_PINNED, hbm_budget_bytes=MB // 4)
    out = run_epoch(ctx, w, src, dst, X, y, Ws, cache_rows=-1, update_first=range(L), **host)
    compare(out, ref, L)
    assert out["stats"].plan_inter == B.HT_INTER_RECOMPUTE and out["stats"].plan_res_h == B.HT_RES_HOST
    g = B.ht_partition(ctx, w.V, src.cuda(), dst.cuda(), 32)
    v_load = B.ht_graph_info_get(g).v_load
    B.ht_graph_destroy(g)
    assert v_load > 2.3 * w.V
    out = run_epoch(ctx, w, src, dst, X, y, Ws, n_chunks=32, **host)
    compare(out, ref, L)
    assert (out["stats"].plan_inter, out["stats"].plan_res_a) == (B.HT_INTER_HYBRID, B.HT_RES_HOST)
    # a caller who places a^l on the host keeps the hybrid
    st = run_epoch(ctx, w, src, dst, X, y, Ws, res_a=B.HT_RES_HOST)["stats"]
    assert st.plan_inter in (B.HT_INTER_MASK, B.HT_INTER_HYBRID) and st.plan_res_a == B.HT_RES_HOST


def test_cfg1_update_first_order(ctx, cfg1):
    # H' = act(A_hat (H W)): the same function as Eq. 2 with the two linear stages swapped
    w, src, dst, X, y, Ws, ref = cfg1
    L = w.n_layers
    out = run_epoch(ctx, w, src, dst, X, y, Ws, order=B.HT_ORDER_UPDATE_FIRST, update_first=range(L))
    compare(out, ref, L)
    assert out["stats"].edges == (w.E + w.V) * 2 * L            # one aggregation per layer and direction
    # AUTO: only layers that get narrower (64 -> 32 -> 8: both)
    compare(run_epoch(ctx, w, src, dst, X, y, Ws, order=B.HT_ORDER_AUTO, update_first=range(L), n_chunks=7), ref, L)
    # host-resident tensors keep the printed order whatever is asked for
    out = run_epoch(ctx, w, src, dst, X, y, Ws, order=B.HT_ORDER_AUTO, x_loc=B.HT_LOC_HOST_PINNED,
                    res_h=B.HT_RES_HOST, res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST)
    compare(out, ref, L)
    with pytest.raises(B.HongtuError):
        run_epoch(ctx, w, src, dst, X, y, Ws, order=7)


def test_update_first_only_where_narrower(ctx):
    w = inputs.Workload("t3w", 6000, 70_000, [24, 40, 20, 12], 5, labelled_one_in=3, graph_seed=6)
    src, dst, X, y, Ws = inputs.make_inputs(w)
    ref = oracle_epoch(w, src, dst, X, y, Ws)
    for l in range(w.n_layers - 1):
        assert np.abs(ref["z"][l]).min() > 1e-7 * np.abs(ref["z"][l]).max()
    compare(run_epoch(ctx, w, src, dst, X, y, Ws, order=B.HT_ORDER_AUTO, update_first=(1, 2)), ref, 3)


def test_three_layers_partial_labels(ctx):
    w = inputs.Workload("t3", 6000, 70_000, [24, 40, 20, 12], 5, labelled_one_in=3, graph_seed=6)
    src, dst, X, y, Ws = inputs.make_inputs(w)
    ref = oracle_epoch(w, src, dst, X, y, Ws)
    for l in range(w.n_layers - 1):     # same ReLU decisions on both sides (this graph seed was picked for it)
        assert np.abs(ref["z"][l]).min() > 1e-7 * np.abs(ref["z"][l]).max()
    compare(run_epoch(ctx, w, src, dst, X, y, Ws), ref, 3)
    compare(run_epoch(ctx, w, src, dst, X, y, Ws, x_loc=B.HT_LOC_HOST_PINNED, res_h=B.HT_RES_HOST,
                      res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST), ref, 3)


def test_empty_chunks_with_schedule_aware_buffer(ctx):
    """Hub destinations swallow several edge targets, so some chunks have no destinations; the schedule may still
    release rows at such a position (room for the chunk after it), and the backward pass must write them back."""
    V = 900
    rng = np.random.default_rng(4)
    src = np.concatenate([rng.integers(0, V, 4000), rng.integers(0, V, 3000), rng.integers(0, V, 2500)])
    dst = np.concatenate([rng.integers(0, V, 4000), np.full(3000, 300), np.full(2500, 301)])
    keep = src != dst
    src, dst = torch.from_numpy(src[keep].astype(np.int32)), torch.from_numpy(dst[keep].astype(np.int32))
    w = inputs.Workload("hubs", V, int(src.numel()), [20, 16, 6], 12)
    X, y, Ws = inputs.features(V, 20), inputs.labels(V, 6), inputs.glorot_weights(w.dims)
    ref = oracle_epoch(w, src, dst, X, y, Ws)
    host = dict(x_loc=B.HT_LOC_HOST_PINNED, res_h=B.HT_RES_HOST, res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST)
    g = B.ht_partition(ctx, V, src.cuda(), dst.cuda(), w.n_chunks)
    cis = [B.ht_graph_chunk_info(g, j) for j in range(w.n_chunks)]
    B.ht_graph_destroy(g)
    assert any(c.dst_end == c.dst_begin for c in cis[:-1]), "the case needs an empty chunk in the middle"
    for kw in (dict(), dict(cache_policy=B.HT_CACHE_FARTHEST), dict(cache_rows=-1),
               dict(cache_rows=int(1.2 * max(c.n_src for c in cis)), cache_policy=B.HT_CACHE_FARTHEST)):
        compare(run_epoch(ctx, w, src, dst, X, y, Ws, **kw, **host), ref, w.n_layers)
        compare(run_epoch(ctx, w, src, dst, X, y, Ws, gather_mode=B.HT_GATHER_BUFFER, **kw), ref, w.n_layers)


def test_uniform_logits_loss_is_ln_C(ctx):
    w = inputs.WORKLOADS["cfg1"]
    src, dst, X, y, _ = inputs.make_inputs(w)
    Ws = [torch.zeros(w.dims[l], w.dims[l + 1]) for l in range(w.n_layers)]
    out = run_epoch(ctx, w, src, dst, X, y, Ws)
    assert abs(out["loss"] - np.log(8.0)) < 1e-6


def test_two_epochs_reuse_workspace_and_loss_decreases(ctx, cfg1):
    w, src, dst, X, y, Ws, ref = cfg1
    g = B.ht_partition(ctx, w.V, src.cuda(), dst.cuda(), w.n_chunks)
    try:
        Xd = B.to_matrix(X)
        Wd = [x.clone().cuda() for x in Ws]
        yd = y.cuda()
        l0, _ = B.ht_epoch(ctx, g, w.dims, Wd, 0.5, Xd, yd)
        l1, _ = B.ht_epoch(ctx, g, w.dims, Wd, 0.5, Xd, yd)
        l2, _ = B.ht_epoch(ctx, g, w.dims, Wd, 0.5, Xd, yd)
        assert abs(l0 - ref["loss"]) <= 1e-4 * ref["loss"]
        assert l2 < l1 < l0
    finally:
        B.ht_graph_destroy(g)


def test_stats_detail_times_only_the_forward_aggregation(ctx, cfg1):
    w, src, dst, X, y, Ws, ref = cfg1
    full = run_epoch(ctx, w, src, dst, X, y, Ws)
    lean = run_epoch(ctx, w, src, dst, X, y, Ws, stats_detail=B.HT_STATS_AGG_FWD)
    assert lean["loss"] == full["loss"]
    for l in range(w.n_layers):
        assert np.array_equal(lean["W_new"][l], full["W_new"][l])
    a, b = full["stats"].as_dict(), lean["stats"].as_dict()
    assert all(t > 0 for t in b["t_agg_fwd_layer_ms"][:w.n_layers]) and b["t_spmm_fwd_ms"] > 0
    for k in ("t_gemm_ms", "t_spmm_bwd_ms", "t_loss_ms", "t_update_ms", "t_agg_fix_ms"):
        assert a[k] > 0 and b[k] == 0, k
    for k in ("edges", "gemm_flops", "n_spmm_fwd", "n_spmm_bwd", "spmm_fwd_alg_bytes", "rows_loaded", "bytes_h2d"):
        assert a[k] == b[k], k
    with pytest.raises(B.HongtuError):
        run_epoch(ctx, w, src, dst, X, y, Ws, stats_detail=7)


def test_hbm_budget_refusals_leave_the_context_usable(cfg1):
    """ht_ctx_set_hbm_budget: a call that would allocate beyond the cap returns HT_ENOMEM at whatever allocation
    crosses it (in the partition, in the epoch's workspace or in a scratch slot), frees what it had taken, and the
    same context works once the cap is lifted."""
    w, src, dst, X, y, Ws, ref = cfg1
    ctx = B.ht_ctx_create(0)
    try:
        refused_part = refused_epoch = passed = 0
        for budget in [1 << 10, 1 << 17, 1 << 20, 3 << 20, 5 << 20, 6 << 20, 7 << 20, 8 << 20, 10 << 20, 12 << 20,
                       16 << 20, 24 << 20, 64 << 20]:
            B.ht_ctx_set_hbm_budget(ctx, budget)
            try:
                g = B.ht_partition(ctx, w.V, src.cuda(), dst.cuda(), w.n_chunks)
            except B.HongtuError as e:
                assert e.code == B.HT_ENOMEM, str(e)
                refused_part += 1
                continue
            try:
                Wd = [x.clone().cuda() for x in Ws]
                loss, _ = B.ht_epoch(ctx, g, w.dims, Wd, w.lr, B.to_matrix(X), y.cuda())
                assert abs(loss - ref["loss"]) <= 1e-4 * abs(ref["loss"])
                passed += 1
            except B.HongtuError as e:
                assert e.code == B.HT_ENOMEM, str(e)
                refused_epoch += 1
            finally:
                B.ht_graph_destroy(g)
        assert refused_part > 0 and passed > 0, (refused_part, refused_epoch, passed)
        # had the refused calls kept their allocations, this cap (enough for one clean run) would now be too small
        out = run_epoch(ctx, w, src, dst, X, y, Ws)
        compare(out, ref, w.n_layers)
        B.ht_ctx_set_hbm_budget(ctx, 0)
        compare(run_epoch(ctx, w, src, dst, X, y, Ws), ref, w.n_layers)
        with pytest.raises(B.HongtuError):
            B.ht_ctx_set_hbm_budget(ctx, -1)
    finally:
        B.ht_ctx_destroy(ctx)


def test_contexts_on_caller_streams(cfg1):
    """A context may run on a stream the caller owns; two contexts on two streams, used in turn, do not disturb each
    other (each has its own workspaces and scratch memory) and give the bits a lone context gives."""
    w, src, dst, X, y, Ws, ref = cfg1
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()        # default priority
    c1 = B.ht_ctx_create(0, hip_stream=s1.cuda_stream)
    c2 = B.ht_ctx_create(0, hip_stream=s2.cuda_stream)
    host = dict(x_loc=B.HT_LOC_HOST_PINNED, res_h=B.HT_RES_HOST, res_a=B.HT_RES_HOST, res_g=B.HT_RES_HOST)
    try:
        lone = run_epoch(c1, w, src, dst, X, y, Ws)
        compare(lone, ref, w.n_layers)
        g1 = B.ht_partition(c1, w.V, src.cuda(), dst.cuda(), w.n_chunks)
        g2 = B.ht_partition(c2, w.V, src.cuda(), dst.cuda(), 7)
        try:
            W1 = [x.clone().cuda() for x in Ws]
            W2 = [x.clone().cuda() for x in Ws]
            X1, X2 = B.to_matrix(X), B.to_matrix(X, B.HT_LOC_HOST_PINNED)
            yd = y.cuda()
            torch.cuda.synchronize()
            # enqueue on both without waiting in between (sync=False skips the binding's device-wide wait)
            l1, _ = B.ht_epoch(c1, g1, w.dims, W1, w.lr, X1, yd, sync=False)
            l2, _ = B.ht_epoch(c2, g2, w.dims, W2, w.lr, X2, yd, sync=False, res_h=B.HT_RES_HOST, res_a=B.HT_RES_HOST,
                               res_g=B.HT_RES_HOST)
            B.ht_sync(c1)
            B.ht_sync(c2)
            assert l1 == lone["loss"]
            assert abs(l2 - ref["loss"]) <= 1e-4 * abs(ref["loss"])
            for l in range(w.n_layers):
                assert np.array_equal(W1[l].cpu().numpy(), lone["W_new"][l])
                assert_close_grad(W2[l].cpu().numpy(), ref["W_new"][l], f"W^{l} on the second stream")
            with pytest.raises(B.HongtuError):      # a graph belongs to the context that made it
                B.ht_epoch(c2, g1, w.dims, W2, w.lr, X1, yd)
        finally:
            B.ht_graph_destroy(g1)
            B.ht_graph_destroy(g2)
        compare(run_epoch(c2, w, src, dst, X, y, Ws, **host), ref, w.n_layers)
    finally:
        B.ht_ctx_destroy(c1)
        B.ht_ctx_destroy(c2)

"""The allocation-free variant of the layer forward (ht_layer_fwd_static): two calls in a row through the C ABI, the
second on a smaller input, each compared bit for bit with ht_layer_fwd (same kernels, scratch in the library's static
array instead of allocated memory); HBM in use must not change across the calls; a layer beyond the array's size
is refused."""
import numpy as np
import pytest
import torch

from paper_2311_14898_amd import binding as B
from tests.util import hub_graph

pytestmark = pytest.mark.gpu


def _case(ctx, V, E, hub_in, d_in, d_out, n_chunks, seed):
    src, dst = hub_graph(V, E, hub_in, 50, seed)           # one destination with hub_in in-edges: rows cut into items
    g = B.ht_partition(ctx, V, src.cuda(), dst.cuda(), n_chunks)
    gen = torch.Generator().manual_seed(seed)
    H = B.to_matrix(torch.randn(V, d_in, generator=gen))
    W = (torch.randn(d_in, d_out, generator=gen) / np.sqrt(d_in)).cuda()
    return g, H, W


def _both(ctx, g, V, d_in, d_out, H, W):
    out_ref, a_ref = B.alloc_matrix(V, d_out), B.alloc_matrix(V, d_in)
    B.ht_layer_fwd(ctx, g, d_in, d_out, B.HT_ACT_RELU, H, W, out_ref, A_ckpt=a_ref)
    out, a = B.alloc_matrix(V, d_out), B.alloc_matrix(V, d_in)
    out.fill_(7.0)
    a.fill_(7.0)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    B.ht_layer_fwd_static(ctx, g, d_in, d_out, B.HT_ACT_RELU, H, W, out, a)
    B.ht_sync(ctx)
    assert torch.cuda.mem_get_info()[0] == free0, "device memory in use changed across the allocation-free call"
    assert torch.equal(a[:, :d_in], a_ref[:, :d_in]) and torch.equal(out[:, :d_out], out_ref[:, :d_out])
    assert float(out_ref[:, :d_out].abs().sum()) > 0


def test_static_scratch_layer_forward_matches_the_allocating_entry_point():
    ctx = B.ht_ctx_create(0)
    gs = []
    try:
        # first call: rows of up to 3000 in-edges (12 partial sums), 8 chunks
        g1, H1, W1 = _case(ctx, 6000, 60_000, 3000, 200, 96, 8, seed=1)
        gs.append(g1)
        _both(ctx, g1, 6000, 200, 96, H1, W1)
        # second call, smaller in every way: the array still holds the first call's packed weights and partial sums
        g2, H2, W2 = _case(ctx, 900, 5_000, 700, 40, 24, 3, seed=2)
        gs.append(g2)
        _both(ctx, g2, 900, 40, 24, H2, W2)
        # and the first again, after the smaller one
        _both(ctx, g1, 6000, 200, 96, H1, W1)
        # beyond the array: a 4096 x 2048 weight matrix packs to 32 MiB
        V = 64
        ids = torch.arange(0, V - 1, dtype=torch.int32, device="cuda")
        g3 = B.ht_partition(ctx, V, ids, ids + 1, 2)
        gs.append(g3)
        Hb, Wb = B.alloc_matrix(V, 4096), torch.zeros(4096, 2048, device="cuda")
        with pytest.raises(B.HongtuError) as err:
            B.ht_layer_fwd_static(ctx, g3, 4096, 2048, B.HT_ACT_NONE, Hb, Wb, B.alloc_matrix(V, 2048), B.alloc_matrix(V, 4096))
        assert err.value.code == B.HT_ENOMEM and "static array" in str(err.value)
        # tensors outside HBM are refused, not staged
        Hp = B.alloc_matrix(900, 40, B.HT_LOC_HOST_PINNED)
        with pytest.raises(B.HongtuError):
            B.ht_layer_fwd_static(ctx, g2, 40, 24, B.HT_ACT_RELU, Hp, W2, B.alloc_matrix(900, 24), B.alloc_matrix(900, 40))
    finally:
        for g in gs:
            B.ht_graph_destroy(g)
        B.ht_ctx_destroy(ctx)

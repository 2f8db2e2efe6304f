"""Pins of the GAT part of the CPU oracle (Eq. 3) against things other than itself: a dense
numpy statement of the same layer on tiny multigraphs, torch's autograd through that dense
statement, the closed form for zero attention parameters, and softmax invariants."""
import numpy as np
import torch

from oracle import oracle as orc


def tiny_graph(V, E, seed):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, V, E)
    dst = rng.integers(0, V, E)
    src[:4], dst[:4] = [1, 1, 2, 2], [0, 0, 0, 3]            # multi-edges
    keep = src != dst
    return src[keep].astype(np.int32), dst[keep].astype(np.int32)


def dense_gat(mult, H, W, a_dst, a_src, slope, relu):
    """The layer written on the dense multiplicity matrix mult[v, u] (torch, fp64, differentiable)."""
    t = H @ W
    y = (t @ a_dst)[:, None] + (t @ a_src)[None, :]                       # y[v, u]
    x = torch.where(y > 0, y, slope * y)
    x = x.masked_fill(mult == 0, -float("inf"))
    e = torch.exp(x - x.max(dim=1, keepdim=True).values) * mult           # a k-fold edge counts k times
    alpha = e / e.sum(dim=1, keepdim=True)
    z = alpha @ t
    return alpha, z, (torch.relu(z) if relu else z)


def case(V=23, E=90, d_in=7, d_out=5, seed=0):
    src, dst = tiny_graph(V, E, seed)
    indptr, col = orc.csc_build(V, src, dst, add_self_loops=True)
    rng = np.random.default_rng(seed + 100)
    H = rng.standard_normal((V, d_in))
    W = rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)
    a_dst, a_src = rng.standard_normal(d_out), rng.standard_normal(d_out)
    mult = np.zeros((V, V))
    for v in range(V):
        for e in range(indptr[v], indptr[v + 1]):
            mult[v, col[e]] += 1.0
    return indptr, col, H, W, a_dst, a_src, mult


def test_forward_equals_dense_statement():
    for seed, relu in ((0, True), (1, False), (2, True)):
        indptr, col, H, W, a_dst, a_src, mult = case(seed=seed)
        o = orc.gat_layer_fwd(indptr, col, H, W, a_dst, a_src, slope=0.2, relu=relu)
        tt = [torch.from_numpy(x) for x in (mult, H, W, a_dst, a_src)]
        alpha, z, h = dense_gat(*tt, 0.2, relu)
        np.testing.assert_allclose(o["z"], z.numpy(), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(o["h"], h.numpy(), rtol=1e-12, atol=1e-13)
        # per-edge coefficients: a k-fold edge holds k equal shares of the dense entry
        for v in range(len(indptr) - 1):
            for e in range(indptr[v], indptr[v + 1]):
                assert abs(o["alpha"][e] - alpha[v, col[e]].item() / mult[v, col[e]]) < 1e-13
        sums = np.add.reduceat(o["alpha"], indptr[:-1])
        np.testing.assert_allclose(sums, 1.0, rtol=1e-13)


def test_backward_equals_autograd_through_dense_statement():
    for seed, relu in ((3, True), (4, False)):
        indptr, col, H, W, a_dst, a_src, mult = case(seed=seed)
        rng = np.random.default_rng(seed)
        dh = rng.standard_normal((H.shape[0], W.shape[1]))
        f = orc.gat_layer_fwd(indptr, col, H, W, a_dst, a_src, relu=relu)
        if relu:
            assert np.abs(f["z"]).min() > 1e-9
        b = orc.gat_layer_bwd(indptr, col, H, W, a_dst, a_src, f, dh, relu=relu)
        Ht, Wt, adt, ast = [torch.from_numpy(x).clone().requires_grad_(True) for x in (H, W, a_dst, a_src)]
        _, _, h = dense_gat(torch.from_numpy(mult), Ht, Wt, adt, ast, 0.2, relu)
        (h * torch.from_numpy(dh)).sum().backward()
        np.testing.assert_allclose(b["dH"], Ht.grad.numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(b["dW"], Wt.grad.numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(b["da_dst"], adt.grad.numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(b["da_src"], ast.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_backward_matches_finite_differences():
    indptr, col, H, W, a_dst, a_src, _ = case(V=15, E=50, d_in=4, d_out=3, seed=7)
    rng = np.random.default_rng(11)
    dh = rng.standard_normal((15, 3))
    loss = lambda H_, W_, ad, as_: float((orc.gat_layer_fwd(indptr, col, H_, W_, ad, as_)["h"] * dh).sum())
    f = orc.gat_layer_fwd(indptr, col, H, W, a_dst, a_src)
    assert np.abs(f["z"]).min() > 1e-4        # no ReLU kink within the difference step
    b = orc.gat_layer_bwd(indptr, col, H, W, a_dst, a_src, f, dh)
    eps = 1e-6
    for name, arr, grad in (("H", H, b["dH"]), ("W", W, b["dW"]), ("a_dst", a_dst, b["da_dst"]), ("a_src", a_src, b["da_src"])):
        flat = arr.reshape(-1)
        for i in rng.choice(flat.size, size=min(8, flat.size), replace=False):
            old = flat[i]
            flat[i] = old + eps
            up = loss(H, W, a_dst, a_src)
            flat[i] = old - eps
            dn = loss(H, W, a_dst, a_src)
            flat[i] = old
            fd = (up - dn) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[i]) <= 1e-6 * max(1.0, abs(fd)), (name, i, fd, grad.reshape(-1)[i])


def test_zero_attention_parameters_give_the_neighbour_mean():
    # a = 0: every score is 0, alpha_e = 1 / in-degree, z_v = mean of t over v's stored in-edges
    indptr, col, H, W, _, _, mult = case(seed=5)
    zero = np.zeros(W.shape[1])
    o = orc.gat_layer_fwd(indptr, col, H, W, zero, zero, relu=False)
    t = H @ W
    np.testing.assert_allclose(o["z"], (mult @ t) / mult.sum(axis=1, keepdims=True), rtol=1e-12, atol=1e-13)


def test_softmax_invariances():
    indptr, col, H, W, a_dst, a_src, _ = case(seed=6)
    base = orc.gat_layer_fwd(indptr, col, H, W, a_dst, a_src, slope=1.0, relu=False)
    # with slope 1 the score is linear, so the destination's own term cancels in the softmax
    other = orc.gat_layer_fwd(indptr, col, H, W, 3.0 * a_dst + 1.0, a_src, slope=1.0, relu=False)
    np.testing.assert_allclose(base["alpha"], other["alpha"], rtol=1e-10, atol=1e-13)
    # huge scores do not overflow
    big = orc.gat_layer_fwd(indptr, col, 1e3 * H, W, a_dst, a_src, relu=False)
    assert np.isfinite(big["z"]).all()

"""ht_layer_fwd / ht_layer_bwd against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2311_14898_amd import binding as B
from paper_2311_14898_amd import inputs
from tests.util import assert_close, assert_close_grad, hub_graph, relu_margin

pytestmark = pytest.mark.gpu
DEV, HOST = B.HT_LOC_DEVICE, B.HT_LOC_HOST_PINNED


@pytest.fixture(scope="module")
def ctx():
    c = B.ht_ctx_create(0)
    yield c
    B.ht_ctx_destroy(c)


class Case:
    """A graph with its oracle CSC, kept for several tests."""

    def __init__(self, ctx, V, src, dst, n, **kw):
        self.V, self.n = V, n
        self.g = B.ht_partition(ctx, V, src.cuda(), dst.cuda(), n, **kw)
        self.indptr, self.col = orc.csc_build(V, src.numpy(), dst.numpy(), kw.get("add_self_loops", True))

    def close(self):
        B.ht_graph_destroy(self.g)


@pytest.fixture(scope="module")
def hub_case(ctx):
    V = 20_011
    src, dst = hub_graph(V, 150_000, hub_in=3000, hub_out=2500, seed=1)
    c = Case(ctx, V, src, dst, 5)
    yield c
    c.close()


@pytest.fixture(scope="module")
def rmat_case(ctx):
    V = 12_000
    src, dst = inputs.rmat_edges(V, 200_000, seed=4)
    c = Case(ctx, V, src, dst, 6)
    yield c
    c.close()


def _mat(x, loc):
    return B.to_matrix(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)), loc)


def _fwd(ctx, case, d_in, d_out, act, loc_in, loc_out, loc_a, gather, seed=0):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((case.V, d_in)).astype(np.float32)
    W = (rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)).astype(np.float32)
    H_in = _mat(H, loc_in)
    H_out = B.alloc_matrix(case.V, d_out, loc_out, zero=False)
    A = B.alloc_matrix(case.V, d_in, loc_a, zero=False) if loc_a is not None else None
    Wd = torch.from_numpy(W).cuda()
    B.ht_layer_fwd(ctx, case.g, d_in, d_out, act, H_in, Wd, H_out, A, gather_mode=gather)
    B.ht_sync(ctx)
    a_ref = orc.aggregate(case.indptr, case.col, H)
    z_ref = orc.matmul(a_ref, W)
    h_ref = np.maximum(z_ref, 0.0) if act == B.HT_ACT_RELU else z_ref
    if A is not None:
        assert_close(A.cpu().numpy()[:, :d_in], a_ref, "a")
    assert_close(H_out.cpu().numpy()[:, :d_out], h_ref, "h_out")


# widths chosen to hit every lane-group / vectors-per-lane variant of the aggregation
# and both column-tile variants of the dense transform, with ragged tails
@pytest.mark.parametrize("d_in,d_out", [(8, 8), (20, 41), (64, 32), (100, 256), (130, 64), (300, 130), (602, 256)])
def test_fwd_widths_direct(ctx, rmat_case, d_in, d_out):
    _fwd(ctx, rmat_case, d_in, d_out, B.HT_ACT_RELU, DEV, DEV, DEV, B.HT_GATHER_DIRECT, seed=d_in)


@pytest.mark.parametrize("loc_in,loc_out,loc_a,gather", [
    (DEV, DEV, None, B.HT_GATHER_AUTO),
    (DEV, DEV, DEV, B.HT_GATHER_BUFFER),
    (HOST, HOST, HOST, B.HT_GATHER_AUTO),
    (HOST, DEV, HOST, B.HT_GATHER_BUFFER),
    (DEV, HOST, DEV, B.HT_GATHER_DIRECT),
])
def test_fwd_residency_and_gather_modes(ctx, hub_case, loc_in, loc_out, loc_a, gather):
    _fwd(ctx, hub_case, 72, 41, B.HT_ACT_NONE, loc_in, loc_out, loc_a, gather, seed=5)


@pytest.mark.parametrize("d_in,d_out,act", [(64, 32, B.HT_ACT_RELU), (602, 256, B.HT_ACT_RELU), (256, 41, B.HT_ACT_NONE),
                                            (20, 130, B.HT_ACT_RELU)])
def test_fwd_update_first(ctx, rmat_case, hub_case, d_in, d_out, act):
    # t = H W first, then the aggregation at width d_out with the activation fused into its last write
    for case in (rmat_case, hub_case):
        rng = np.random.default_rng(d_in + d_out)
        H = rng.standard_normal((case.V, d_in)).astype(np.float32)
        W = (rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)).astype(np.float32)
        H_out = B.alloc_matrix(case.V, d_out, DEV, zero=False)
        B.ht_layer_fwd(ctx, case.g, d_in, d_out, act, _mat(H, DEV), torch.from_numpy(W).cuda(), H_out,
                       order=B.HT_ORDER_UPDATE_FIRST)
        B.ht_sync(ctx)
        z_ref = orc.matmul(orc.aggregate(case.indptr, case.col, H), W)
        assert_close(H_out.cpu().numpy()[:, :d_out], np.maximum(z_ref, 0.0) if act == B.HT_ACT_RELU else z_ref, "h_out")


def test_update_first_needs_hbm(ctx, rmat_case):
    c = rmat_case
    H = B.alloc_matrix(c.V, 16, HOST)
    W = torch.zeros(16, 8, device="cuda")
    with pytest.raises(B.HongtuError):
        B.ht_layer_fwd(ctx, c.g, 16, 8, B.HT_ACT_NONE, H, W, B.alloc_matrix(c.V, 8, DEV), order=B.HT_ORDER_UPDATE_FIRST)
    with pytest.raises(B.HongtuError):
        B.ht_layer_fwd(ctx, c.g, 16, 8, B.HT_ACT_NONE, B.alloc_matrix(c.V, 16, DEV), W, B.alloc_matrix(c.V, 8, DEV), order=5)


def test_fwd_hub_rows_wide(ctx, hub_case):
    _fwd(ctx, hub_case, 256, 256, B.HT_ACT_RELU, DEV, DEV, DEV, B.HT_GATHER_DIRECT, seed=6)
    _fwd(ctx, hub_case, 602, 64, B.HT_ACT_RELU, DEV, DEV, DEV, B.HT_GATHER_BUFFER, seed=7)


def test_fwd_all_ones_gives_normalised_degree_sums(ctx, rmat_case):
    c = rmat_case
    d = 16
    H_in = _mat(np.ones((c.V, d)), DEV)
    W = torch.eye(d, dtype=torch.float32).cuda()
    H_out = B.alloc_matrix(c.V, d)
    B.ht_layer_fwd(ctx, c.g, d, d, B.HT_ACT_NONE, H_in, W, H_out)
    B.ht_sync(ctx)
    s = orc.norm(c.indptr)
    ref = np.array([s[v] * s[c.col[c.indptr[v]:c.indptr[v + 1]]].sum() for v in range(c.V)])
    assert_close(H_out.cpu().numpy()[:, :d], np.repeat(ref[:, None], d, axis=1), "degree sums")


def test_fwd_deterministic(ctx, hub_case):
    c = hub_case
    rng = np.random.default_rng(2)
    H_in = _mat(rng.standard_normal((c.V, 100)), DEV)
    W = torch.from_numpy(rng.standard_normal((100, 47)).astype(np.float32)).cuda()
    outs = []
    for _ in range(2):
        H_out = B.alloc_matrix(c.V, 47)
        A = B.alloc_matrix(c.V, 100)
        B.ht_layer_fwd(ctx, c.g, 100, 47, B.HT_ACT_RELU, H_in, W, H_out, A)
        B.ht_sync(ctx)
        outs.append((H_out[:, :47].clone(), A[:, :100].clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


def _bwd_ref(case, a, W, dh, relu):
    z = orc.matmul(a, W)
    dz = np.where(z > 0.0, dh, 0.0) if relu else np.asarray(dh, dtype=np.float64)
    dW = orc.matmul_tn(a, dz)
    da = orc.matmul_nt(dz, W)
    dhin = orc.aggregate_T(case.indptr, case.col, da)
    return z, dW, da, dhin


def _bwd_inputs(case, d_in, d_out, ckpt_input, structured, seed):
    """Checkpoint, W and dH_out.  With structured=True every pre-activation z = aW is far
    from 0 (sign(z[v,c]) = r_v * q_c by construction), so the fp32 path and the fp64 oracle
    take the same ReLU decisions; with structured=False the inputs are plain N(0,1)."""
    rng = np.random.default_rng(seed)
    dh = rng.standard_normal((case.V, d_out)).astype(np.float32)
    if not structured:
        W = (rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)).astype(np.float32)
        ck = rng.standard_normal((case.V, d_in)).astype(np.float32)
        return ck, W, dh
    q = rng.choice([-1.0, 1.0], size=d_out)
    W = (q[None, :] * (np.abs(rng.standard_normal((d_in, d_out))) + 0.25) / np.sqrt(d_in)).astype(np.float32)
    ck = np.abs(rng.standard_normal((case.V, d_in))) + 0.25
    if not ckpt_input:                      # the checkpoint is a^l itself: give rows a sign too
        ck = rng.choice([-1.0, 1.0], size=case.V)[:, None] * ck
    return ck.astype(np.float32), W, dh


def _bwd(ctx, case, d_in, d_out, relu, loc, gather, mask_from_h, ckpt_input=False, want_dhin=True, seed=0,
         structured=True, order=B.HT_ORDER_AGG_FIRST):
    ck_np, W, dh = _bwd_inputs(case, d_in, d_out, ckpt_input, structured and relu, seed)
    a = orc.aggregate(case.indptr, case.col, ck_np) if ckpt_input else ck_np
    ck = _mat(ck_np, loc)
    z, dW_ref, da_ref, dhin_ref = _bwd_ref(case, a, W, dh, relu)
    if relu:
        # both sides must take the same ReLU decisions: pre-activations stay clear of fp32 rounding
        assert relu_margin(z) > (1e-3 if structured else 1e-7), "pre-activation too close to 0 for this seed"
    Wd = torch.from_numpy(W).cuda()
    dH_out = _mat(dh, loc)
    H_out = _mat(np.maximum(z, 0.0), loc) if (mask_from_h and relu) else None
    dW = torch.empty(d_in, d_out, dtype=torch.float32, device="cuda")
    dH_in = B.alloc_matrix(case.V, d_in, loc) if want_dhin else None
    B.ht_layer_bwd(ctx, case.g, d_in, d_out, B.HT_ACT_RELU if relu else B.HT_ACT_NONE, ck, Wd, dH_out, dW,
                   dH_in=dH_in, H_out=H_out, ckpt_kind=B.HT_CKPT_INPUT if ckpt_input else B.HT_CKPT_AGG,
                   gather_mode=gather, order=order)
    B.ht_sync(ctx)
    assert_close_grad(dW.cpu().numpy(), dW_ref, "dW")
    if want_dhin:
        assert_close_grad(dH_in.cpu().numpy()[:, :d_in], dhin_ref, "dH_in")


@pytest.mark.parametrize("d_in,d_out", [(8, 8), (64, 32), (100, 41), (256, 256), (602, 130)])
def test_bwd_widths(ctx, rmat_case, d_in, d_out):
    _bwd(ctx, rmat_case, d_in, d_out, True, DEV, B.HT_GATHER_DIRECT, mask_from_h=False, seed=10 + d_in)


@pytest.mark.parametrize("d_in,d_out,seed", [(8, 8, 1), (64, 32, 2)])
def test_bwd_gaussian_inputs(ctx, rmat_case, d_in, d_out, seed):
    _bwd(ctx, rmat_case, d_in, d_out, True, DEV, B.HT_GATHER_DIRECT, mask_from_h=False, seed=seed, structured=False)


@pytest.mark.parametrize("loc,gather,mask_from_h,ckpt_input", [
    (DEV, B.HT_GATHER_DIRECT, True, False),
    (DEV, B.HT_GATHER_BUFFER, False, False),      # in-place gradient buffer, rows leave by a GPU add
    (HOST, B.HT_GATHER_AUTO, False, False),       # host-resident: D2H compaction + CPU accumulation
    (HOST, B.HT_GATHER_AUTO, True, False),
    (DEV, B.HT_GATHER_DIRECT, False, True),       # pure recomputation: aggregate again from h^l
    (HOST, B.HT_GATHER_AUTO, False, True),
])
def test_bwd_residency_modes(ctx, hub_case, loc, gather, mask_from_h, ckpt_input):
    _bwd(ctx, hub_case, 72, 40, True, loc, gather, mask_from_h, ckpt_input, seed=21)


@pytest.mark.parametrize("d_in,d_out,relu,want_dhin", [(64, 32, True, True), (256, 41, False, True), (602, 256, True, False),
                                                       (72, 130, True, True)])
def test_bwd_update_first(ctx, rmat_case, hub_case, d_in, d_out, relu, want_dhin):
    # the checkpoint is the layer input h^l; dt = A_hat^T dz at width d_out, dW = h^T dt, dH_in = dt W^T
    for case in (rmat_case, hub_case):
        _bwd(ctx, case, d_in, d_out, relu, DEV, B.HT_GATHER_AUTO, mask_from_h=True, ckpt_input=True,
             want_dhin=want_dhin, seed=40 + d_in, order=B.HT_ORDER_UPDATE_FIRST)


def test_bwd_no_activation_no_input_gradient(ctx, rmat_case):
    _bwd(ctx, rmat_case, 32, 8, False, DEV, B.HT_GATHER_AUTO, mask_from_h=False, want_dhin=False, seed=3)


def test_bwd_mask_and_recompute_agree_bitwise(ctx, rmat_case):
    # Sec. 4.2: the regenerated intermediate data are identical
    c = rmat_case
    rng = np.random.default_rng(8)
    d_in, d_out = 64, 48
    a = _mat(rng.standard_normal((c.V, d_in)), DEV)
    W = torch.from_numpy((rng.standard_normal((d_in, d_out)) / 8).astype(np.float32)).cuda()
    dh = _mat(rng.standard_normal((c.V, d_out)), DEV)
    H_out = B.alloc_matrix(c.V, d_out)
    res = []
    for use_mask in (False, True):
        dW = torch.empty(d_in, d_out, device="cuda")
        dH_in = B.alloc_matrix(c.V, d_in)
        if use_mask:
            z = (a[:, :d_in].double() @ W.double())
            H_out[:, :d_out] = torch.clamp(z, min=0).float()
        B.ht_layer_bwd(ctx, c.g, d_in, d_out, B.HT_ACT_RELU, a, W, dh, dW, dH_in=dH_in,
                       H_out=H_out if use_mask else None)
        B.ht_sync(ctx)
        res.append((dW.clone(), dH_in.clone()))
    zmin = (a[:, :d_in].double() @ W.double()).abs().min().item()
    assert zmin > 1e-6
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1][:, :d_in], res[1][1][:, :d_in])


def test_shape_errors(ctx, rmat_case):
    c = rmat_case
    H = B.alloc_matrix(c.V, 16)
    W = torch.zeros(16, 8, device="cuda")
    out = B.alloc_matrix(c.V, 8)
    bad = torch.zeros(c.V - 1, 16, device="cuda")
    with pytest.raises(B.HongtuError) as e:
        B.ht_layer_fwd(ctx, c.g, 16, 8, 0, bad, W, out)
    assert e.value.code == B.HT_ESHAPE
    odd = torch.zeros(c.V, 18, device="cuda")[:, :17]          # pitch 18: not a multiple of 4
    with pytest.raises(B.HongtuError):
        B.ht_layer_fwd(ctx, c.g, 16, 8, 0, odd, W, out)
    Hh = B.alloc_matrix(c.V, 16, HOST)
    with pytest.raises(B.HongtuError):
        B.ht_layer_fwd(ctx, c.g, 16, 8, 0, Hh, W, out, gather_mode=B.HT_GATHER_DIRECT)

"""CPU pins of the test-side helpers that turn undecidable activation decisions into intervals
(tests/gat_ties.py, tests/util.py): they are checked against the oracle's own backward pass, which is linear in the
slope that the non-positive scores get."""
import numpy as np

from oracle import oracle as orc
from tests import gat_ties
from tests.test_oracle_gat_pins import case
from tests.util import assert_close, assert_in_interval, row_errors


def test_edge_flip_slack_is_the_change_of_the_oracle_backward():
    # Same forward result, two slopes in the backward pass: only the edges with y_e <= 0 change, each dy_e by
    # dx_e (s2 - s1).  The helper's per-edge terms, summed, must give exactly the difference of the two oracle runs.
    indptr, col, H, W, a_dst, a_src, _ = case(seed=8)
    V = len(indptr) - 1
    rng = np.random.default_rng(2)
    dh = rng.standard_normal((V, W.shape[1]))
    f = orc.gat_layer_fwd(indptr, col, H, W, a_dst, a_src, slope=0.2)
    b1 = orc.gat_layer_bwd(indptr, col, H, W, a_dst, a_src, f, dh, slope=0.2)
    b2 = orc.gat_layer_bwd(indptr, col, H, W, a_dst, a_src, f, dh, slope=0.7)
    dst_of = np.repeat(np.arange(V), np.diff(indptr))
    y = (f["t"] @ a_dst)[dst_of] + (f["t"] @ a_src)[col]
    e = np.nonzero(y <= 0)[0]
    assert 0 < len(e) < len(y)
    dz = np.where(f["z"] > 0, dh, 0.0)
    dx = gat_ties.edge_dx(dst_of[e], col[e], f["alpha"][e], f["t"], f["z"], dz)
    sl = gat_ties.edge_flip_slack(dst_of[e], col[e], dx * (0.7 - 0.2), H, W, a_dst, a_src, f["t"])
    for k in ("dW", "da_dst", "da_src"):
        lo, hi = sl[k]
        assert (lo <= 0).all() and (hi >= 0).all()
        np.testing.assert_allclose(lo + hi, b2[k] - b1[k], rtol=1e-10, atol=1e-12)
    rows, lo, hi = sl["dH"]
    full = np.zeros_like(b1["dH"])
    full[rows] = lo + hi
    np.testing.assert_allclose(full, b2["dH"] - b1["dH"], rtol=1e-10, atol=1e-12)


def test_interval_and_row_checks_catch_what_they_should():
    rng = np.random.default_rng(0)
    ref = rng.standard_normal((50, 8))
    ref[7] *= 1e-3                                   # a low-magnitude row beside ordinary ones
    x = ref.copy()
    x[7] = -ref[7]                                   # wholly wrong, yet invisible to the per-tensor norms
    assert np.abs(x - ref).max() / np.abs(ref).max() < 2e-3
    assert row_errors(x, ref)[1] == 7 and row_errors(x, ref)[0] > 1.0
    try:
        assert_close(x, ref, "planted", tol=1e-2)
    except AssertionError as err:
        assert "row 7" in str(err)
    else:
        raise AssertionError("the per-row bound did not fire")
    # inside the slack: accepted; outside by more than the tolerance: refused
    lo, hi = np.zeros_like(ref), np.zeros_like(ref)
    hi[3, 2], lo[4, 1] = 0.5, -0.25
    y = ref.copy()
    y[3, 2] += 0.4
    y[4, 1] -= 0.25
    assert_in_interval(y, ref, lo, hi, "inside")
    y[3, 2] += 0.2
    try:
        assert_in_interval(y, ref, lo, hi, "outside")
    except AssertionError:
        pass
    else:
        raise AssertionError("a value outside the interval passed")


def test_relu_tie_slack_contains_every_flip():
    # A huge rounding factor makes many pre-activations "ties".  Flipping ReLU's derivative on any subset of them, in
    # a numpy restatement of the backward pass built on the oracle's forward values, must keep every weight gradient
    # inside the helper's interval; and flipping all of them at once must leave the interval's interior somewhere.
    from tests.util import relu_tie_slack
    rng = np.random.default_rng(0)
    V, E, dims = 300, 3000, [12, 10, 9, 5]
    src, dst = rng.integers(0, V, E).astype(np.int32), rng.integers(0, V, E).astype(np.int32)
    indptr, col = orc.csc_build(V, src, dst)
    X = rng.standard_normal((V, dims[0])).astype(np.float32)
    Ws = [(rng.standard_normal((dims[l], dims[l + 1])) / 3).astype(np.float32) for l in range(3)]
    y = rng.integers(0, 5, V).astype(np.int32)
    ref = orc.gcn_epoch(indptr, col, dims, X, Ws, y, want=("a", "z", "gh"))
    sl = relu_tie_slack(ref, indptr, col, Ws, dims, factor=3e5)
    assert all(len(sl[l][2][0]) > 20 for l in range(2)) and len(sl[2][2][0]) == 0

    def backward(masks):
        gh = ref["gh"][2]
        gW = [None] * 3
        for l in (2, 1, 0):
            dz = gh if l == 2 else gh * masks[l]
            gW[l] = ref["a"][l].T @ dz
            if l > 0:
                gh = orc.aggregate_T(indptr, col, dz @ Ws[l].astype(np.float64).T)
        return gW

    base_masks = [ref["z"][l] > 0 for l in range(2)]
    base = backward(base_masks)
    for l in range(3):
        np.testing.assert_allclose(base[l], ref["gW"][l], rtol=1e-9, atol=1e-12)
    moved = False
    for trial in range(6):
        masks = [m.copy() for m in base_masks]
        for l in range(2):
            tv, tc = sl[l][2]
            pick = np.ones(len(tv), bool) if trial == 0 else rng.random(len(tv)) < 0.5
            masks[l][tv[pick], tc[pick]] ^= True
        got = backward(masks)
        for l in range(3):
            lo, hi, _ = sl[l]
            err = got[l] - ref["gW"][l]
            assert (err >= lo - 1e-12).all() and (err <= hi + 1e-12).all(), (trial, l)
            moved |= bool((np.abs(err) > 1e-9).any())
    assert moved

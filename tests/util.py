"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

# Tolerance of the fp32 path against the fp64 oracle, per tensor:
#   max|x - ref| / max|ref| <= TOL   and   ||x - ref||_F / ||ref||_F <= TOL
TOL = 1e-4


def rel_errors(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0
    assert np.isfinite(x).all(), "non-finite values in the GPU result"
    dmax = np.abs(x - ref).max()
    rmax = np.abs(ref).max()
    dfro = np.linalg.norm((x - ref).ravel())
    rfro = np.linalg.norm(ref.ravel())
    return (dmax / rmax if rmax > 0 else dmax), (dfro / rfro if rfro > 0 else dfro)


ROW_FLOOR = 1e-3
# Gradient tensors hold rows that are small by cancellation: grad h^l[u] sums signed terms over u's out-edges, ReLU
# masks most of a row away, and in a GAT layer the softmax's backward gives sum_e alpha_e (d alpha_e - S_v) = 0 exactly
# for a destination whose scores all take the same LeakyReLU slope.  fp32 rounds relative to the terms, not to their
# sum, so such a row carries an error of a few eps of a typical row, which no bound relative to the row's own norm
# admits (seen: up to 6e-7 of the median row norm, on rows 1e-3 .. 1e-9 of it).  For gradients the floor is a tenth
# of the median row norm: every row must still be right to 1e-5 of a typical row, so a row that lost a partial sum
# or was never written fails unless it is itself below that.
GRAD_ROW_FLOOR = 1e-1


def row_errors(x, ref, row_floor=ROW_FLOOR):
    """Per-row check for 2-D tensors: every row v must satisfy
    ||x_v - ref_v||_2 <= TOL * max(||ref_v||_2, row_floor * median_v ||ref_v||_2)
    (the floor keeps rows that are zero, or nearly so, from demanding exact zeros' worth of precision; the median is
    taken over the rows that are not exactly zero).  Returns (worst ratio error/allowance-per-TOL, its row)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.ndim != 2 or ref.shape[0] == 0:
        return 0.0, -1
    rn = np.sqrt((ref * ref).sum(axis=1))
    en = np.sqrt(((x - ref) ** 2).sum(axis=1))
    nz = rn[rn > 0]
    floor = row_floor * (np.median(nz) if nz.size else 0.0)
    allow = np.maximum(rn, floor)
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(allow > 0, en / allow, np.where(en > 0, np.inf, 0.0))
    v = int(np.argmax(ratio))
    return float(ratio[v]), v


def assert_close(x, ref, name="", tol=TOL, rows=True, row_floor=ROW_FLOOR):
    emax, efro = rel_errors(x, ref)
    assert emax <= tol and efro <= tol, f"{name}: max-norm rel err {emax:.3e}, Frobenius rel err {efro:.3e} > {tol}"
    if rows:
        erow, v = row_errors(x, ref, row_floor)
        assert erow <= tol, (f"{name}: row {v} is off by {erow:.3e} of its own norm (allowed {tol}); "
                             f"||ref_v|| = {np.linalg.norm(np.asarray(ref, dtype=np.float64)[v]):.3e}")
    return emax, efro


def assert_close_grad(x, ref, name="", tol=TOL):
    """assert_close for gradient tensors (see GRAD_ROW_FLOOR)."""
    return assert_close(x, ref, name, tol, row_floor=GRAD_ROW_FLOOR)


def assert_in_interval(x, base, lo_slack, hi_slack, name="", tol=TOL, row_floor=GRAD_ROW_FLOOR):
    """x must lie in [base + lo_slack, base + hi_slack] (lo_slack <= 0 <= hi_slack, element-wise: what the
    undecidable decisions can move) widened by the per-tensor tolerances of assert_close: the part of x - base
    outside the slack is held to the max-norm and Frobenius bounds, and row by row to the per-row bound."""
    x = np.asarray(x, dtype=np.float64)
    base = np.asarray(base, dtype=np.float64)
    assert x.shape == base.shape and np.isfinite(x).all()
    assert (np.asarray(lo_slack) <= 0).all() and (np.asarray(hi_slack) >= 0).all()
    err = x - base
    excess = np.maximum(err - hi_slack, 0.0) + np.minimum(err - lo_slack, 0.0)   # distance to the interval, signed
    return assert_close(base + excess, base, name, tol, row_floor=row_floor)


def relu_margin(z, rel=1e-6):
    """Smallest |z| relative to max|z|: the ReLU decision is safe in fp32 when this is well above rounding."""
    z = np.asarray(z)
    return np.abs(z).min() / max(np.abs(z).max(), 1e-300)


def hub_graph(V, E, hub_in, hub_out, seed):
    """Random graph plus one destination with hub_in in-edges and one source with hub_out out-edges."""
    rng = np.random.default_rng(seed)
    src = rng.integers(0, V, size=E)
    dst = rng.integers(0, V, size=E)
    hs = rng.integers(0, V, size=hub_in)
    hd = rng.integers(0, V, size=hub_out)
    src = np.concatenate([src, hs, np.full(hub_out, 5)])
    dst = np.concatenate([dst, np.full(hub_in, 3), hd])
    keep = src != dst
    return torch.from_numpy(src[keep].astype(np.int32)), torch.from_numpy(dst[keep].astype(np.int32))


from oracle.ties import relu_tie_slack  # noqa: E402,F401  (the interval helper lives beside the oracle: bench.py's parity leg uses it too)

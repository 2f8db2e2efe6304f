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


def assert_close(x, ref, name="", tol=TOL):
    emax, efro = rel_errors(x, ref)
    assert emax <= tol and efro <= tol, f"{name}: max-norm rel err {emax:.3e}, Frobenius rel err {efro:.3e} > {tol}"
    return emax, efro


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

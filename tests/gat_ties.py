"""What an undecidable LeakyReLU decision can move in the backward pass of a GAT layer (Eq. 3).

Test code, numpy only, fed with the oracle's fp64 values and the seeded inputs: nothing here comes from the
kernels.  An fp32 implementation and the fp64 oracle may take different sides of LeakyReLU's kink for an edge
whose score y_e lies within fp32 rounding of 0 (a "tie"); either side is right.  The backward pass is linear in the
per-edge slope f_e in {1, slope}: dy_e = dx_e f_e with dx_e = alpha_e dz_v . (t_u - z_v), and from dy_e on
everything is sums.  So flipping the decision of edge e = (u -> v) adds D_e = +-dx_e (1 - slope) to dy_e and hence
  D_e t_v to da_dst,  D_e t_u to da_src,  D_e a_dst to dt_v,  D_e a_src to dt_u,
  D_e (H_v (x) a_dst + H_u (x) a_src) to dW,   D_e W a_dst to dH_v,   D_e W a_src to dH_u.
For every output the reference becomes base + [lo, hi], lo / hi = the sums of the negative / positive parts of
these terms over the ties (for dW the two outer products of a tie are bounded separately: a superset).
"""
import numpy as np

EPS32 = 2.0 ** -24


def score_halves_error(H, W, a, t, sigmas=8.0):
    """Bound on the fp32 rounding error of p_v = a . t_v with t = H W accumulated in fp32 (random-walk model,
    `sigmas` standard deviations): per vertex."""
    H, W, a, t = (np.asarray(x, dtype=np.float64) for x in (H, W, a, t))
    e_t = EPS32 * np.sqrt(H.shape[1]) * np.sqrt((H * H) @ (W * W))          # [V x d_out]
    return sigmas * (np.sqrt(((a * e_t) ** 2).sum(axis=1)) + EPS32 * np.sqrt(len(a)) * np.sqrt(((a * t) ** 2).sum(axis=1)))


def edge_flip_slack(edges_v, edges_u, delta, H, W, a_dst, a_src, t):
    """Slack of every backward output for decisions that may flip on the edges (u -> v) given by edges_v, edges_u,
    each flip adding delta[e] to dy_e.  Returns {"dW": (lo, hi), "da_dst": ..., "da_src": ..., "dH": (rows, lo, hi)}
    where dH's slack is given for the listed rows only (all other rows: none)."""
    H, W, a_dst, a_src, t = (np.asarray(x, dtype=np.float64) for x in (H, W, a_dst, a_src, t))
    v, u, D = np.asarray(edges_v, dtype=np.int64), np.asarray(edges_u, dtype=np.int64), np.asarray(delta, dtype=np.float64)
    pos, neg = (lambda x: np.maximum(x, 0.0)), (lambda x: np.minimum(x, 0.0))
    out = {}
    for key, rows in (("da_dst", v), ("da_src", u)):
        c = D[:, None] * t[rows]
        out[key] = (neg(c).sum(axis=0), pos(c).sum(axis=0))
    lo = np.zeros((H.shape[1], W.shape[1]))
    hi = np.zeros_like(lo)
    for rows, a in ((v, a_dst), (u, a_src)):
        c = D[:, None] * H[rows]
        P, N = pos(c).sum(axis=0), neg(c).sum(axis=0)
        hi += np.outer(P, pos(a)) + np.outer(N, neg(a))
        lo += np.outer(N, pos(a)) + np.outer(P, neg(a))
    out["dW"] = (lo, hi)
    rows = np.unique(np.concatenate([v, u]))
    lo = np.zeros((len(rows), H.shape[1]))
    hi = np.zeros_like(lo)
    for r, wa in ((v, W @ a_dst), (u, W @ a_src)):
        c = D[:, None] * wa[None, :]
        idx = np.searchsorted(rows, r)
        np.add.at(hi, idx, pos(c))
        np.add.at(lo, idx, neg(c))
    out["dH"] = (rows, lo, hi)
    return out


def edge_dx(edges_v, edges_u, alpha_e, t, z, dz):
    """dx_e = alpha_e dz_v . (t_u - z_v): the gradient that reaches LeakyReLU's output on edge e (the softmax's
    backward with sum_e' alpha_e' (dz_v . t_u') = dz_v . z_v)."""
    v, u = np.asarray(edges_v, dtype=np.int64), np.asarray(edges_u, dtype=np.int64)
    return np.asarray(alpha_e, dtype=np.float64) * np.einsum("ek,ek->e", dz[v], t[u] - z[v])

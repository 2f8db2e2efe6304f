"""Intervals for the decisions fp32 cannot take: which ReLU derivatives of a GCN epoch are undecidable, and how far the
weight gradients can move with them.  TEST INFRASTRUCTURE like the rest of oracle/: used by tests/ and by the parity leg of
bench.py; computed from the oracle's own fp64 values, never from kernel output.  Pinned in tests/test_tie_helpers.py (every
subset of flipped decisions, applied in a numpy restatement of the backward pass, stays inside the interval)."""
import numpy as np

from . import oracle as orc


def relu_tie_slack(ref, indptr, col, Ws, dims, factor=16.0):
    """How far the weight gradients of a GCN epoch can move when ReLU's derivative is taken on the other side for
    the pre-activations that fp32 cannot tell from 0.  Everything comes from the oracle's own epoch `ref`
    (orc.gcn_epoch with want = a, z, gh) and the seeded weights; no kernel output enters.

    An element z^l[v, c] is a tie when |z| <= factor * eps32 sqrt(d_l) sqrt(sum_k a_vk^2 W_kc^2), a random-walk bound on
    the fp32 rounding of the aggregate and the product (on the 232,965 x 602 x 256 layer the fp32 path's largest error is 5.2
    of these units, and the decisions that differ from fp64's all lie below 0.3 units; 16 leaves a factor 3).  Taking the other side changes dz^l[v, c] by d = gh^{l+1}[v, c], hence
      grad W^l[:, c]   by  a^l[v, :] d                                        (signed: an interval), and, one layer down,
      grad W^{l-1}     by at most |d| * (A_hat |a^{l-1}|)[v, :] (x) |W^l[:, c]|   (through grad a^l, grad h^l, the mask).
    Returns per layer (lo, hi, ties) with ties = (rows, columns) of that layer's undecidable elements.  Deeper propagation (two layers down) does not occur for L <= 3."""
    L = len(dims) - 1
    assert L <= 3
    eps32 = 2.0 ** -24
    out = [[np.zeros((dims[l], dims[l + 1])), np.zeros((dims[l], dims[l + 1])), (np.zeros(0, np.int64), np.zeros(0, np.int64))] for l in range(L)]
    for l in range(L - 1):                                    # the last layer has no activation
        a, z, gh = ref["a"][l], ref["z"][l], ref["gh"][l]
        W = np.asarray(Ws[l], dtype=np.float64)
        zerr = factor * eps32 * np.sqrt(dims[l]) * np.sqrt((a * a) @ (W * W))
        tv, tc = np.nonzero(np.abs(z) <= zerr)
        out[l][2] = (tv, tc)
        if len(tv) == 0:
            continue
        d = gh[tv, tc]
        # the oracle counted the element iff z > 0: the other side removes (z > 0) or adds (z <= 0) a_v d
        contrib = a[tv] * np.where(z[tv, tc] > 0, -d, d)[:, None]          # [ties x d_l], goes to column tc
        np.add.at(out[l][1].T, tc, np.maximum(contrib, 0.0))
        np.add.at(out[l][0].T, tc, np.minimum(contrib, 0.0))
        if l > 0:
            agg_abs = orc.aggregate(indptr, col, np.abs(ref["a"][l - 1]))[tv]         # [ties x d_{l-1}]
            bound = (np.abs(d)[:, None] * agg_abs).T @ np.abs(W[:, tc]).T             # [d_{l-1} x d_l]
            out[l - 1][1] += bound
            out[l - 1][0] -= bound
    return [tuple(x) for x in out]

"""numpy front end of the CPU oracle (oracle/gcn_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing in the product package imports it, and
it imports nothing from the product package.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.orc_csc_build.restype = C.c_int64
        _lib.orc_chunk_nsrc.restype = C.c_int64
        _lib.orc_softmax_ce.restype = C.c_double
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=np.int32)


def _i64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=np.int64)


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=np.float64)


def csc_build(V: int, src, dst, add_self_loops: bool = True) -> Tuple[np.ndarray, np.ndarray]:
    src, dst = _i32(src), _i32(dst)
    E = src.shape[0]
    indptr = np.zeros(V + 1, dtype=np.int64)
    col = np.zeros(E + (V if add_self_loops else 0), dtype=np.int32)
    Ep = lib().orc_csc_build(C.c_int64(V), C.c_int64(E), _p(src), _p(dst), C.c_int(int(add_self_loops)),
                             _p(indptr), _p(col))
    assert Ep == col.shape[0]
    return indptr, col


def chunk_bounds(indptr: np.ndarray, n: int, mode: int = 0) -> np.ndarray:
    V = indptr.shape[0] - 1
    b = np.zeros(n + 1, dtype=np.int64)
    lib().orc_chunk_bounds(C.c_int64(V), _p(indptr), C.c_int(n), C.c_int(mode), _p(b))
    return b


def chunk_dedup(indptr: np.ndarray, col: np.ndarray, b0: int, b1: int) -> Dict[str, np.ndarray]:
    ns = lib().orc_chunk_nsrc(_p(indptr), _p(col), C.c_int64(b0), C.c_int64(b1))
    ne = int(indptr[b1] - indptr[b0])
    N = np.zeros(ns, dtype=np.int32)
    cl = np.zeros(ne, dtype=np.int32)
    sptr = np.zeros(ns + 1, dtype=np.int64)
    sdst = np.zeros(ne, dtype=np.int32)
    lib().orc_chunk_dedup(_p(indptr), _p(col), C.c_int64(b0), C.c_int64(b1), _p(N), _p(cl), _p(sptr), _p(sdst))
    return {"N": N, "col_local": cl, "sptr": sptr, "sdst": sdst}


def reuse_split(prev, cur) -> Tuple[np.ndarray, np.ndarray]:
    prev, cur = _i32(prev), _i32(cur)
    R = np.zeros(cur.shape[0], dtype=np.int32)
    Ld = np.zeros(cur.shape[0], dtype=np.int32)
    nR, nLd = C.c_int64(0), C.c_int64(0)
    lib().orc_reuse_split(_p(prev), C.c_int64(prev.shape[0]), _p(cur), C.c_int64(cur.shape[0]), _p(R), _p(Ld),
                          C.byref(nR), C.byref(nLd))
    return R[: nR.value].copy(), Ld[: nLd.value].copy()


def volumes(indptr: np.ndarray, col: np.ndarray, b: np.ndarray) -> Tuple[int, int]:
    V = indptr.shape[0] - 1
    b = _i64(b)
    vo, vr = C.c_int64(0), C.c_int64(0)
    lib().orc_volumes(C.c_int64(V), _p(indptr), _p(col), C.c_int(b.shape[0] - 1), _p(b), C.byref(vo), C.byref(vr))
    return vo.value, vr.value


def chunk_order(indptr: np.ndarray, col: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Greedy schedule order of the chunks (Alg. 4, phase 2, one GPU): order[j] = chunk id at position j."""
    b = _i64(b)
    n = b.shape[0] - 1
    order = np.zeros(n, dtype=np.int32)
    lib().orc_chunk_order(_p(indptr), _p(col), C.c_int(n), _p(b), _p(order))
    return order


def volumes_mn(indptr, col, b, m: int, n: int, layout=None) -> Tuple[int, int, int]:
    """(V_ori, V_+p2p, V_+ru) of Sec. 5.3 for m partitions of n subgraphs; b has m*n+1 boundaries; layout[i*n+j] =
    subgraph of partition i in batch j (default: subgraph j)."""
    indptr, col, b = _i64(indptr), _i32(col), _i64(b)
    assert len(b) == m * n + 1
    lay = _i32(np.tile(np.arange(n), m) if layout is None else layout)
    assert len(lay) == m * n
    out = np.zeros(3, dtype=np.int64)
    lib().orc_volumes_mn(_p(indptr), _p(col), C.c_int(m), C.c_int(n), _p(b), _p(lay), _p(out))
    return int(out[0]), int(out[1]), int(out[2])


def reorganize(indptr, col, b, m: int, n: int) -> np.ndarray:
    """Partition reorganisation (Alg. 4, both phases): layout[i*n+j] = subgraph of partition i that ends up in batch j."""
    indptr, col, b = _i64(indptr), _i32(col), _i64(b)
    assert len(b) == m * n + 1
    lay = np.zeros(m * n, dtype=np.int32)
    lib().orc_reorganize(_p(indptr), _p(col), C.c_int(m), C.c_int(n), _p(b), _p(lay))
    return lay


def cache_schedule(indptr, col, b, order, rows: int, policy: int) -> List[Dict[str, np.ndarray]]:
    """Per schedule position the rows reused, loaded and released (after the chunk) by a buffer of `rows` rows.
    policy 0: adjacent reuse (Sec. 5.1); policy 1: release only for room, farthest next use first."""
    b, order = _i64(b), _i32(order)
    n = b.shape[0] - 1
    tot = int(sum(len(np.unique(col[indptr[b[k]]:indptr[b[k + 1]]])) for k in range(n)))
    nr, nl, nv = (np.zeros(n, dtype=np.int64) for _ in range(3))
    reuse, load, leave = (np.zeros(max(tot, 1), dtype=np.int32) for _ in range(3))
    lib().orc_cache_schedule(_p(_i64(indptr)), _p(_i32(col)), C.c_int(n), _p(b), _p(order), C.c_int64(rows), C.c_int(policy),
                             _p(nr), _p(nl), _p(nv), _p(reuse), _p(load), _p(leave))
    out, ro, lo, vo = [], 0, 0, 0
    for j in range(n):
        out.append({"reuse": reuse[ro:ro + nr[j]].copy(), "load": load[lo:lo + nl[j]].copy(),
                    "leave": leave[vo:vo + nv[j]].copy()})
        ro, lo, vo = ro + nr[j], lo + nl[j], vo + nv[j]
    return out


def norm(indptr: np.ndarray) -> np.ndarray:
    V = indptr.shape[0] - 1
    s = np.zeros(V, dtype=np.float64)
    lib().orc_norm(C.c_int64(V), _p(indptr), _p(s))
    return s


def aggregate(indptr, col, h, rows: Optional[Tuple[int, int]] = None, s: Optional[np.ndarray] = None) -> np.ndarray:
    """a = diag(s) A~ diag(s) h; with rows=(v0, v1) only those rows are filled.
    s defaults to norm(indptr); a caller that holds only part of the edges passes the full graph's s."""
    h = _f64(h)
    V, d = h.shape
    s = norm(indptr) if s is None else _f64(s)
    a = np.zeros((V, d), dtype=np.float64)
    v0, v1 = rows if rows is not None else (0, V)
    lib().orc_aggregate(_p(indptr), _p(col), _p(s), C.c_int64(v0), C.c_int64(v1), C.c_int64(d), _p(h), _p(a))
    return a


def aggregate_T(indptr, col, x) -> np.ndarray:
    x = _f64(x)
    V, d = x.shape
    s = norm(indptr)
    g = np.zeros((V, d), dtype=np.float64)
    lib().orc_aggregate_T(C.c_int64(V), _p(indptr), _p(col), _p(s), C.c_int64(d), _p(x), _p(g))
    return g


def matmul(A, B) -> np.ndarray:
    A, B = _f64(A), _f64(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    Cm = np.zeros((M, N), dtype=np.float64)
    lib().orc_matmul(C.c_int64(M), C.c_int64(K), C.c_int64(N), _p(A), _p(B), _p(Cm))
    return Cm


def matmul_tn(A, B) -> np.ndarray:
    A, B = _f64(A), _f64(B)
    M, K = A.shape
    M2, N = B.shape
    assert M == M2
    Cm = np.zeros((K, N), dtype=np.float64)
    lib().orc_matmul_tn(C.c_int64(M), C.c_int64(K), C.c_int64(N), _p(A), _p(B), _p(Cm))
    return Cm


def matmul_nt(A, B) -> np.ndarray:
    A, B = _f64(A), _f64(B)
    M, N = A.shape
    K, N2 = B.shape
    assert N == N2
    Cm = np.zeros((M, K), dtype=np.float64)
    lib().orc_matmul_nt(C.c_int64(M), C.c_int64(N), C.c_int64(K), _p(A), _p(B), _p(Cm))
    return Cm


def softmax_ce(logits, labels) -> Tuple[float, np.ndarray]:
    logits = _f64(logits)
    labels = _i32(labels)
    V, Cc = logits.shape
    g = np.zeros((V, Cc), dtype=np.float64)
    loss = lib().orc_softmax_ce(C.c_int64(V), C.c_int64(Cc), _p(logits), _p(labels), _p(g))
    return float(loss), g


def gcn_epoch(indptr, col, dims: Sequence[int], X, Ws: Sequence[np.ndarray], labels, lr: float = 0.01,
              want: Sequence[str] = ("a", "z", "h", "gh", "ga")) -> Dict[str, object]:
    """One epoch on the whole graph.  Returns loss, gW (list), W_new (list) and the
    per-layer arrays named in `want` (lists indexed by layer l)."""
    L = len(dims) - 1
    V = indptr.shape[0] - 1
    X = np.ascontiguousarray(np.asarray(X), dtype=np.float32)
    assert X.shape == (V, dims[0])
    Wcat = np.concatenate([np.ascontiguousarray(np.asarray(w), dtype=np.float32).reshape(-1) for w in Ws])
    labels = _i32(labels)
    dims_a = _i32(dims)
    out: Dict[str, object] = {}
    ptr_arrays = {}
    shapes = {"a": lambda l: dims[l], "z": lambda l: dims[l + 1], "h": lambda l: dims[l + 1],
              "gh": lambda l: dims[l + 1], "ga": lambda l: dims[l]}
    for key in ("a", "z", "h", "gh", "ga"):
        arrs = [np.zeros((V, shapes[key](l)), dtype=np.float64) if key in want else None for l in range(L)]
        out[key] = arrs
        PA = (C.c_void_p * L)(*[None if a is None else a.ctypes.data for a in arrs])
        ptr_arrays[key] = PA
    gW = np.zeros(Wcat.shape[0], dtype=np.float64)
    Wn = np.zeros(Wcat.shape[0], dtype=np.float64)
    loss = C.c_double(0.0)
    rc = lib().orc_gcn_epoch(C.c_int64(V), _p(indptr), _p(col), C.c_int(L), _p(dims_a), _p(X), _p(Wcat),
                             _p(labels), C.c_double(lr), ptr_arrays["a"],
                             ptr_arrays["z"], ptr_arrays["h"], ptr_arrays["gh"], ptr_arrays["ga"], _p(gW),
                             _p(Wn), C.byref(loss))
    assert rc == 0
    out["loss"] = loss.value
    off = 0
    out["gW"], out["W_new"] = [], []
    for l in range(L):
        n = dims[l] * dims[l + 1]
        out["gW"].append(gW[off:off + n].reshape(dims[l], dims[l + 1]).copy())
        out["W_new"].append(Wn[off:off + n].reshape(dims[l], dims[l + 1]).copy())
        off += n
    return out


def layer_fwd_chunked(indptr, col, b, h) -> np.ndarray:
    h = _f64(h)
    V, d = h.shape
    b = _i64(b)
    a = np.zeros((V, d), dtype=np.float64)
    lib().orc_layer_fwd_chunked(C.c_int64(V), _p(indptr), _p(col), C.c_int(b.shape[0] - 1), _p(b), C.c_int64(d),
                                _p(h), _p(a))
    return a


def layer_bwd_chunked(indptr, col, b, ga) -> np.ndarray:
    ga = _f64(ga)
    V, d = ga.shape
    b = _i64(b)
    gh = np.zeros((V, d), dtype=np.float64)
    lib().orc_layer_bwd_chunked(C.c_int64(V), _p(indptr), _p(col), C.c_int(b.shape[0] - 1), _p(b), C.c_int64(d),
                                _p(ga), _p(gh))
    return gh


# ---------------------------------------------------------------- GAT layer (Eq. 3)

def gat_layer_fwd(indptr, col, H, W, a_dst, a_src, slope: float = 0.2, relu: bool = True) -> Dict[str, np.ndarray]:
    """One attention head over the stored edges: t = H W, alpha = neighbour softmax of
    LeakyReLU(a_dst.t_v + a_src.t_u), z_v = sum alpha_e t_u, h = ReLU(z) (or z)."""
    H, W, a_dst, a_src = _f64(H), _f64(W), _f64(a_dst), _f64(a_src)
    V, d_in = H.shape
    d_out = W.shape[1]
    assert W.shape[0] == d_in and a_dst.shape == (d_out,) and a_src.shape == (d_out,)
    indptr, col = _i64(indptr), _i32(col)
    out = {"t": np.zeros((V, d_out)), "alpha": np.zeros(int(indptr[-1])), "z": np.zeros((V, d_out)),
           "h": np.zeros((V, d_out))}
    lib().orc_gat_fwd(C.c_int64(V), _p(indptr), _p(col), C.c_int64(d_in), C.c_int64(d_out), _p(H), _p(W), _p(a_dst),
                      _p(a_src), C.c_double(slope), C.c_int(int(relu)), _p(out["t"]), _p(out["alpha"]), _p(out["z"]),
                      _p(out["h"]))
    return out


def gat_layer_bwd(indptr, col, H, W, a_dst, a_src, fwd: Dict[str, np.ndarray], dh, slope: float = 0.2,
                  relu: bool = True, want_dH: bool = True) -> Dict[str, np.ndarray]:
    """Gradients of the layer above given dh = grad h; `fwd` is gat_layer_fwd's result."""
    H, W, a_dst, a_src, dh = _f64(H), _f64(W), _f64(a_dst), _f64(a_src), _f64(dh)
    V, d_in = H.shape
    d_out = W.shape[1]
    indptr, col = _i64(indptr), _i32(col)
    out = {"dH": np.zeros((V, d_in)) if want_dH else None, "dW": np.zeros((d_in, d_out)), "da_dst": np.zeros(d_out),
           "da_src": np.zeros(d_out)}
    lib().orc_gat_bwd(C.c_int64(V), _p(indptr), _p(col), C.c_int64(d_in), C.c_int64(d_out), _p(H), _p(W), _p(a_dst),
                      _p(a_src), C.c_double(slope), C.c_int(int(relu)), _p(fwd["t"]), _p(fwd["alpha"]), _p(fwd["z"]),
                      _p(dh), _p(out["dH"]), _p(out["dW"]), _p(out["da_dst"]), _p(out["da_src"]))
    return out

"""ctypes binding of libhongtu (include/hongtu.h): argument marshalling only.

Every function here has the name of the C entry point it calls.  torch is used
for device / pinned memory and nothing else; all compute runs in the library.
There is no fallback: if the library is not built, load() raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhongtu.so")

HT_OK = 0
HT_EINVAL, HT_ENOMEM, HT_EHIP, HT_ESHAPE, HT_ESTATE = -1, -2, -3, -4, -5
HT_LOC_DEVICE, HT_LOC_HOST_PINNED = 0, 1
HT_BALANCE_EDGES, HT_BALANCE_VERTICES = 0, 1
HT_PTR_DEVICE, HT_PTR_HOST = 0, 1
HT_CACHE_ADJACENT, HT_CACHE_FARTHEST = 0, 1
HT_ACT_NONE, HT_ACT_RELU = 0, 1
HT_GATHER_AUTO, HT_GATHER_DIRECT, HT_GATHER_BUFFER = 0, 1, 2
HT_CKPT_AGG, HT_CKPT_INPUT = 0, 1
HT_ORDER_AGG_FIRST, HT_ORDER_UPDATE_FIRST, HT_ORDER_AUTO = 0, 1, 2
HT_RES_AUTO, HT_RES_HBM, HT_RES_HOST = 0, 1, 2
HT_STATS_ALL, HT_STATS_AGG_FWD = 0, 1
HT_INTER_AUTO, HT_INTER_MASK, HT_INTER_HYBRID, HT_INTER_RECOMPUTE = 0, 1, 2, 3
HT_BUF_H, HT_BUF_A, HT_BUF_GH, HT_BUF_DW = 0, 1, 2, 3
HT_MAX_LAYERS = 8


class ht_tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int32), ("ld", C.c_int64), ("loc", C.c_int32)]


class ht_part_opts(C.Structure):
    _fields_ = [("add_self_loops", C.c_int32), ("balance_mode", C.c_int32), ("ptr_loc", C.c_int32),
                ("reorder_chunks", C.c_int32), ("cache_rows", C.c_int64), ("cache_policy", C.c_int32),
                ("reserved", C.c_int32)]


class ht_graph_info(C.Structure):
    _fields_ = [("V", C.c_int64), ("E_stored", C.c_int64), ("n_chunks", C.c_int32), ("reserved", C.c_int32),
                ("v_ori", C.c_int64), ("v_ru", C.c_int64), ("alpha", C.c_double), ("max_nsrc", C.c_int64),
                ("max_ndst", C.c_int64), ("max_nnz", C.c_int64), ("cache_rows", C.c_int64), ("hbm_bytes", C.c_int64),
                ("v_load", C.c_int64), ("partition_ms", C.c_double)]


class ht_chunk_info(C.Structure):
    _fields_ = [("dst_begin", C.c_int64), ("dst_end", C.c_int64), ("nnz", C.c_int64), ("n_src", C.c_int64),
                ("n_reuse", C.c_int64), ("n_load", C.c_int64), ("n_leave", C.c_int64)]


class ht_chunk_host(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in
                ("indptr", "col", "nbr", "col_local", "sptr", "sdst", "reuse", "load", "slot", "leave")]


class ht_layer_desc(C.Structure):
    _fields_ = [("d_in", C.c_int32), ("d_out", C.c_int32), ("act", C.c_int32), ("gather_mode", C.c_int32),
                ("ckpt_kind", C.c_int32), ("order", C.c_int32)]


class ht_stats(C.Structure):
    _fields_ = [("t_total_ms", C.c_double), ("t_gather_ms", C.c_double), ("t_spmm_fwd_ms", C.c_double),
                ("t_spmm_bwd_ms", C.c_double), ("t_gemm_ms", C.c_double), ("t_loss_ms", C.c_double),
                ("t_copy_ms", C.c_double), ("t_cpu_accum_ms", C.c_double), ("t_update_ms", C.c_double),
                ("n_spmm_fwd", C.c_int64), ("n_spmm_bwd", C.c_int64), ("n_gemm", C.c_int64), ("edges", C.c_int64),
                ("rows_loaded", C.c_int64), ("rows_reused", C.c_int64), ("bytes_h2d", C.c_int64),
                ("bytes_d2h", C.c_int64), ("bytes_h2d_nodedup", C.c_int64), ("spmm_fwd_alg_bytes", C.c_double),
                ("spmm_bwd_alg_bytes", C.c_double), ("gemm_flops", C.c_double),
                ("t_agg_fwd_layer_ms", C.c_double * HT_MAX_LAYERS),
                ("agg_fwd_layer_alg_bytes", C.c_double * HT_MAX_LAYERS),
                ("n_agg_fwd_layer", C.c_int64 * HT_MAX_LAYERS), ("t_agg_fix_ms", C.c_double),
                ("t_gat_softmax_ms", C.c_double), ("t_gat_dst_ms", C.c_double), ("t_gat_src_ms", C.c_double),
                ("plan_inter", C.c_int32), ("plan_res_h", C.c_int32), ("plan_res_a", C.c_int32),
                ("plan_res_g", C.c_int32)]

    def as_dict(self):
        out = {}
        for k, _ in self._fields_:
            v = getattr(self, k)
            out[k] = list(v) if hasattr(v, "__len__") else v
        return out


class ht_model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("reserved", C.c_int32), ("dims", C.POINTER(C.c_int32)),
                ("W", C.POINTER(C.c_void_p)), ("lr", C.c_float), ("reserved2", C.c_int32)]


class ht_gat_desc(C.Structure):
    _fields_ = [("d_in", C.c_int32), ("d_out", C.c_int32), ("act", C.c_int32), ("slope", C.c_float)]


class ht_gat_model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("res_h", C.c_int32), ("dims", C.POINTER(C.c_int32)),
                ("W", C.POINTER(C.c_void_p)), ("a_dst", C.POINTER(C.c_void_p)), ("a_src", C.POINTER(C.c_void_p)),
                ("lr", C.c_float), ("slope", C.c_float)]


class ht_plan_opts(C.Structure):
    _fields_ = [("res_h", C.c_int32), ("res_a", C.c_int32), ("res_g", C.c_int32), ("inter", C.c_int32),
                ("gather_mode", C.c_int32), ("order", C.c_int32), ("hbm_budget_bytes", C.c_int64),
                ("reuse_input_aggregate", C.c_int32), ("use_graph", C.c_int32), ("stats_detail", C.c_int32),
                ("reserved", C.c_int32)]


EXPORTS = ["ht_ctx_create", "ht_ctx_destroy", "ht_sync", "ht_ctx_set_hbm_budget", "ht_ctx_graph_launches", "ht_tensor_zero", "ht_strerror", "ht_last_error",
           "ht_partition", "ht_graph_destroy", "ht_graph_info_get", "ht_graph_chunk_info", "ht_graph_export_chunk",
           "ht_graph_export_csc", "ht_graph_chunk_order", "ht_graph_reorganize", "ht_layer_fwd", "ht_layer_fwd_static", "ht_layer_bwd", "ht_epoch", "ht_epoch_buffer", "ht_tensor_to_host", "ht_memory_model",
           "ht_chunk_rows_model", "ht_gat_layer_fwd", "ht_gat_layer_bwd", "ht_gat_epoch", "ht_comm_cost_model"]

_lib = None


class HongtuError(RuntimeError):
    def __init__(self, code: int, detail: str):
        super().__init__(f"libhongtu error {code} ({detail})")
        self.code = code


def load():
    """Load libhongtu.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2311_14898_amd.build); "
                           "there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    lib.ht_strerror.restype = C.c_char_p
    lib.ht_last_error.restype = C.c_char_p
    lib.ht_last_error.argtypes = [C.c_void_p]
    lib.ht_chunk_rows_model.restype = C.c_double
    lib.ht_chunk_rows_model.argtypes = [C.c_int64, C.c_int32, C.c_double]
    lib.ht_comm_cost_model.restype = C.c_double
    lib.ht_comm_cost_model.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_double, C.c_double, C.c_double]
    lib.ht_ctx_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_void_p]
    lib.ht_ctx_destroy.argtypes = [C.c_void_p]
    lib.ht_sync.argtypes = [C.c_void_p]
    lib.ht_ctx_set_hbm_budget.argtypes = [C.c_void_p, C.c_int64]
    lib.ht_ctx_graph_launches.argtypes = [C.c_void_p]
    lib.ht_ctx_graph_launches.restype = C.c_int64
    lib.ht_partition.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32,
                                 C.POINTER(ht_part_opts), C.POINTER(C.c_void_p)]
    lib.ht_graph_destroy.argtypes = [C.c_void_p]
    lib.ht_graph_info_get.argtypes = [C.c_void_p, C.POINTER(ht_graph_info)]
    lib.ht_graph_chunk_info.argtypes = [C.c_void_p, C.c_int32, C.POINTER(ht_chunk_info)]
    lib.ht_graph_export_chunk.argtypes = [C.c_void_p, C.c_int32, C.POINTER(ht_chunk_host)]
    lib.ht_graph_export_csc.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ht_graph_chunk_order.argtypes = [C.c_void_p, C.c_void_p]
    lib.ht_graph_reorganize.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ht_layer_fwd.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ht_layer_desc), C.POINTER(ht_tensor), C.c_void_p,
                                 C.POINTER(ht_tensor), C.POINTER(ht_tensor), C.POINTER(ht_stats)]
    lib.ht_layer_fwd_static.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ht_layer_desc), C.POINTER(ht_tensor), C.c_void_p,
                                        C.POINTER(ht_tensor), C.POINTER(ht_tensor)]
    lib.ht_layer_bwd.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ht_layer_desc), C.POINTER(ht_tensor), C.c_void_p,
                                 C.POINTER(ht_tensor), C.POINTER(ht_tensor), C.POINTER(ht_tensor), C.c_void_p,
                                 C.POINTER(ht_stats)]
    lib.ht_epoch.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ht_model), C.POINTER(ht_tensor), C.c_void_p,
                             C.POINTER(ht_plan_opts), C.POINTER(C.c_float), C.POINTER(ht_stats)]
    lib.ht_epoch_buffer.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(ht_tensor)]
    lib.ht_tensor_zero.argtypes = [C.c_void_p, C.POINTER(ht_tensor)]
    lib.ht_tensor_to_host.argtypes = [C.c_void_p, C.POINTER(ht_tensor), C.c_void_p]
    lib.ht_memory_model.argtypes = [C.c_int64, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_double),
                                    C.POINTER(C.c_double)]
    lib.ht_gat_layer_fwd.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ht_gat_desc), C.POINTER(ht_tensor), C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.POINTER(ht_tensor), C.POINTER(ht_stats)]
    lib.ht_gat_layer_bwd.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ht_gat_desc), C.POINTER(ht_tensor), C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.POINTER(ht_tensor), C.POINTER(ht_tensor),
                                     C.POINTER(ht_tensor), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(ht_stats)]
    lib.ht_gat_epoch.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ht_gat_model), C.POINTER(ht_tensor), C.c_void_p,
                                 C.POINTER(C.c_float), C.POINTER(ht_stats)]
    _lib = lib
    return lib


def _check(rc: int, ctx=None):
    if rc != HT_OK:
        lib = load()
        detail = lib.ht_strerror(rc).decode()
        if ctx:
            detail += ": " + lib.ht_last_error(ctx).decode()
        raise HongtuError(rc, detail)


def pad_ld(d: int, loc: int = HT_LOC_HOST_PINNED) -> int:
    """Row pitch in floats: in HBM whole 16-byte vectors, whole 128-byte lines when that costs <= 3 %; in pinned
    host memory whole 64-byte blocks (rows that cross the link in whole requests)."""
    p4, p16, p32 = (d + 3) // 4 * 4, (d + 15) // 16 * 16, (d + 31) // 32 * 32
    if loc != HT_LOC_DEVICE:
        return p16
    return p32 if p32 * 100 <= p4 * 103 else p4


def alloc_matrix(rows: int, cols: int, loc: int = HT_LOC_DEVICE, zero: bool = True) -> torch.Tensor:
    """A [rows x pad_ld(cols)] fp32 tensor in HBM or in pinned host memory."""
    f = torch.zeros if zero else torch.empty
    if loc == HT_LOC_DEVICE:
        return f(rows, pad_ld(cols, loc), dtype=torch.float32, device="cuda")
    return f(rows, pad_ld(cols, loc), dtype=torch.float32, pin_memory=True)


def to_matrix(x: torch.Tensor, loc: int = HT_LOC_DEVICE) -> torch.Tensor:
    """Copy a dense [rows x cols] CPU tensor into a padded matrix at `loc`."""
    m = alloc_matrix(x.shape[0], x.shape[1], loc)
    m[:, : x.shape[1]].copy_(x)
    return m


def tensor_view(t: torch.Tensor, cols: int) -> ht_tensor:
    """ht_tensor over a 2-D fp32 torch tensor whose first `cols` columns are data."""
    assert t.dtype == torch.float32 and t.dim() == 2 and t.stride(1) == 1
    loc = HT_LOC_DEVICE if t.is_cuda else HT_LOC_HOST_PINNED
    if not t.is_cuda:
        assert t.is_pinned(), "host tensors must be pinned"
    return ht_tensor(t.data_ptr(), t.shape[0], cols, t.stride(0), loc)


# ------------------------------------------------------------------ context

def ht_ctx_create(device: int = 0, hip_stream: Optional[int] = None):
    ctx = C.c_void_p()
    _check(load().ht_ctx_create(C.byref(ctx), device, C.c_void_p(hip_stream) if hip_stream else None))
    return ctx


def ht_ctx_destroy(ctx):
    _check(load().ht_ctx_destroy(ctx))


def ht_sync(ctx):
    _check(load().ht_sync(ctx), ctx)


def ht_ctx_graph_launches(ctx) -> int:
    return int(load().ht_ctx_graph_launches(ctx))


def ht_ctx_set_hbm_budget(ctx, nbytes: int):
    _check(load().ht_ctx_set_hbm_budget(ctx, nbytes), ctx)


# ---------------------------------------------------------------- partition

def ht_partition(ctx, V: int, src: torch.Tensor, dst: torch.Tensor, n_chunks: int, add_self_loops: bool = True,
                 balance_mode: int = HT_BALANCE_EDGES, cache_rows: int = 0, reorder_chunks: bool = False,
                 cache_policy: int = 0):
    assert src.dtype == torch.int32 and dst.dtype == torch.int32 and src.numel() == dst.numel()
    assert src.is_cuda == dst.is_cuda
    src, dst = src.contiguous(), dst.contiguous()
    opts = ht_part_opts(int(add_self_loops), balance_mode, HT_PTR_DEVICE if src.is_cuda else HT_PTR_HOST,
                        int(reorder_chunks), cache_rows, cache_policy, 0)
    if src.is_cuda:
        torch.cuda.synchronize()
    g = C.c_void_p()
    _check(load().ht_partition(ctx, V, src.numel(), C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), n_chunks,
                               C.byref(opts), C.byref(g)), ctx)
    return g


def ht_graph_destroy(g):
    _check(load().ht_graph_destroy(g))


def ht_graph_info_get(g) -> ht_graph_info:
    info = ht_graph_info()
    _check(load().ht_graph_info_get(g, C.byref(info)))
    return info


def ht_graph_chunk_info(g, j: int) -> ht_chunk_info:
    ci = ht_chunk_info()
    _check(load().ht_graph_chunk_info(g, j, C.byref(ci)))
    return ci


def ht_graph_export_chunk(g, j: int) -> dict:
    ci = ht_graph_chunk_info(g, j)
    nd = ci.dst_end - ci.dst_begin
    arrs = {"indptr": np.zeros(nd + 1, np.int64), "col": np.zeros(ci.nnz, np.int32),
            "nbr": np.zeros(ci.n_src, np.int32), "col_local": np.zeros(ci.nnz, np.int32),
            "sptr": np.zeros(ci.n_src + 1, np.int64), "sdst": np.zeros(ci.nnz, np.int32),
            "reuse": np.zeros(ci.n_reuse, np.int32), "load": np.zeros(ci.n_load, np.int32),
            "slot": np.zeros(ci.n_src, np.int32), "leave": np.zeros(ci.n_leave, np.int32)}
    ch = ht_chunk_host(*[arrs[k].ctypes.data for k, _ in ht_chunk_host._fields_])
    _check(load().ht_graph_export_chunk(g, j, C.byref(ch)))
    arrs["info"] = ci
    return arrs


def ht_graph_export_csc(g):
    info = ht_graph_info_get(g)
    indptr = np.zeros(info.V + 1, np.int64)
    col = np.zeros(info.E_stored, np.int32)
    s = np.zeros(info.V, np.float32)
    b = np.zeros(info.n_chunks + 1, np.int64)
    _check(load().ht_graph_export_csc(g, indptr.ctypes.data, col.ctypes.data, s.ctypes.data, b.ctypes.data))
    return indptr, col, s, b


def ht_graph_chunk_order(g) -> np.ndarray:
    info = ht_graph_info_get(g)
    order = np.zeros(info.n_chunks, np.int32)
    _check(load().ht_graph_chunk_order(g, order.ctypes.data))
    return order


def ht_graph_reorganize(ctx, g, m: int):
    """(layout[m*n], (V_ori, V_+p2p, V_+ru) before, the same after) for the graph's chunks read as m partitions."""
    info = ht_graph_info_get(g)
    layout = np.zeros(info.n_chunks, np.int32)
    before, after = np.zeros(3, np.int64), np.zeros(3, np.int64)
    _check(load().ht_graph_reorganize(ctx, g, m, layout.ctypes.data, before.ctypes.data, after.ctypes.data), ctx)
    return layout, tuple(int(x) for x in before), tuple(int(x) for x in after)


# -------------------------------------------------------------------- layer

def ht_layer_fwd(ctx, g, d_in: int, d_out: int, act: int, H_in: torch.Tensor, W: torch.Tensor, H_out: torch.Tensor,
                 A_ckpt: Optional[torch.Tensor] = None, gather_mode: int = HT_GATHER_AUTO, want_stats: bool = False,
                 order: int = HT_ORDER_AGG_FIRST):
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == (d_in, d_out)
    desc = ht_layer_desc(d_in, d_out, act, gather_mode, 0, order)
    hin, hout = tensor_view(H_in, d_in), tensor_view(H_out, d_out)
    ack = tensor_view(A_ckpt, d_in) if A_ckpt is not None else None
    st = ht_stats() if want_stats else None
    torch.cuda.synchronize()
    _check(load().ht_layer_fwd(ctx, g, C.byref(desc), C.byref(hin), C.c_void_p(W.data_ptr()), C.byref(hout),
                               C.byref(ack) if ack is not None else None, C.byref(st) if st is not None else None),
           ctx)
    return st


def ht_layer_fwd_static(ctx, g, d_in: int, d_out: int, act: int, H_in: torch.Tensor, W: torch.Tensor, H_out: torch.Tensor,
                        A_ckpt: torch.Tensor):
    """ht_layer_fwd without any device allocation (all tensors in HBM, scratch in the library's static array)."""
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == (d_in, d_out)
    desc = ht_layer_desc(d_in, d_out, act, HT_GATHER_AUTO, 0, HT_ORDER_AGG_FIRST)
    hin, hout, ack = tensor_view(H_in, d_in), tensor_view(H_out, d_out), tensor_view(A_ckpt, d_in)
    _check(load().ht_layer_fwd_static(ctx, g, C.byref(desc), C.byref(hin), C.c_void_p(W.data_ptr()), C.byref(hout),
                                      C.byref(ack)), ctx)


def ht_layer_bwd(ctx, g, d_in: int, d_out: int, act: int, ckpt: torch.Tensor, W: torch.Tensor, dH_out: torch.Tensor,
                 dW: torch.Tensor, dH_in: Optional[torch.Tensor] = None, H_out: Optional[torch.Tensor] = None,
                 ckpt_kind: int = HT_CKPT_AGG, gather_mode: int = HT_GATHER_AUTO, want_stats: bool = False,
                 order: int = HT_ORDER_AGG_FIRST):
    assert W.is_cuda and W.is_contiguous() and tuple(W.shape) == (d_in, d_out)
    assert dW.is_cuda and dW.is_contiguous() and tuple(dW.shape) == (d_in, d_out) and dW.dtype == torch.float32
    desc = ht_layer_desc(d_in, d_out, act, gather_mode, ckpt_kind, order)
    ck, dho = tensor_view(ckpt, d_in), tensor_view(dH_out, d_out)
    ho = tensor_view(H_out, d_out) if H_out is not None else None
    dhi = tensor_view(dH_in, d_in) if dH_in is not None else None
    st = ht_stats() if want_stats else None
    torch.cuda.synchronize()
    _check(load().ht_layer_bwd(ctx, g, C.byref(desc), C.byref(ck), C.c_void_p(W.data_ptr()), C.byref(dho),
                               C.byref(ho) if ho is not None else None, C.byref(dhi) if dhi is not None else None,
                               C.c_void_p(dW.data_ptr()), C.byref(st) if st is not None else None), ctx)
    return st


# ---------------------------------------------------------------- GAT layer

def _vec(t: torch.Tensor, n: int):
    assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == n
    return C.c_void_p(t.data_ptr())


def ht_gat_layer_fwd(ctx, g, d_in: int, d_out: int, act: int, H_in: torch.Tensor, W: torch.Tensor, a_dst: torch.Tensor,
                     a_src: torch.Tensor, H_out: torch.Tensor, slope: float = 0.2, want_stats: bool = False):
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == (d_in, d_out)
    desc = ht_gat_desc(d_in, d_out, act, slope)
    hin, hout = tensor_view(H_in, d_in), tensor_view(H_out, d_out)
    st = ht_stats() if want_stats else None
    torch.cuda.synchronize()
    _check(load().ht_gat_layer_fwd(ctx, g, C.byref(desc), C.byref(hin), C.c_void_p(W.data_ptr()), _vec(a_dst, d_out),
                                   _vec(a_src, d_out), C.byref(hout), C.byref(st) if st is not None else None), ctx)
    return st


def ht_gat_layer_bwd(ctx, g, d_in: int, d_out: int, act: int, H_in: torch.Tensor, W: torch.Tensor, a_dst: torch.Tensor,
                     a_src: torch.Tensor, H_out: torch.Tensor, dH_out: torch.Tensor, dW: torch.Tensor,
                     da_dst: torch.Tensor, da_src: torch.Tensor, dH_in: Optional[torch.Tensor] = None,
                     slope: float = 0.2, want_stats: bool = False):
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == (d_in, d_out)
    assert dW.is_cuda and dW.dtype == torch.float32 and dW.is_contiguous() and tuple(dW.shape) == (d_in, d_out)
    desc = ht_gat_desc(d_in, d_out, act, slope)
    hin, hout, dho = tensor_view(H_in, d_in), tensor_view(H_out, d_out), tensor_view(dH_out, d_out)
    dhi = tensor_view(dH_in, d_in) if dH_in is not None else None
    st = ht_stats() if want_stats else None
    torch.cuda.synchronize()
    _check(load().ht_gat_layer_bwd(ctx, g, C.byref(desc), C.byref(hin), C.c_void_p(W.data_ptr()), _vec(a_dst, d_out),
                                   _vec(a_src, d_out), C.byref(hout), C.byref(dho),
                                   C.byref(dhi) if dhi is not None else None, C.c_void_p(dW.data_ptr()),
                                   _vec(da_dst, d_out), _vec(da_src, d_out), C.byref(st) if st is not None else None), ctx)
    return st


def ht_comm_cost_model(v_ori: int, v_p2p: int, v_ru: int, bytes_per_row: int, t_hd: float, t_dd: float, t_ru: float) -> float:
    return float(load().ht_comm_cost_model(v_ori, v_p2p, v_ru, bytes_per_row, t_hd, t_dd, t_ru))


def ht_gat_epoch(ctx, g, dims: Sequence[int], Ws: List[torch.Tensor], a_dst: List[torch.Tensor], a_src: List[torch.Tensor],
                 lr: float, X: torch.Tensor, labels: torch.Tensor, slope: float = 0.2, want_stats: bool = False,
                 res_h: int = 0):
    """One GAT epoch; Ws, a_dst, a_src (device tensors) are updated in place.  Returns (loss, stats or None)."""
    L = len(dims) - 1
    assert len(Ws) == L and len(a_dst) == L and len(a_src) == L and labels.is_cuda and labels.dtype == torch.int32
    for l in range(L):
        assert Ws[l].is_cuda and Ws[l].is_contiguous() and tuple(Ws[l].shape) == (dims[l], dims[l + 1])
        _vec(a_dst[l], dims[l + 1]), _vec(a_src[l], dims[l + 1])
    dims_a = (C.c_int32 * (L + 1))(*dims)
    Wp = (C.c_void_p * L)(*[w.data_ptr() for w in Ws])
    Ap = (C.c_void_p * L)(*[a.data_ptr() for a in a_dst])
    Sp = (C.c_void_p * L)(*[a.data_ptr() for a in a_src])
    model = ht_gat_model(L, res_h, dims_a, Wp, Ap, Sp, lr, slope)
    x = tensor_view(X, dims[0])
    loss = C.c_float(0.0)
    st = ht_stats() if want_stats else None
    torch.cuda.synchronize()
    _check(load().ht_gat_epoch(ctx, g, C.byref(model), C.byref(x), C.c_void_p(labels.data_ptr()), C.byref(loss),
                               C.byref(st) if st is not None else None), ctx)
    return loss.value, st


# -------------------------------------------------------------------- epoch

def ht_epoch(ctx, g, dims: Sequence[int], Ws: List[torch.Tensor], lr: float, X: torch.Tensor, labels: torch.Tensor,
             res_h: int = HT_RES_AUTO, res_a: int = HT_RES_AUTO, res_g: int = HT_RES_AUTO, inter: int = HT_INTER_AUTO,
             gather_mode: int = HT_GATHER_AUTO, hbm_budget_bytes: int = 0, want_stats: bool = False, sync: bool = True,
             order: int = HT_ORDER_AGG_FIRST, reuse_input_aggregate: bool = False, use_graph: bool = False,
             stats_detail: int = 0):
    """One epoch; Ws (device tensors) are updated in place.  Returns (loss, stats or None)."""
    L = len(dims) - 1
    assert len(Ws) == L and labels.is_cuda and labels.dtype == torch.int32
    for l, w in enumerate(Ws):
        assert w.is_cuda and w.is_contiguous() and tuple(w.shape) == (dims[l], dims[l + 1])
    dims_a = (C.c_int32 * (L + 1))(*dims)
    Wp = (C.c_void_p * L)(*[w.data_ptr() for w in Ws])
    model = ht_model(L, 0, dims_a, Wp, lr, 0)
    plan = ht_plan_opts(res_h, res_a, res_g, inter, gather_mode, order, hbm_budget_bytes, int(reuse_input_aggregate), int(use_graph),
                        stats_detail, 0)
    x = tensor_view(X, dims[0])
    loss = C.c_float(0.0)
    st = ht_stats() if want_stats else None
    if sync:
        torch.cuda.synchronize()
    _check(load().ht_epoch(ctx, g, C.byref(model), C.byref(x), C.c_void_p(labels.data_ptr()), C.byref(plan),
                           C.byref(loss), C.byref(st) if st is not None else None), ctx)
    return loss.value, st


def ht_tensor_zero(ctx, t: torch.Tensor, cols: int):
    """Zero a [rows x ld] tensor (HBM or pinned host) through the library."""
    tv = tensor_view(t, cols)
    torch.cuda.synchronize()
    _check(load().ht_tensor_zero(ctx, C.byref(tv)), ctx)


def ht_epoch_buffer(ctx, kind: int, layer: int) -> torch.Tensor:
    """Copy of an internal epoch buffer as a CPU tensor [rows x cols] (padding dropped)."""
    t = ht_tensor()
    _check(load().ht_epoch_buffer(ctx, kind, layer, C.byref(t)), ctx)
    return ht_tensor_to_host(ctx, t)


class _DeviceArray:
    """A [rows x ld] fp32 device buffer seen through the CUDA array interface (no copy)."""

    def __init__(self, t: ht_tensor):
        self.__cuda_array_interface__ = {"shape": (int(t.rows), int(t.ld)), "typestr": "<f4", "data": (int(t.ptr), False),
                                         "version": 3, "strides": None}


def ht_epoch_buffer_rows(ctx, kind: int, layer: int, rows, cols=None) -> torch.Tensor:
    """The data columns of the given rows (an index array or a slice) of an internal epoch buffer, as a CPU tensor; the rows
    are indexed where the buffer lives (HBM or pinned host memory), so a multi-gigabyte buffer is never copied whole."""
    t = ht_tensor()
    _check(load().ht_epoch_buffer(ctx, kind, layer, C.byref(t)), ctx)
    ht_sync(ctx)
    if t.loc == HT_LOC_DEVICE:
        whole = torch.as_tensor(_DeviceArray(t), device="cuda")
    else:
        whole = torch.from_numpy(np.ctypeslib.as_array(C.cast(C.c_void_p(t.ptr), C.POINTER(C.c_float)), shape=(int(t.rows), int(t.ld))))
    if cols is not None:                             # a subset of the data columns, picked where the buffer lives
        cidx = torch.as_tensor(np.asarray(cols, dtype=np.int64))
        assert cidx.numel() == 0 or (int(cidx.min()) >= 0 and int(cidx.max()) < t.cols)
        cidx = cidx.to(whole.device)
    if isinstance(rows, slice):                      # a contiguous row range
        part = whole[rows]
    else:
        idx = torch.as_tensor(np.asarray(rows, dtype=np.int64))
        assert idx.numel() == 0 or (int(idx.min()) >= 0 and int(idx.max()) < t.rows)
        part = whole[idx.to(whole.device)]
    part = part[:, : t.cols] if cols is None else part[:, cidx]
    return part.cpu().clone()


def ht_tensor_to_host(ctx, t: ht_tensor) -> torch.Tensor:
    out = torch.empty(t.rows, t.cols, dtype=torch.float32)
    _check(load().ht_tensor_to_host(ctx, C.byref(t), C.c_void_p(out.data_ptr())), ctx)
    return out


def ht_memory_model(V: int, dims: Sequence[int]):
    L = len(dims) - 1
    d = (C.c_int32 * (L + 1))(*dims)
    vb, ib = C.c_double(0), C.c_double(0)
    _check(load().ht_memory_model(V, L, d, C.byref(vb), C.byref(ib)))
    return vb.value, ib.value


def ht_chunk_rows_model(V: int, n_chunks: int, alpha: float) -> float:
    return load().ht_chunk_rows_model(V, n_chunks, alpha)


def ht_strerror_text(code: int) -> str:
    return load().ht_strerror(code).decode()

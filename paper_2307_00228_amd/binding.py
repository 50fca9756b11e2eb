"""ctypes binding of ``libinferturbo_hip.so``: argument marshalling only.

Same names as the C ABI (``include/inferturbo.h``).  Tensors are torch CUDA(HIP)
tensors used purely as device memory; bf16 tensors are ``torch.bfloat16``.
Every step of the path runs inside the library's kernels; there is no CPU
fallback -- if the library has not been built, importing fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libinferturbo_hip.so")

ITB_F32, ITB_BF16 = 0, 1
AGG_SUM, AGG_MEAN, AGG_GCN, AGG_GAT, AGG_MAX, AGG_MIN, AGG_NONE = 0, 1, 2, 3, 4, 5, 6
ACT_NONE, ACT_RELU = 0, 1
PLAN_GATHER_UPDATE, PLAN_PROJECT_GATHER, PLAN_ATTENTION, PLAN_UPDATE_ONLY, PLAN_GATHER_UPDATE_CHAINED = 0, 1, 2, 3, 4
INT64_MAX = (1 << 63) - 1

STATUS = {0: "ITB_OK", -1: "ITB_ERR_NULL", -2: "ITB_ERR_SIZE", -3: "ITB_ERR_RANGE", -4: "ITB_ERR_DTYPE",
          -5: "ITB_ERR_UNSUPPORTED", -6: "ITB_ERR_WORKSPACE", -7: "ITB_ERR_DEVICE"}


class InferTurboError(RuntimeError):
    def __init__(self, call: str, code: int):
        super().__init__(f"{call} failed: {STATUS.get(code, code)}")
        self.code = code


class itb_split(C.Structure):
    _fields_ = [("threshold", C.c_int64), ("n_hubs", C.c_int64), ("n_shadows", C.c_int64),
                ("hub_ids", C.c_void_p), ("hub_shadow_off", C.c_void_p),
                ("shadow_begin", C.c_void_p), ("shadow_end", C.c_void_p), ("shadow_owner", C.c_void_p)]


class itb_gather_desc(C.Structure):
    _fields_ = [("agg", C.c_int32), ("dtype_in", C.c_int32), ("dtype_out", C.c_int32), ("dim", C.c_int32),
                ("heads", C.c_int32), ("leaky_slope", C.c_float), ("act", C.c_int32), ("bias", C.c_void_p),
                ("edge_coef", C.c_void_p), ("addend", C.c_void_p)]


class itb_apply_desc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("d_in", C.c_int32), ("d_out", C.c_int32), ("act", C.c_int32),
                ("heads", C.c_int32)]


class itb_layer(C.Structure):
    _fields_ = [("agg", C.c_int32), ("d_in", C.c_int32), ("d_out", C.c_int32), ("act", C.c_int32),
                ("heads", C.c_int32), ("leaky_slope", C.c_float),
                ("w_self", C.c_void_p), ("w_nbr", C.c_void_p), ("bias", C.c_void_p),
                ("att_src", C.c_void_p), ("att_dst", C.c_void_p), ("w_edge", C.c_void_p)]


class itb_apply_chain(C.Structure):
    _fields_ = [("w_first", C.c_void_p), ("w_second", C.c_void_p), ("dc", C.c_int32), ("out_first", C.c_void_p),
                ("out_second", C.c_void_p)]


class itb_stage_events(C.Structure):
    _fields_ = [("events", C.POINTER(C.c_void_p)), ("n_events", C.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i64, i32, szp = C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_size_t)
    lib.build_csr_by_dst.argtypes = [i64, i64, vp, vp, vp, vp, vp, vp, szp, vp]
    lib.split_hubs.argtypes = [i64, vp, i64, C.POINTER(i64), C.POINTER(i64), vp, vp, vp, vp, vp, vp, szp, vp]
    lib.gcn_norm_scales.argtypes = [i64, vp, vp, vp, vp, vp]
    lib.gcn_edge_coefficients.argtypes = [i64, vp, vp, vp, vp]
    lib.gather_layer.argtypes = [C.POINTER(itb_gather_desc), i64, vp, vp, C.POINTER(itb_split), vp, vp, vp, vp,
                                 i64, i64, vp, szp, vp]
    lib.apply_layer.argtypes = [C.POINTER(itb_apply_desc), i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                C.POINTER(itb_apply_chain), vp]
    lib.infer_layer_plan.argtypes = [i32, i32, C.POINTER(itb_layer), C.POINTER(i32)]
    lib.scale_rows.argtypes = [i32, i64, i32, vp, vp, vp, vp]
    lib.copy_columns.argtypes = [i32, i64, i32, i32, vp, vp, vp]
    lib.gather_layer_noalloc.argtypes = [C.POINTER(itb_gather_desc), i64, vp, vp, C.POINTER(itb_split), vp, vp, vp, vp,
                                         i64, i64, vp]
    lib.infer_full_graph.argtypes = [i64, i64, vp, vp, vp, C.POINTER(itb_split), i32, i32, C.POINTER(itb_layer),
                                     vp, vp, i64, vp, i32, vp, szp, C.POINTER(itb_stage_events), vp]
    lib.aggregate_edge_features.argtypes = [i32, i32, i64, vp, C.POINTER(itb_split), i32, vp, vp, vp, vp, vp, szp, vp]
    lib.itb_shutdown.argtypes = []
    lib.itb_random_row_read.argtypes = [vp, i64, i32, vp, i64, vp, i64, vp]
    lib.hub_threshold_heuristic.argtypes = [i64, i64, C.c_double, C.POINTER(i64)]
    lib.itb_set_tuning.argtypes = [i32, i32]
    lib.itb_copy_bytes.argtypes = [vp, vp, i64, vp]
    for f in ("itb_copy_bytes", "scale_rows", "build_csr_by_dst", "split_hubs", "gcn_norm_scales", "gather_layer", "apply_layer",
              "infer_full_graph", "itb_set_tuning", "hub_threshold_heuristic", "gcn_edge_coefficients",
              "gather_layer_noalloc", "itb_shutdown", "itb_random_row_read", "infer_layer_plan",
              "aggregate_edge_features", "copy_columns"):
        getattr(lib, f).restype = i32
    return lib


lib = _load()


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor required"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(call: str, rc: int):
    if rc != 0:
        raise InferTurboError(call, rc)


def _workspace(nbytes: int) -> Optional[torch.Tensor]:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return ITB_F32
    if t.dtype == torch.bfloat16:
        return ITB_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def copy_bytes(src: torch.Tensor, dst: torch.Tensor):
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    _check("itb_copy_bytes", lib.itb_copy_bytes(_ptr(src), _ptr(dst), n, _stream()))


def random_row_read(table: torch.Tensor, idx: torch.Tensor, sink: Optional[torch.Tensor] = None):
    """Measurement aid: reads row idx[i] of ``table`` ([rows x row_bytes] as any dtype) for every i; returns the sink."""
    n_rows = table.shape[0]
    row_bytes = table.shape[1] * table.element_size()
    assert idx.dtype == torch.int32
    if sink is None:
        sink = torch.empty(2048 * 256, dtype=torch.int32, device="cuda")
    _check("itb_random_row_read", lib.itb_random_row_read(_ptr(table), n_rows, row_bytes, _ptr(idx), idx.numel(), _ptr(sink),
                                                          sink.numel() * 4, _stream()))
    return sink


def shutdown():
    _check("itb_shutdown", lib.itb_shutdown())


def set_tuning(key: int, value: int):
    _check("itb_set_tuning", lib.itb_set_tuning(key, value))


# --------------------------------------------------------------------------------------------
def build_csr_by_dst(n_nodes: int, src: torch.Tensor, dst: torch.Tensor, want_deg_out: bool = True,
                     workspace: Optional[torch.Tensor] = None):
    """Returns (rowptr int64 [N+1], col int32 [E], deg_out int32 [N] or None)."""
    e = src.numel()
    assert src.dtype == torch.int32 and dst.dtype == torch.int32 and dst.numel() == e
    rowptr = torch.empty(n_nodes + 1, dtype=torch.int64, device="cuda")
    col = torch.empty(e, dtype=torch.int32, device="cuda")
    deg_out = torch.empty(n_nodes, dtype=torch.int32, device="cuda") if want_deg_out else None
    need = C.c_size_t(0)
    _check("build_csr_by_dst(size)", lib.build_csr_by_dst(n_nodes, e, None, None, None, None, None, None, C.byref(need), None))
    ws = workspace if workspace is not None and workspace.numel() >= need.value else _workspace(need.value)
    size = C.c_size_t(ws.numel())
    _check("build_csr_by_dst", lib.build_csr_by_dst(n_nodes, e, _ptr(src), _ptr(dst), _ptr(rowptr), _ptr(col),
                                                    _ptr(deg_out), _ptr(ws), C.byref(size), _stream()))
    return rowptr, col, deg_out


def hub_threshold_heuristic(total_edges: int, total_workers: int, lam: float = 0.1) -> int:
    t = C.c_int64(0)
    _check("hub_threshold_heuristic", lib.hub_threshold_heuristic(total_edges, total_workers, lam, C.byref(t)))
    return t.value


@dataclass
class Split:
    threshold: int
    n_hubs: int
    n_shadows: int
    hub_ids: torch.Tensor
    hub_shadow_off: torch.Tensor
    shadow_begin: torch.Tensor
    shadow_end: torch.Tensor
    shadow_owner: torch.Tensor

    def c_struct(self) -> itb_split:
        return itb_split(self.threshold, self.n_hubs, self.n_shadows, self.hub_ids.data_ptr(),
                         self.hub_shadow_off.data_ptr(), self.shadow_begin.data_ptr(),
                         self.shadow_end.data_ptr(), self.shadow_owner.data_ptr())


def split_hubs(rowptr: torch.Tensor, threshold: int) -> Split:
    n = rowptr.numel() - 1
    need = C.c_size_t(0)
    nh, ns = C.c_int64(0), C.c_int64(0)
    _check("split_hubs(size)", lib.split_hubs(n, None, threshold, C.byref(nh), C.byref(ns), None, None, None, None, None,
                                              None, C.byref(need), None))
    ws = _workspace(need.value)
    size = C.c_size_t(ws.numel())
    _check("split_hubs(count)", lib.split_hubs(n, _ptr(rowptr), threshold, C.byref(nh), C.byref(ns), None, None, None, None,
                                               None, _ptr(ws), C.byref(size), _stream()))
    h, s = nh.value, ns.value
    dev = "cuda"
    sp = Split(threshold, h, s,
               torch.empty(max(h, 1), dtype=torch.int32, device=dev)[:h],
               torch.empty(h + 1, dtype=torch.int64, device=dev),
               torch.empty(max(s, 1), dtype=torch.int64, device=dev)[:s],
               torch.empty(max(s, 1), dtype=torch.int64, device=dev)[:s],
               torch.empty(max(s, 1), dtype=torch.int32, device=dev)[:s])
    _check("split_hubs(fill)", lib.split_hubs(n, _ptr(rowptr), threshold, C.byref(nh), C.byref(ns), _ptr(sp.hub_ids),
                                              _ptr(sp.hub_shadow_off), _ptr(sp.shadow_begin), _ptr(sp.shadow_end),
                                              _ptr(sp.shadow_owner), _ptr(ws), C.byref(size), _stream()))
    return sp


def copy_columns(a: torch.Tensor, cols_out: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """[rows x cols_in] -> [rows x cols_out]: zero columns appended, or the first cols_out columns kept."""
    rows, cols_in = a.shape
    if out is None:
        out = torch.empty((rows, cols_out), dtype=a.dtype, device="cuda")
    _check("copy_columns", lib.copy_columns(dtype_code(a), rows, cols_in, cols_out, _ptr(a), _ptr(out), _stream()))
    return out


def gcn_norm_scales(rowptr: torch.Tensor, deg_out: torch.Tensor):
    n = rowptr.numel() - 1
    s_src = torch.empty(n, dtype=torch.float32, device="cuda")
    s_dst = torch.empty(n, dtype=torch.float32, device="cuda")
    _check("gcn_norm_scales", lib.gcn_norm_scales(n, _ptr(rowptr), _ptr(deg_out), _ptr(s_src), _ptr(s_dst), _stream()))
    return s_src, s_dst


def gcn_edge_coefficients(col: torch.Tensor, src_scale: torch.Tensor, out: Optional[torch.Tensor] = None):
    e = col.numel()
    if out is None:
        out = torch.empty(e, dtype=torch.float32, device="cuda")
    _check("gcn_edge_coefficients", lib.gcn_edge_coefficients(e, _ptr(col), _ptr(src_scale), _ptr(out), _stream()))
    return out


def gather_layer(agg: int, rowptr, col, h, split: Optional[Split] = None, src_scale=None, dst_scale=None,
                 out_dtype=None, heads: int = 1, leaky_slope: float = 0.2, edge_lo: int = 0, edge_hi: int = INT64_MAX,
                 out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                 act: int = ACT_NONE, bias: Optional[torch.Tensor] = None, edge_coef: Optional[torch.Tensor] = None,
                 addend: Optional[torch.Tensor] = None):
    n, dim = h.shape
    out_dtype = out_dtype or h.dtype
    if out is None:
        out = torch.empty((n, dim), dtype=out_dtype, device="cuda")
    assert addend is None or (addend.shape == out.shape and addend.dtype == out.dtype and addend.is_contiguous())
    desc = itb_gather_desc(agg, dtype_code(h), dtype_code(out), dim, heads, leaky_slope, act,
                           bias.data_ptr() if bias is not None else None,
                           edge_coef.data_ptr() if edge_coef is not None else None,
                           addend.data_ptr() if addend is not None else None)
    sp = split.c_struct() if split is not None else None
    spp = C.byref(sp) if sp is not None else None
    need = C.c_size_t(0)
    _check("gather_layer(size)", lib.gather_layer(C.byref(desc), n, None, None, spp, None, None, None, None, edge_lo, edge_hi,
                                                  None, C.byref(need), None))
    ws = workspace if workspace is not None and workspace.numel() >= need.value else _workspace(need.value)
    size = C.c_size_t(ws.numel())
    _check("gather_layer", lib.gather_layer(C.byref(desc), n, _ptr(rowptr), _ptr(col), spp, _ptr(h), _ptr(src_scale),
                                            _ptr(dst_scale), _ptr(out), edge_lo, edge_hi, _ptr(ws), C.byref(size), _stream()))
    return out


def gather_layer_noalloc(agg: int, rowptr, col, h, out: torch.Tensor, split: Optional[Split] = None, src_scale=None,
                         dst_scale=None, heads: int = 1, leaky_slope: float = 0.2, edge_lo: int = 0, edge_hi: int = INT64_MAX,
                         act: int = ACT_NONE, bias: Optional[torch.Tensor] = None, edge_coef: Optional[torch.Tensor] = None,
                         addend: Optional[torch.Tensor] = None):
    """gather_layer on the library's built-in scratch: the caller passes inputs and the output, nothing is allocated."""
    n, dim = h.shape
    desc = itb_gather_desc(agg, dtype_code(h), dtype_code(out), dim, heads, leaky_slope, act,
                           bias.data_ptr() if bias is not None else None,
                           edge_coef.data_ptr() if edge_coef is not None else None,
                           addend.data_ptr() if addend is not None else None)
    sp = split.c_struct() if split is not None else None
    spp = C.byref(sp) if sp is not None else None
    _check("gather_layer_noalloc", lib.gather_layer_noalloc(C.byref(desc), n, _ptr(rowptr), _ptr(col), spp, _ptr(h),
                                                            _ptr(src_scale), _ptr(dst_scale), _ptr(out), edge_lo, edge_hi,
                                                            _stream()))
    return out


def aggregate_edge_features(agg: int, rowptr, edge_feat: torch.Tensor, split: Optional[Split] = None, edge_coef=None,
                            dst_scale=None, out: Optional[torch.Tensor] = None):
    """Per-destination reduce of the per-edge feature table ([E x d_e], CSR order): [N x d_e]."""
    n = rowptr.numel() - 1
    d_e = edge_feat.shape[1]
    if out is None:
        out = torch.empty((n, d_e), dtype=edge_feat.dtype, device="cuda")
    sp = split.c_struct() if split is not None else None
    spp = C.byref(sp) if sp is not None else None
    need = C.c_size_t(0)
    _check("aggregate_edge_features(size)", lib.aggregate_edge_features(agg, dtype_code(edge_feat), n, None, spp, d_e, None, None,
                                                                        None, None, None, C.byref(need), None))
    ws = _workspace(need.value)
    size = C.c_size_t(ws.numel())
    _check("aggregate_edge_features", lib.aggregate_edge_features(agg, dtype_code(edge_feat), n, _ptr(rowptr), spp, d_e,
                                                                  _ptr(edge_feat), _ptr(edge_coef), _ptr(dst_scale), _ptr(out),
                                                                  _ptr(ws), C.byref(size), _stream()))
    return out


def scale_rows(x: torch.Tensor, row_scale: torch.Tensor, out: Optional[torch.Tensor] = None):
    n, dim = x.shape
    if out is None:
        out = torch.empty_like(x)
    _check("scale_rows", lib.scale_rows(dtype_code(x), n, dim, _ptr(x), _ptr(row_scale), _ptr(out), _stream()))
    return out


def apply_layer(h_self, agg, w_self, w_nbr, bias, act: int, out: Optional[torch.Tensor] = None,
                heads: int = 0, att_src=None, att_dst=None, msg_scale=None, msg_out=None, addend=None,
                w_second=None, out_second=None, chain=None, store_out: bool = True):
    """Returns out; with heads > 0 (out, s_src, s_dst); with w_second (out, out_second); with chain = (w_first, w_second[,
    out_first, out_second]) -- the chained projection of the finished rows -- (out, out_first, out_second), where out is
    None when store_out is False (the rows themselves are then never written)."""
    n, d_in = agg.shape
    d_out = w_nbr.shape[1]
    if out is None and (store_out or chain is None):
        out = torch.empty((n, d_out), dtype=agg.dtype, device="cuda")
    ch = None
    if chain is not None:
        cw1, cw2 = chain[0], chain[1]
        dc = cw1.shape[1]
        co1 = chain[2] if len(chain) > 2 and chain[2] is not None else torch.empty((n, dc), dtype=agg.dtype, device="cuda")
        co2 = chain[3] if len(chain) > 3 and chain[3] is not None else torch.empty((n, dc), dtype=agg.dtype, device="cuda")
        assert cw1.shape == cw2.shape == (d_out, dc) and co1.shape == co2.shape == (n, dc)
        ch = itb_apply_chain(cw1.data_ptr(), cw2.data_ptr(), dc, co1.data_ptr(), co2.data_ptr())
        if not store_out:
            out = None
    desc = itb_apply_desc(dtype_code(agg), d_in, d_out, act, heads)
    s_src = s_dst = None
    if heads:
        s_src = torch.empty((n, heads), dtype=torch.float32, device="cuda")
        s_dst = torch.empty((n, heads), dtype=torch.float32, device="cuda")
    if w_second is not None and out_second is None:
        out_second = torch.empty((n, d_out), dtype=agg.dtype, device="cuda")
    _check("apply_layer", lib.apply_layer(C.byref(desc), n, _ptr(h_self), _ptr(agg), _ptr(w_self), _ptr(w_nbr), _ptr(bias),
                                          _ptr(out), _ptr(att_src), _ptr(att_dst), _ptr(s_src), _ptr(s_dst),
                                          _ptr(msg_scale), _ptr(msg_out), _ptr(addend), _ptr(w_second), _ptr(out_second),
                                          C.byref(ch) if ch is not None else None, _stream()))
    if ch is not None:
        return out, co1, co2
    if w_second is not None:
        return out, out_second
    return (out, s_src, s_dst) if heads else out


@dataclass
class DeviceLayer:
    agg: int
    d_in: int
    d_out: int
    act: int
    w_self: Optional[torch.Tensor]
    w_nbr: torch.Tensor
    bias: Optional[torch.Tensor]
    heads: int = 1
    leaky_slope: float = 0.2
    att_src: Optional[torch.Tensor] = None
    att_dst: Optional[torch.Tensor] = None
    w_edge: Optional[torch.Tensor] = None


def _layer_array(layers: List[DeviceLayer]):
    arr = (itb_layer * len(layers))()
    for i, l in enumerate(layers):
        arr[i] = itb_layer(l.agg, l.d_in, l.d_out, l.act, l.heads, l.leaky_slope,
                           l.w_self.data_ptr() if l.w_self is not None else None, l.w_nbr.data_ptr(),
                           l.bias.data_ptr() if l.bias is not None else None,
                           l.att_src.data_ptr() if l.att_src is not None else None,
                           l.att_dst.data_ptr() if l.att_dst is not None else None,
                           l.w_edge.data_ptr() if l.w_edge is not None else None)
    return arr


def infer_layer_plan(layers: List["DeviceLayer"], dtype) -> List[int]:
    """The evaluation order the library takes for every layer (PLAN_* codes)."""
    arr = _layer_array(layers)
    plan = (C.c_int32 * len(layers))()
    _check("infer_layer_plan", lib.infer_layer_plan(ITB_BF16 if dtype in (torch.bfloat16, "bf16") else ITB_F32, len(layers), arr, plan))
    return list(plan)


def infer_workspace_bytes(n_nodes, n_edges, split: Optional[Split], dtype, layers: List[DeviceLayer], edge_chunk=0,
                          edge_dim=0) -> int:
    arr = _layer_array(layers)
    sp = split.c_struct() if split is not None else None
    need = C.c_size_t(0)
    _check("infer_full_graph(size)", lib.infer_full_graph(n_nodes, n_edges, None, None, None,
                                                          C.byref(sp) if sp is not None else None,
                                                          ITB_BF16 if dtype == torch.bfloat16 else ITB_F32, len(layers), arr,
                                                          None, None, edge_chunk, None, edge_dim, None, C.byref(need), None,
                                                          None))
    return need.value


def infer_full_graph(rowptr, col, deg_out, split: Optional[Split], layers: List[DeviceLayer], x,
                     out: Optional[torch.Tensor] = None, edge_chunk: int = 0, workspace: Optional[torch.Tensor] = None,
                     events=None, edge_feat: Optional[torch.Tensor] = None):
    """``events``: optional list of torch.cuda.Event objects (timing enabled, each recorded once so that its handle
    exists), four per layer, which the call records at layer begin / before gather / after gather / layer end."""
    n = x.shape[0]
    e = col.numel()
    if out is None:
        out = torch.empty((n, layers[-1].d_out), dtype=x.dtype, device="cuda")
    arr = _layer_array(layers)
    sp = split.c_struct() if split is not None else None
    spp = C.byref(sp) if sp is not None else None
    edge_dim = edge_feat.shape[1] if edge_feat is not None else 0
    if workspace is None:
        workspace = _workspace(infer_workspace_bytes(n, e, split, x.dtype, layers, edge_chunk, edge_dim))
    size = C.c_size_t(workspace.numel())
    evp = None
    if events:
        handles = (C.c_void_p * len(events))(*[ev.cuda_event for ev in events])
        evs = itb_stage_events(handles, len(events))
        evp = C.byref(evs)
    _check("infer_full_graph", lib.infer_full_graph(n, e, _ptr(rowptr), _ptr(col), _ptr(deg_out), spp, dtype_code(x),
                                                    len(layers), arr, _ptr(x), _ptr(out), edge_chunk, _ptr(edge_feat), edge_dim,
                                                    _ptr(workspace), C.byref(size), evp, _stream()))
    return out


# --------------------------------------------------------------------------------------------
def to_device(a, dtype: str = "f32"):
    """numpy stored tensor (fp32 array or bf16 bits as uint16) -> device tensor."""
    import numpy as np
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_numpy(t: torch.Tensor):
    """device tensor -> numpy stored tensor (bf16 as uint16 bits)."""
    import numpy as np
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def device_layers(layers) -> List[DeviceLayer]:
    """Upload workload layers (numpy) to the device."""
    out = []
    for l in layers:
        out.append(DeviceLayer(l.agg, l.d_in, l.d_out, l.act, to_device(l.w_self), to_device(l.w_nbr), to_device(l.bias),
                               l.heads, l.leaky_slope, to_device(l.att_src), to_device(l.att_dst),
                               to_device(getattr(l, "w_edge", None))))
    return out

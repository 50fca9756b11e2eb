"""CPU oracle (fp64, per-vertex) for the Gather-Apply-Scatter layer.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg.  It never imports the HIP package and the HIP
package never imports it.

The arithmetic lives in ``gas_oracle.c`` (plain C, compiled with gcc by
``oracle.build()``); this file marshals numpy arrays and strings the per-layer
calls together in the order of the paper's layer loop (Sec. IV-C: k supersteps
for a k-layer model, h^0 = x).

Stored tensors: fp32 arrays, or bf16 bit patterns in ``uint16`` arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libgas_oracle.so")
_lib = None

SUM, MEAN, GCN, GAT, MAX, MIN, NONE = 0, 1, 2, 3, 4, 5, 6
ACT_NONE, ACT_RELU = 0, 1


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc (OpenMP over vertices)."""
    src = os.path.join(_HERE, "gas_oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", _SO, src, "-lm"])
    return _SO


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_SO)
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    """Numeric fp32 view of a stored tensor (bf16 bits widen exactly)."""
    if a is None:
        return None
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (np.ascontiguousarray(a).astype(np.uint32) << np.uint32(16)).view(np.float32)
    return np.ascontiguousarray(a, dtype=np.float32)


def set_threads(n: int = 0) -> int:
    return int(lib().oracle_set_threads(C.c_int(n)))


# ------------------------------------------------------------------ integer steps
def hub_threshold(total_edges, total_workers, lam=(1, 10)):
    """floor(lambda * E / W) with lambda = num/den (Sec. IV-D heuristic), at least 1."""
    t = C.c_int64(0)
    rc = lib().oracle_hub_threshold(C.c_int64(total_edges), C.c_int64(total_workers), C.c_int64(lam[0]), C.c_int64(lam[1]),
                                    C.byref(t))
    if rc != 0:
        raise ValueError("oracle_hub_threshold: bad arguments")
    return t.value


def build_csr(n_nodes, src, dst):
    src, dst = _i32(src), _i32(dst)
    e = len(src)
    rowptr = np.zeros(n_nodes + 1, dtype=np.int64)
    col = np.zeros(e, dtype=np.int32)
    deg_out = np.zeros(n_nodes, dtype=np.int32)
    rc = lib().oracle_build_csr(C.c_int64(n_nodes), C.c_int64(e), _p(src, C.c_int32), _p(dst, C.c_int32),
                                _p(rowptr, C.c_int64), _p(col, C.c_int32), _p(deg_out, C.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_build_csr failed: {rc}")
    return rowptr, col, deg_out


def split_hubs(rowptr, threshold):
    rowptr = _i64(rowptr)
    n = len(rowptr) - 1
    nh, ns = C.c_int64(0), C.c_int64(0)
    rc = lib().oracle_split_hubs(C.c_int64(n), _p(rowptr, C.c_int64), C.c_int64(threshold),
                                 C.byref(nh), C.byref(ns), None, None, None, None, None)
    if rc != 0:
        raise ValueError(f"oracle_split_hubs failed: {rc}")
    h, s = nh.value, ns.value
    out = dict(hub_ids=np.zeros(h, np.int32), hub_shadow_off=np.zeros(h + 1, np.int64),
               shadow_begin=np.zeros(s, np.int64), shadow_end=np.zeros(s, np.int64),
               shadow_owner=np.zeros(s, np.int32))
    rc = lib().oracle_split_hubs(C.c_int64(n), _p(rowptr, C.c_int64), C.c_int64(threshold),
                                 C.byref(nh), C.byref(ns), _p(out["hub_ids"], C.c_int32),
                                 _p(out["hub_shadow_off"], C.c_int64), _p(out["shadow_begin"], C.c_int64),
                                 _p(out["shadow_end"], C.c_int64), _p(out["shadow_owner"], C.c_int32))
    assert rc == 0
    out["n_hubs"], out["n_shadows"] = h, s
    return out


# ------------------------------------------------------------------ feature steps
def gather(agg, rowptr, col, h, deg_out=None, verts=None):
    """fp64 aggregate per vertex; ``h`` is a stored tensor [N x D]."""
    rowptr, col, hf = _i64(rowptr), _i32(col), _f32(h)
    n, d = hf.shape
    vs = None if verts is None else _i64(verts)
    out = np.zeros((n if vs is None else len(vs), d), dtype=np.float64)
    do = None if deg_out is None else _i32(deg_out)
    rc = lib().oracle_gather(C.c_int(agg), C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32),
                             C.c_int64(d), _p(hf, C.c_float), _p(do, C.c_int32),
                             _p(vs, C.c_int64), C.c_int64(0 if vs is None else len(vs)), _p(out, C.c_double))
    if rc != 0:
        raise ValueError(f"oracle_gather failed: {rc}")
    return out


def gather_weighted(agg, rowptr, col, h, edge_w, verts=None):
    """fp64 aggregate of edge-weighted messages w_e * h[col[e]] (SUM or MEAN); ``edge_w`` is [E] fp32 in CSR order."""
    rowptr, col, hf = _i64(rowptr), _i32(col), _f32(h)
    n, d = hf.shape
    w = np.ascontiguousarray(edge_w, dtype=np.float32)
    assert len(w) == len(col)
    vs = None if verts is None else _i64(verts)
    out = np.zeros((n if vs is None else len(vs), d), dtype=np.float64)
    rc = lib().oracle_gather_weighted(C.c_int(agg), C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32),
                                      C.c_int64(d), _p(hf, C.c_float), _p(w, C.c_float),
                                      _p(vs, C.c_int64), C.c_int64(0 if vs is None else len(vs)), _p(out, C.c_double))
    if rc != 0:
        raise ValueError(f"oracle_gather_weighted failed: {rc}")
    return out


def gather_edge_features(agg, rowptr, col, h, edge_feat, w_edge, deg_out=None, verts=None):
    """fp64 aggregate of messages h[u] + ef[e] . W_e (SUM, MEAN or GCN); ``edge_feat`` is a stored tensor [E x d_e]
    in CSR order, ``w_edge`` a stored tensor [d_e x D]."""
    rowptr, col, hf = _i64(rowptr), _i32(col), _f32(h)
    n, d = hf.shape
    ef, we = _f32(edge_feat), _f32(w_edge)
    assert ef.shape[0] == len(col) and we.shape == (ef.shape[1], d)
    vs = None if verts is None else _i64(verts)
    out = np.zeros((n if vs is None else len(vs), d), dtype=np.float64)
    do = None if deg_out is None else _i32(deg_out)
    rc = lib().oracle_gather_edge_features(C.c_int(agg), C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32),
                                           C.c_int64(d), _p(hf, C.c_float), _p(do, C.c_int32),
                                           C.c_int64(ef.shape[1]), _p(ef, C.c_float), _p(we, C.c_float),
                                           _p(vs, C.c_int64), C.c_int64(0 if vs is None else len(vs)), _p(out, C.c_double))
    if rc != 0:
        raise ValueError(f"oracle_gather_edge_features failed: {rc}")
    return out


def gather_split(agg, rowptr, col, h, split, deg_out=None):
    """Same aggregate computed through the shadow segments; returns (agg, edge_count)."""
    rowptr, col, hf = _i64(rowptr), _i32(col), _f32(h)
    n, d = hf.shape
    out = np.zeros((n, d), dtype=np.float64)
    cnt = np.zeros(n, dtype=np.int64)
    do = None if deg_out is None else _i32(deg_out)
    rc = lib().oracle_gather_split(C.c_int(agg), C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32),
                                   C.c_int64(d), _p(hf, C.c_float), _p(do, C.c_int32),
                                   C.c_int64(split["n_hubs"]), _p(_i32(split["hub_ids"]), C.c_int32),
                                   _p(_i64(split["hub_shadow_off"]), C.c_int64),
                                   _p(_i64(split["shadow_begin"]), C.c_int64),
                                   _p(_i64(split["shadow_end"]), C.c_int64),
                                   _p(out, C.c_double), _p(cnt, C.c_int64))
    if rc != 0:
        raise ValueError(f"oracle_gather_split failed: {rc}")
    return out, cnt


def apply(h_self, agg, w_self, w_nbr, bias, act):
    """fp64 dense update per vertex; all tensor arguments are stored tensors."""
    af = _f32(agg)
    n, d_in = af.shape
    wn = _f32(w_nbr)
    d_out = wn.shape[1]
    hs, ws = _f32(h_self), _f32(w_self)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    out = np.zeros((n, d_out), dtype=np.float64)
    rc = lib().oracle_apply(C.c_int64(n), C.c_int64(d_in), C.c_int64(d_out), _p(hs, C.c_float),
                            _p(af, C.c_float), _p(ws, C.c_float), _p(wn, C.c_float), _p(b, C.c_float),
                            C.c_int(act), _p(out, C.c_double))
    if rc != 0:
        raise ValueError(f"oracle_apply failed: {rc}")
    return out


def gat_scores(z64, att):
    z64 = np.ascontiguousarray(z64, dtype=np.float64)
    att = np.ascontiguousarray(att, dtype=np.float32)
    heads, dh = att.shape
    n = z64.shape[0]
    s = np.zeros((n, heads), dtype=np.float64)
    rc = lib().oracle_gat_scores(C.c_int64(n), C.c_int64(heads), C.c_int64(dh), _p(z64, C.c_double),
                                 _p(att, C.c_float), _p(s, C.c_double))
    assert rc == 0
    return s


def gat_gather(rowptr, col, z, s_src, s_dst, heads, slope=0.2, verts=None):
    rowptr, col, zf = _i64(rowptr), _i32(col), _f32(z)
    n, dim = zf.shape
    ss = np.ascontiguousarray(s_src, dtype=np.float32)
    sd = np.ascontiguousarray(s_dst, dtype=np.float32)
    vs = None if verts is None else _i64(verts)
    out = np.zeros((n if vs is None else len(vs), dim), dtype=np.float64)
    rc = lib().oracle_gat_gather(C.c_int64(n), _p(rowptr, C.c_int64), _p(col, C.c_int32),
                                 C.c_int64(heads), C.c_int64(dim // heads), C.c_double(slope),
                                 _p(zf, C.c_float), _p(ss, C.c_float), _p(sd, C.c_float),
                                 _p(vs, C.c_int64), C.c_int64(0 if vs is None else len(vs)), _p(out, C.c_double))
    assert rc == 0
    return out


# ------------------------------------------------------------------ storage rounding
def round_store(x64, dtype):
    """Round fp64 results once to the storage dtype: 'f32' -> float32 array,
    'bf16' -> uint16 bit patterns (round to nearest even)."""
    x64 = np.ascontiguousarray(x64, dtype=np.float64)
    if dtype == "f32":
        return x64.astype(np.float32)
    out = np.zeros(x64.shape, dtype=np.float32)
    rc = lib().oracle_round_bf16(C.c_int64(x64.size), _p(x64, C.c_double), _p(out, C.c_float))
    assert rc == 0
    return (out.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# ------------------------------------------------------------------ whole layers
def dense_layer(rowptr, col, deg_out, h, layer, dtype, verts=None, round_agg=False, return_agg64=False, edge_feat=None):
    """One SAGE/GCN-style layer: gather (sum, mean, degree-normalised sum, max or min), then apply: Eq. (1) in fp64
    with no intermediate rounding, whatever order or storage an implementation uses between the two steps.
    Returns (agg_stored, y64) -- agg_stored is the aggregate rounded to the storage dtype, for stage-wise checks --
    and with ``return_agg64`` also the unrounded aggregate.  A layer without a gather (NONE: encoder before the first
    round, prediction head after the last, Sec. IV-C) is the update of the vertex's own state alone: (None, y64).
    ``round_agg=True`` evaluates the update on the ROUNDED aggregate instead: the arithmetic of an implementation
    that stores agg(h) in the storage dtype between gather and update (kept for stage-wise comparisons; it is not
    the yardstick of a layer)."""
    if layer.agg == NONE:
        hs = h if verts is None else np.asarray(h)[np.asarray(verts)]
        y = apply(None, hs, None, layer.w_nbr, layer.bias, layer.act)
        return (None, y, None) if return_agg64 else (None, y)
    if getattr(layer, "w_edge", None) is not None:
        # messages carry the edge's feature vector: m_e = h[u] + ef[e] . W_e (``edge_feat`` [E x d_e], CSR order)
        a64 = gather_edge_features(layer.agg, rowptr, col, h, edge_feat, layer.w_edge, deg_out=deg_out, verts=verts)
    else:
        a64 = gather(layer.agg, rowptr, col, h, deg_out=deg_out, verts=verts)
    a_st = round_store(a64, dtype)
    hs = h if verts is None else np.asarray(h)[np.asarray(verts)]
    if layer.w_self is None:      # no self matrix: the update sees the aggregate only
        hs = None
    if round_agg:
        y64 = apply(hs, a_st, layer.w_self, layer.w_nbr, layer.bias, layer.act)
    else:
        # same update on the unrounded aggregate; apply() takes fp32 storage, so the neighbour product is done here
        y64 = apply(hs, np.zeros_like(_f32(a_st)), layer.w_self, layer.w_nbr, layer.bias, ACT_NONE)
        y64 = y64 + a64 @ _f32(layer.w_nbr).astype(np.float64)
        if layer.act == ACT_RELU:
            y64 = np.maximum(y64, 0.0)
    return (a_st, y64, a64) if return_agg64 else (a_st, y64)


def gat_layer(rowptr, col, h, layer, dtype, verts=None):
    """One GAT layer in the order project -> softmax-reduce -> bias -> activation.
    Returns (z_stored, s_src32, s_dst32, y64)."""
    z64 = apply(None, h, None, layer.w_nbr, None, ACT_NONE)
    s_src = gat_scores(z64, layer.att_src).astype(np.float32)
    s_dst = gat_scores(z64, layer.att_dst).astype(np.float32)
    z_st = round_store(z64, dtype)
    o64 = gat_gather(rowptr, col, z_st, s_src, s_dst, layer.heads, layer.leaky_slope, verts=verts)
    y64 = o64 + layer.bias.astype(np.float64)[None, :]
    if layer.act == ACT_RELU:
        y64 = np.maximum(y64, 0.0)
    return z_st, s_src, s_dst, y64


def infer_full_graph(rowptr, col, deg_out, x, layers, dtype, return_all=False, edge_feat=None):
    """L layers over every vertex, h^0 = x; each layer's output is rounded once
    to the storage dtype before the next layer reads it.  ``edge_feat`` ([E x d_e], CSR order) feeds the layers
    that have an edge matrix ``w_edge``."""
    h = x
    outs = []
    for layer in layers:
        if layer.agg == GAT:
            y64 = gat_layer(rowptr, col, h, layer, dtype)[3]
        else:
            y64 = dense_layer(rowptr, col, deg_out, h, layer, dtype, edge_feat=edge_feat)[1]
        h = round_store(y64, dtype)
        outs.append(h)
    return outs if return_all else h

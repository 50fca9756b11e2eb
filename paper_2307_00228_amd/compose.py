"""The layer loop of ``infer_full_graph`` issued call by call through the C ABI.

Same kernels, same order, same strategy choices as the single call (the results are bitwise identical, which
the tests assert); it exists so that the benchmark can bracket each gather with events and the stage-wise
parity tests can look at every intermediate tensor.  It allocates torch tensors for the intermediates and does
nothing else: every step of the path runs inside the library.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, List, Optional

import torch

from . import binding as B


@dataclass
class LayerTrace:
    gather_src: torch.Tensor        # rows the gather read (state, message rows, or projected rows)
    agg: torch.Tensor               # gather output (GAT and projected layers: the new state)
    out: Optional[torch.Tensor]     # new state; None for a layer whose update is chained into the next layer's projection
    projected: bool                 # W_nbr applied before the gather, update fused into the gather's epilogue
    scores: Optional[tuple] = None  # GAT: (s_src, s_dst)
    self_product: Optional[torch.Tensor] = None   # projected layers: h . W_self, the addend of the gather's epilogue
    edge_term: Optional[torch.Tensor] = None      # layers with an edge matrix: (reduced edge features) . W_e


def plan(layers, dtype) -> List[bool]:
    """Which layers apply W_nbr before their gather: asked of the library (infer_layer_plan), not decided here."""
    return [p == B.PLAN_PROJECT_GATHER for p in B.infer_layer_plan(layers, dtype)]


def chained(layers, dtype) -> List[bool]:
    """Which layers' updates also produce the next layer's h . [W_nbr | W_self] (and never store their own state)."""
    return [p == B.PLAN_GATHER_UPDATE_CHAINED for p in B.infer_layer_plan(layers, dtype)]


def run_layers(rowptr, col, deg_out, split, layers: List[B.DeviceLayer], x: torch.Tensor,
               mark: Optional[Callable[[str, int], None]] = None, buffers: Optional[dict] = None,
               edge_feat: Optional[torch.Tensor] = None) -> List[LayerTrace]:
    """``mark(tag, layer)`` is called right before/after the gather and the update of every layer
    (tags: gather_begin, gather_end, apply_begin, apply_end; for sum/mean/GCN layers also project_begin, project_end around
    the optional projection before the gather).  ``buffers`` caches the intermediates across calls."""
    mark = mark or (lambda tag, i: None)
    buffers = buffers if buffers is not None else {}
    n = x.shape[0]

    def buf(key, cols, dtype=x.dtype):
        t = buffers.get(key)
        if t is None or t.shape != (n, cols) or t.dtype != dtype:
            t = torch.empty((n, cols), dtype=dtype, device="cuda")
            buffers[key] = t
        return t

    sd = coef = None
    if any(l.agg == B.AGG_GCN for l in layers):
        ss, sd = B.gcn_norm_scales(rowptr, deg_out)
        cb = buffers.get("edge_coef")
        coef = B.gcn_edge_coefficients(col, ss, out=cb if cb is not None and cb.numel() == col.numel() else None)
        buffers["edge_coef"] = coef
    # edge features are reduced per destination once per aggregator that a layer with an edge matrix uses
    edge_sums = {}
    for l in layers:
        if l.w_edge is not None and l.agg not in edge_sums:
            edge_sums[l.agg] = B.aggregate_edge_features(l.agg, rowptr, edge_feat, split, edge_coef=coef if l.agg == B.AGG_GCN else None,
                                                         dst_scale=sd if l.agg == B.AGG_GCN else None)
    traces = []
    h = x
    projected = plan(layers, x.dtype)
    chain = chained(layers, x.dtype)
    handed_over = None   # (h . W_nbr, h . W_self) of this layer, produced by the previous layer's update
    # a projected last layer whose width is not whole 16-byte pieces runs on zero-padded copies of its matrices and bias
    piece = 8 if x.dtype == torch.bfloat16 else 4
    last = layers[-1]
    dp_last = (last.d_out + piece - 1) // piece * piece
    padded = None
    if projected[-1] and dp_last != last.d_out:
        padded = (B.copy_columns(last.w_nbr, dp_last), B.copy_columns(last.w_self, dp_last),
                  B.copy_columns(last.bias.view(1, -1), dp_last).view(-1) if last.bias is not None else None)
    for i, l in enumerate(layers):
        gcn, gat = l.agg == B.AGG_GCN, l.agg == B.AGG_GAT
        out = buf(("out", i), l.d_out) if not chain[i] else None
        if l.agg == B.AGG_NONE:       # encoder / prediction head: the update alone
            mark("gather_begin", i)
            mark("gather_end", i)
            mark("apply_begin", i)
            B.apply_layer(None, h, None, l.w_nbr, l.bias, l.act, out=out)
            mark("apply_end", i)
            traces.append(LayerTrace(h, h, out, False))
            h = out
            continue
        if gat:
            mark("apply_begin", i)
            z, s_src, s_dst = B.apply_layer(None, h, None, l.w_nbr, None, B.ACT_NONE, out=buf(("z", i), l.d_out), heads=l.heads,
                                            att_src=l.att_src, att_dst=l.att_dst)
            mark("apply_end", i)
            mark("gather_begin", i)
            B.gather_layer(l.agg, rowptr, col, z, split, s_src, s_dst, heads=l.heads, leaky_slope=l.leaky_slope, act=l.act,
                           bias=l.bias, out=out)
            mark("gather_end", i)
            traces.append(LayerTrace(z, out, out, False, (s_src, s_dst)))
            h = out
            continue
        if projected[i]:
            # h . [W_nbr | W_self] in one launch, then the gather of the first product with the update in its epilogue
            mark("project_begin", i)
            pad = padded if i == len(layers) - 1 else None
            width = dp_last if pad else l.d_out
            w_nbr, w_self, bias = pad if pad else (l.w_nbr, l.w_self, l.bias)
            if handed_over is not None:
                proj, selfp = handed_over
                handed_over = None
            else:
                proj, selfp = B.apply_layer(None, h, None, w_nbr, None, B.ACT_NONE, out=buf(("proj", i), width),
                                            w_second=w_self, out_second=buf(("selfp", i), width))
            mark("project_end", i)
            mark("gather_begin", i)
            wide = buf(("padded_out", i), width) if pad else out
            B.gather_layer(l.agg, rowptr, col, proj, split, None, sd if gcn else None, out=wide,
                           edge_coef=coef if gcn else None, addend=selfp, bias=bias, act=l.act)
            if pad:
                B.copy_columns(wide, l.d_out, out=out)       # drop the padding columns
            mark("gather_end", i)
            mark("apply_begin", i)
            mark("apply_end", i)
            traces.append(LayerTrace(proj, out, out, True, None, selfp))
            h = out
            continue
        mark("project_begin", i)
        edge_term = None
        if l.w_edge is not None:
            edge_term = B.apply_layer(None, edge_sums[l.agg], None, l.w_edge, None, B.ACT_NONE, out=buf(("edge", i), l.d_in))
        mark("project_end", i)
        mark("gather_begin", i)
        agg = B.gather_layer(l.agg, rowptr, col, h, split, None, sd if gcn else None, out=buf(("agg", i), h.shape[1]),
                             edge_coef=coef if gcn else None, addend=edge_term)
        mark("gather_end", i)
        mark("apply_begin", i)
        if chain[i]:
            nxt = layers[i + 1]
            nxt_pad = padded if i + 1 == len(layers) - 1 else None
            nw, ns, nwidth = (nxt_pad[0], nxt_pad[1], dp_last) if nxt_pad else (nxt.w_nbr, nxt.w_self, nxt.d_out)
            _, p1, p2 = B.apply_layer(h if l.w_self is not None else None, agg, l.w_self, l.w_nbr, l.bias, l.act,
                                      chain=(nw, ns, buf(("proj", i + 1), nwidth), buf(("selfp", i + 1), nwidth)),
                                      store_out=False)
            handed_over = (p1, p2)
            out = None
        else:
            B.apply_layer(h if l.w_self is not None else None, agg, l.w_self, l.w_nbr, l.bias, l.act, out=out)
        mark("apply_end", i)
        traces.append(LayerTrace(h, agg, out, False, None, None, edge_term))
        h = out
    return traces

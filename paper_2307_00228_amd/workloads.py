"""Seeded synthetic inputs: graphs, features and weights.

This module only *draws inputs*. It holds none of the method's arithmetic (no
CSR construction, no degree normalisation, no aggregation, no dense update) and
imports neither the HIP binding nor the CPU oracle; both of those consume the
arrays produced here.

The workloads stand in for the paper's synthetic Power-Law graphs (Sec. V-A,
Tab. I: about ten edges per node, in-degree following a power law) and for its
hub experiment (Sec. V-B, partial-gather analysis).  The real-world datasets of
Tab. I are not reproduced.

All randomness: numpy ``Generator(PCG64(SeedSequence([seed, tag])))`` with one
sub-stream per purpose (topology, features, weights), so a workload is a pure
function of (name, scale, seed).  Large arrays are drawn in fixed-size chunks,
each from its own child stream (``Generator.spawn``), by a small thread pool:
the result does not depend on the number of threads, and the 2e9-edge workload
is generated in about a minute instead of several.

bf16 tensors are carried as ``uint16`` bit patterns (numpy has no bf16).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

_POOL = None


def _pool() -> ThreadPoolExecutor:
    """Worker threads for the chunked draws (numpy releases the GIL in its fill, sort and gather loops)."""
    global _POOL
    if _POOL is None:
        _POOL = ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1)))
    return _POOL


def _chunks(n: int, step: int):
    return [(i, min(i + step, n)) for i in range(0, n, step)]

F32 = "f32"
BF16 = "bf16"

AGG_SUM, AGG_MEAN, AGG_GCN, AGG_GAT, AGG_MAX, AGG_MIN, AGG_NONE = 0, 1, 2, 3, 4, 5, 6
ACT_NONE, ACT_RELU = 0, 1


# ----------------------------------------------------------------------------
# bf16 <-> fp32 bit plumbing (storage format only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_f32(a: np.ndarray) -> np.ndarray:
    """Numeric fp32 view of a stored tensor (fp32 array or bf16 bit array)."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a)
    return np.ascontiguousarray(a, dtype=np.float32)


def store(a: np.ndarray, dtype: str) -> np.ndarray:
    """Put numeric fp32 data into its storage format."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return f32_to_bf16_bits(a) if dtype == BF16 else a


# ----------------------------------------------------------------------------
# containers
# ----------------------------------------------------------------------------
@dataclass
class Layer:
    agg: int                 # AGG_*
    d_in: int
    d_out: int
    act: int                 # ACT_*
    w_self: Optional[np.ndarray]   # [d_in, d_out] storage dtype (None for GAT)
    w_nbr: np.ndarray              # [d_in, d_out] storage dtype (GAT: the projection W)
    bias: np.ndarray               # [d_out] fp32
    heads: int = 1
    att_src: Optional[np.ndarray] = None   # [heads, d_out/heads] fp32 (GAT)
    att_dst: Optional[np.ndarray] = None
    leaky_slope: float = 0.2
    w_edge: Optional[np.ndarray] = None    # [d_e, d_in] storage dtype: messages h[u] + ef[e] . W_e (sum / mean / GCN layers)


@dataclass
class Workload:
    name: str
    n_nodes: int
    n_edges: int
    src: np.ndarray          # int32 [E]
    dst: np.ndarray          # int32 [E]
    x: np.ndarray            # [N, d0] storage dtype
    dtype: str               # F32 | BF16
    threshold: int           # hub threshold on in-degree (huge => no split)
    layers: List[Layer] = field(default_factory=list)
    recipe: str = ""


def _rng(seed: int, tag: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tag])))


# ----------------------------------------------------------------------------
# topology recipes
# ----------------------------------------------------------------------------
def zipf_rank_destinations(rng, n_nodes: int, n_edges: int, s: float) -> np.ndarray:
    """dst ids whose rank r (1..N) is drawn with P(r) ~ r^-s; rank->id by a random permutation."""
    w = np.arange(1, n_nodes + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    ranks = np.searchsorted(cdf, rng.random(n_edges), side="right")
    ranks = np.minimum(ranks, n_nodes - 1)
    perm = rng.permutation(n_nodes).astype(np.int32)
    return perm[ranks]


def power_law_degree_sequence(rng, n_nodes: int, total: int, exponent: float, d_max: int) -> np.ndarray:
    """Degree sequence with P(d) ~ d^-exponent on 1..d_max, rescaled and topped up to sum == total."""
    if n_nodes == 0:
        return np.zeros(0, dtype=np.int64)
    d = np.arange(1, d_max + 1, dtype=np.float64)
    cdf = np.cumsum(d ** (-exponent))
    cdf /= cdf[-1]
    u = rng.random(n_nodes)
    deg = np.empty(n_nodes, dtype=np.int64)

    def look_up(span):
        deg[span[0]:span[1]] = 1 + np.searchsorted(cdf, u[span[0]:span[1]], side="right")

    list(_pool().map(look_up, _chunks(n_nodes, 1 << 22)))
    del u
    deg = np.minimum(deg, d_max)
    s = int(deg.sum())
    if s > 0 and s != total:
        deg = np.minimum(np.floor(deg * (total / s)).astype(np.int64), d_max)
    diff = total - int(deg.sum())
    while diff != 0:
        k = min(abs(diff), n_nodes)
        idx = rng.choice(n_nodes, size=k, replace=False)
        if diff > 0:
            deg[idx] += 1
            diff -= k
        else:
            ok = idx[deg[idx] > 0]
            deg[ok] -= 1
            diff += len(ok)
    return deg


def destinations_from_degrees(rng, deg_by_slot: np.ndarray, n_nodes: int) -> np.ndarray:
    """Expand a degree sequence into a dst list; slot -> node id by a random permutation."""
    ids = rng.permutation(n_nodes).astype(np.int32)[: len(deg_by_slot)]
    total = int(deg_by_slot.sum())
    if total <= (1 << 27):
        return np.repeat(ids, deg_by_slot)
    # slot ranges of roughly equal output size, expanded side by side
    ends = np.cumsum(deg_by_slot)
    cuts = np.searchsorted(ends, np.linspace(0, total, 65)[1:-1], side="left")
    bounds = np.unique(np.concatenate([[0], cuts, [len(deg_by_slot)]]))
    out = np.empty(total, dtype=np.int32)

    def expand(k):
        a, b = int(bounds[k]), int(bounds[k + 1])
        o0 = int(ends[a - 1]) if a > 0 else 0
        out[o0:int(ends[b - 1])] = np.repeat(ids[a:b], deg_by_slot[a:b])

    list(_pool().map(expand, range(len(bounds) - 1)))
    return out


def shuffle_edges(rng, src: np.ndarray, dst: np.ndarray, log=None):
    """Deliver the edge list unsorted.  Up to 2^27 edges: one uniform permutation.  Beyond that (where a single
    permutation would take minutes and tens of GB): a stride-64 interleave followed by an independent uniform
    permutation inside each of the 64 parts -- every part draws from the whole destination range."""
    e = len(src)
    if e <= (1 << 27):
        p = rng.permutation(e)
        return np.ascontiguousarray(src[p]), np.ascontiguousarray(dst[p])
    parts = 64
    out_s, out_d = np.empty_like(src), np.empty_like(dst)
    sizes = [len(range(k, e, parts)) for k in range(parts)]
    starts = np.concatenate([[0], np.cumsum(sizes)])
    streams = rng.spawn(parts)
    done = []

    def one(k):
        s_k, d_k = src[k::parts], dst[k::parts]
        p = streams[k].permutation(len(s_k))
        out_s[starts[k]:starts[k + 1]] = s_k[p]
        out_d[starts[k]:starts[k + 1]] = d_k[p]
        done.append(k)
        if log and len(done) % 16 == 0:
            log(f"  shuffle: {len(done)}/{parts} parts")

    list(_pool().map(one, range(parts)))
    return out_s, out_d


# ----------------------------------------------------------------------------
# features and weights
# ----------------------------------------------------------------------------
def normal_features(rng, n: int, d: int, dtype: str, log=None) -> np.ndarray:
    """N(0,1) features in the storage dtype, drawn and rounded chunk by chunk (bounded temporary memory)."""
    out = np.empty((n, d), dtype=np.uint16 if dtype == BF16 else np.float32)
    spans = _chunks(n, max(1, (1 << 22) // max(d, 1)))
    streams = rng.spawn(len(spans))
    done = []

    def fill(k):
        a, b = spans[k]
        out[a:b] = store(streams[k].standard_normal((b - a, d), dtype=np.float32), dtype)
        done.append(k)
        if log and len(done) % 256 == 0:
            log(f"  features: {len(done)}/{len(spans)} chunks")

    list(_pool().map(fill, range(len(spans))))
    return out


def glorot(rng, fan_in: int, fan_out: int, shape, dtype: str) -> np.ndarray:
    a = np.sqrt(6.0 / (fan_in + fan_out))
    return store(rng.uniform(-a, a, size=shape).astype(np.float32), dtype)


def dense_layers(rng, agg, dims, dtype: str, bias_random: bool = False) -> List[Layer]:
    """``agg`` is one aggregator for every layer or a sequence with one entry per layer; an AGG_NONE entry is a
    per-vertex layer (encoder / prediction head) that has no self matrix."""
    layers = []
    kinds = [agg] * (len(dims) - 1) if isinstance(agg, int) else list(agg)
    assert len(kinds) == len(dims) - 1
    for i in range(len(dims) - 1):
        di, do = dims[i], dims[i + 1]
        b = (rng.uniform(-0.1, 0.1, size=do).astype(np.float32) if bias_random
             else np.zeros(do, dtype=np.float32))
        w_self = glorot(rng, di, do, (di, do), dtype)
        layers.append(Layer(agg=kinds[i], d_in=di, d_out=do,
                            act=ACT_RELU if i < len(dims) - 2 else ACT_NONE,
                            w_self=None if kinds[i] == AGG_NONE else w_self,
                            w_nbr=glorot(rng, di, do, (di, do), dtype),
                            bias=b))
    return layers


def gat_layers(rng, dims, heads: int, dtype: str, bias_random: bool = False) -> List[Layer]:
    layers = []
    for i in range(len(dims) - 1):
        di, do = dims[i], dims[i + 1]
        dh = do // heads
        a = np.sqrt(6.0 / (dh + 1))
        b = (rng.uniform(-0.1, 0.1, size=do).astype(np.float32) if bias_random
             else np.zeros(do, dtype=np.float32))
        layers.append(Layer(agg=AGG_GAT, d_in=di, d_out=do,
                            act=ACT_RELU if i < len(dims) - 2 else ACT_NONE,
                            w_self=None, w_nbr=glorot(rng, di, do, (di, do), dtype), bias=b,
                            heads=heads,
                            att_src=rng.uniform(-a, a, size=(heads, dh)).astype(np.float32),
                            att_dst=rng.uniform(-a, a, size=(heads, dh)).astype(np.float32)))
    return layers


# ----------------------------------------------------------------------------
# the named workloads
# ----------------------------------------------------------------------------
NO_SPLIT = 1 << 62

NAMES = ("tiny_powerlaw", "medium_uniform", "hub_heavy", "hub_heavy_uniform_control",
         "attention", "huge_share", "huge_share_slice")


def make(name: str, scale: float = 1.0, seed: int = 0, bias_random: bool = False,
         features: bool = True, log=None) -> Workload:
    """Build a named workload.  ``scale`` shrinks node and edge counts together
    (hub sizes and thresholds shrink with it) for parity tests; 1.0 is the full size.
    ``log`` (e.g. ``print``) receives a line per generation stage of the large workloads."""
    topo, feat, wts = _rng(seed, 1), _rng(seed, 2), _rng(seed, 3)
    say = log or (lambda msg: None)

    def sz(v, lo=1):
        return max(lo, int(round(v * scale)))

    if name == "tiny_powerlaw":
        n, e = sz(10_000), sz(100_000)
        dst = zipf_rank_destinations(topo, n, e, 1.2)
        src = topo.integers(0, n, size=e, dtype=np.int32)
        dtype, dims, agg, thr = F32, (64, 64, 16), AGG_MEAN, NO_SPLIT
        recipe = "rank-Zipf(1.2) in-degree, uniform sources, SAGE-mean 64-64-16 fp32, no split"
    elif name == "medium_uniform":
        n, e = sz(1_000_000), sz(20_000_000)
        src = topo.integers(0, n, size=e, dtype=np.int32)
        dst = topo.integers(0, n, size=e, dtype=np.int32)
        dtype, dims, agg, thr = F32, (128, 128, 64), AGG_GCN, NO_SPLIT
        recipe = "uniform src/dst, GCN-normalised sum 128-128-64 fp32"
    elif name in ("hub_heavy", "hub_heavy_uniform_control"):
        n, e = sz(4_000_000, 64), sz(64_000_000, 1024)
        if name == "hub_heavy":
            n_hubs = 16
            hub_deg = np.floor(np.linspace(1_000_000, 4_000_000, n_hubs) * scale).astype(np.int64)
            hub_deg = np.maximum(hub_deg, 1)
            rest = e - int(hub_deg.sum())
            tail = power_law_degree_sequence(topo, n - n_hubs, rest, 2.1, max(2, sz(100_000)))
            deg = np.concatenate([hub_deg, tail])
            dst = destinations_from_degrees(topo, deg, n)
            recipe = "16 planted hubs (1e6..4e6 in-edges) + power-law(2.1) tail, SAGE-mean 128-128-128 bf16, T=4096"
        else:
            dst = topo.integers(0, n, size=e, dtype=np.int32)
            recipe = "uniform-degree control of hub_heavy (same N, E, D, dtype)"
        src = topo.integers(0, n, size=e, dtype=np.int32)
        src, dst = shuffle_edges(topo, src, dst)
        dtype, dims, agg = BF16, (128, 128, 128), AGG_MEAN
        thr = max(4, sz(4096)) if scale < 1.0 else 4096
    elif name == "attention":
        n, e = sz(2_000_000, 16), sz(40_000_000, 64)
        dst = zipf_rank_destinations(topo, n, e, 1.5)
        src = topo.integers(0, n, size=e, dtype=np.int32)
        dtype, dims, agg = BF16, (256, 256, 256, 256), AGG_GAT
        thr = max(4, sz(8192)) if scale < 1.0 else 8192
        recipe = "rank-Zipf(1.5) in-degree, 3-layer GAT 4x64 bf16, T=8192"
    elif name in ("huge_share", "huge_share_slice"):
        if name == "huge_share":
            n, e = sz(100_000_000, 64), sz(2_000_000_000, 1024)
            d_max = max(2, sz(10_000_000))
        else:
            # the shape of huge_share that matters to the address arithmetic -- a state buffer beyond 4 GiB, tens of
            # millions of rows, a hub far above the threshold -- with an edge count that a test can afford
            n, e = sz(50_000_000, 64), sz(250_000_000, 1024)
            d_max = max(2, sz(1_000_000))
        say(f"{name}: degree sequence for {n} vertices")
        deg = power_law_degree_sequence(topo, n, e - d_max, 2.0, d_max)
        deg[0] += d_max
        say(f"{name}: expanding {e} destinations")
        dst = destinations_from_degrees(topo, deg, n)
        del deg
        say(f"{name}: drawing sources")
        src = np.empty(e, dtype=np.int32)
        spans = _chunks(e, 1 << 25)
        streams = topo.spawn(len(spans))

        def draw(k):
            src[spans[k][0]:spans[k][1]] = streams[k].integers(0, n, size=spans[k][1] - spans[k][0], dtype=np.int32)

        list(_pool().map(draw, range(len(spans))))
        say(f"{name}: shuffling the edge list")
        src, dst = shuffle_edges(topo, src, dst, log)
        dtype, dims, agg = BF16, (64, 64, 32), AGG_MEAN
        thr = max(4, sz(16384)) if scale < 1.0 else 16384
        recipe = (f"power-law(2.0) in-degree with one ~{d_max:.0e} hub, SAGE-mean 64-64-32 bf16, T=16384"
                  + (" (half the vertices and an eighth of the edges of huge_share)" if name == "huge_share_slice" else ""))
    else:
        raise ValueError(f"unknown workload {name!r}")

    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    say(f"{name}: features {n} x {dims[0]} {dtype}")
    x = normal_features(feat, n, dims[0], dtype, log) if features else np.zeros((0, dims[0]), np.float32)
    if agg == AGG_GAT:
        layers = gat_layers(wts, dims, 4, dtype, bias_random)
    else:
        layers = dense_layers(wts, agg, dims, dtype, bias_random)
    return Workload(name=name, n_nodes=n, n_edges=len(src), src=src, dst=dst, x=x, dtype=dtype,
                    threshold=thr, layers=layers, recipe=f"{recipe}; scale={scale}, seed={seed}")


def random_small_graph(seed: int, n_nodes: int, n_edges: int, d: int, dtype: str = F32,
                       hub_fraction: float = 0.0):
    """Small random multigraph (duplicates and self-loops allowed) with optional hub:
    ``hub_fraction`` of the edges point at node 0."""
    rng = _rng(seed, 7)
    src = rng.integers(0, max(n_nodes, 1), size=n_edges, dtype=np.int32)
    dst = rng.integers(0, max(n_nodes, 1), size=n_edges, dtype=np.int32)
    if hub_fraction > 0 and n_edges > 0:
        k = int(n_edges * hub_fraction)
        dst[rng.choice(n_edges, size=k, replace=False)] = 0
    x = normal_features(rng, n_nodes, d, dtype)
    return src, dst, x

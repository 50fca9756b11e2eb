"""Parity at the full workload sizes, in the launch configuration bench.py times.

Integer structures are compared in full (the oracle's counting sort handles 6e7 edges in seconds);
features are compared on sampled vertices -- every hub plus a few thousand random ones -- which the oracle
evaluates one by one.  Layer l+1 is checked by feeding the oracle the state the GPU stored for layer l,
so each stage is held to the bar on its own (errors cannot hide by compounding or cancelling)."""
import os

import numpy as np
import pytest

import oracle
from paper_2307_00228_amd import workloads as W

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

N_SAMPLE = 3000


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2307_00228_amd import binding
    return binding


def tolerance_ok(got_st, want64, dtype):
    got = W.as_f32(got_st).astype(np.float64)
    err = np.abs(got - want64)
    if dtype == W.F32:
        return err.max() <= 1e-4, err.max()
    tol = 2e-2 * (np.abs(want64) + np.sqrt(np.mean(want64 ** 2)))
    return bool((err <= tol).all()), float((err / tol).max())


def sample_vertices(rng, n, rowptr, split, extra=()):
    deg = np.diff(rowptr)
    picks = [rng.choice(n, size=min(N_SAMPLE, n), replace=False), np.argsort(deg)[-50:], np.nonzero(deg == 0)[0][:50]]
    if split is not None and split["n_hubs"]:
        picks.append(split["hub_ids"].astype(np.int64))
    picks.append(np.asarray(extra, dtype=np.int64))
    return np.unique(np.concatenate(picks)).astype(np.int64)


@pytest.mark.parametrize("name", ["medium_uniform", "hub_heavy"])
def test_full_size_dense_workloads(B, name):
    import torch
    w = W.make(name, 1.0)
    n, e = w.n_nodes, w.n_edges
    src, dst = torch.from_numpy(w.src).cuda(), torch.from_numpy(w.dst).cuda()
    rowptr, col, deg_out = B.build_csr_by_dst(n, src, dst)
    use_split = w.threshold < W.NO_SPLIT
    split = B.split_hubs(rowptr, w.threshold) if use_split else None

    r, c, d = oracle.build_csr(n, w.src, w.dst)
    assert np.array_equal(rowptr.cpu().numpy(), r), "rowptr"
    assert np.array_equal(col.cpu().numpy(), c), "col"
    assert np.array_equal(deg_out.cpu().numpy(), d), "deg_out"
    osplit = None
    if use_split:
        osplit = oracle.split_hubs(r, w.threshold)
        assert split.n_hubs == osplit["n_hubs"] and split.n_shadows == osplit["n_shadows"]
        for k in ("hub_ids", "hub_shadow_off", "shadow_begin", "shadow_end", "shadow_owner"):
            assert np.array_equal(getattr(split, k).cpu().numpy(), osplit[k]), k
        if name == "hub_heavy":
            assert osplit["n_hubs"] >= 16 and np.diff(r).max() >= 4_000_000

    from paper_2307_00228_amd import compose
    layers = B.device_layers(w.layers)
    x = B.to_device(w.x)
    verts = sample_vertices(np.random.default_rng(5), n, r, osplit)
    vt = torch.from_numpy(verts).cuda()
    traces = compose.run_layers(rowptr, col, deg_out, split, layers, x)
    h_host = w.x
    for i, (lay, tr) in enumerate(zip(w.layers, traces)):
        # the whole layer from the state the GPU stored for the previous one
        a_st, y64 = oracle.dense_layer(r, c, d, h_host, lay, w.dtype, verts=verts)
        ok, worst = tolerance_ok(B.to_numpy(tr.out[vt]), y64, w.dtype)
        assert ok, f"layer {i + 1}: {worst}"
        if not tr.projected:
            # stage-wise: the aggregate, then the update on the aggregate the GPU stored
            a64 = oracle.gather(lay.agg, r, c, h_host, deg_out=d, verts=verts)
            ok, worst = tolerance_ok(B.to_numpy(tr.agg[vt]), a64, w.dtype)
            assert ok, f"layer {i + 1} gather: {worst}"
            y64 = oracle.apply(np.asarray(h_host)[verts], B.to_numpy(tr.agg[vt]), lay.w_self, lay.w_nbr, lay.bias, lay.act)
            ok, worst = tolerance_ok(B.to_numpy(tr.out[vt]), y64, w.dtype)
            assert ok, f"layer {i + 1} apply: {worst}"
        else:
            # W_nbr was applied before the gather: the gather itself is a plain aggregate of the projected rows
            p64 = oracle.gather(lay.agg, r, c, B.to_numpy(tr.gather_src), deg_out=d, verts=verts)
            ok, worst = tolerance_ok(B.to_numpy(tr.agg[vt]), p64, w.dtype)
            assert ok, f"layer {i + 1} gather of projected rows: {worst}"
        h_host = B.to_numpy(tr.out)
    h_dev = traces[-1].out

    # the single-call path launches the same kernels: bitwise identical, also when issued in edge-range chunks
    view = torch.int16 if w.dtype == W.BF16 else torch.int32
    whole = B.infer_full_graph(rowptr, col, deg_out, split, layers, x)
    assert torch.equal(whole.view(view), h_dev.view(view))
    chunked = B.infer_full_graph(rowptr, col, deg_out, split, layers, x, edge_chunk=e // 8 + 1)
    assert torch.equal(chunked.view(view), whole.view(view))


def test_full_size_attention(B):
    import torch
    w = W.make("attention", 1.0)
    n = w.n_nodes
    rowptr, col, deg_out = B.build_csr_by_dst(n, torch.from_numpy(w.src).cuda(), torch.from_numpy(w.dst).cuda())
    split = B.split_hubs(rowptr, w.threshold)
    r, c, d = oracle.build_csr(n, w.src, w.dst)
    assert np.array_equal(rowptr.cpu().numpy(), r) and np.array_equal(col.cpu().numpy(), c)
    osplit = oracle.split_hubs(r, w.threshold)
    for k in ("hub_ids", "hub_shadow_off", "shadow_begin", "shadow_end", "shadow_owner"):
        assert np.array_equal(getattr(split, k).cpu().numpy(), osplit[k]), k
    verts = sample_vertices(np.random.default_rng(6), n, r, osplit)
    vt = torch.from_numpy(verts).cuda()
    lay, dl = w.layers[0], B.device_layers(w.layers)[0]
    x = B.to_device(w.x)
    # stage 1: projection and scores on the sampled rows
    z, s_src, s_dst = B.apply_layer(None, x, None, dl.w_nbr, None, W.ACT_NONE, heads=dl.heads, att_src=dl.att_src,
                                    att_dst=dl.att_dst)
    z64 = oracle.apply(None, np.asarray(w.x)[verts], None, lay.w_nbr, None, oracle.ACT_NONE)
    ok, worst = tolerance_ok(B.to_numpy(z[vt]), z64, w.dtype)
    assert ok, f"projection: {worst}"
    for got, att in ((s_src, lay.att_src), (s_dst, lay.att_dst)):
        want = oracle.gat_scores(z64, att)
        assert np.abs(got[vt].cpu().numpy() - want).max() <= 1e-3 * max(1.0, np.abs(want).max())
    # stage 2: the attention reduce on the projected state and scores the GPU stored
    out = B.gather_layer(W.AGG_GAT, rowptr, col, z, split, s_src, s_dst, heads=dl.heads, leaky_slope=dl.leaky_slope,
                         act=dl.act, bias=dl.bias)
    o64 = oracle.gat_gather(r, c, B.to_numpy(z), s_src.cpu().numpy(), s_dst.cpu().numpy(), lay.heads, lay.leaky_slope,
                            verts=verts)
    y64 = np.maximum(o64 + lay.bias.astype(np.float64), 0.0) if lay.act == W.ACT_RELU else o64 + lay.bias
    ok, worst = tolerance_ok(B.to_numpy(out[vt]), y64, w.dtype)
    assert ok, f"attention reduce: {worst}"


@pytest.mark.skipif(os.environ.get("ITB_RUN_HUGE") != "1", reason="2e9-edge run: minutes of host-side generation; set ITB_RUN_HUGE=1")
def test_full_size_huge_share(B):
    """Single-GPU share of a huge graph: 1e8 vertices, 2e9 edges, 8 edge-range chunks of 2^28."""
    import torch
    say = lambda msg: print(msg, flush=True)     # run with -s: every stage reports, none is silent for minutes
    w = W.make("huge_share", 1.0, log=say)
    n, e = w.n_nodes, w.n_edges
    say("GPU: build_csr_by_dst + split_hubs")
    rowptr, col, deg_out = B.build_csr_by_dst(n, torch.from_numpy(w.src).cuda(), torch.from_numpy(w.dst).cuda(), want_deg_out=False)
    split = B.split_hubs(rowptr, w.threshold)
    say(f"GPU: {split.n_hubs} hubs, {split.n_shadows} segments; oracle: counting sort of {e} edges")
    r, c, d = oracle.build_csr(n, w.src, w.dst)
    say("oracle CSR done; comparing")
    assert np.array_equal(rowptr.cpu().numpy(), r) and np.array_equal(col.cpu().numpy(), c)
    osplit = oracle.split_hubs(r, w.threshold)
    for k in ("hub_ids", "hub_shadow_off", "shadow_begin", "shadow_end", "shadow_owner"):
        assert np.array_equal(getattr(split, k).cpu().numpy(), osplit[k]), k
    layers = B.device_layers(w.layers)
    x = B.to_device(w.x)
    say("GPU: infer_full_graph in 2^28-edge chunks")
    torch.cuda.synchronize()
    import time
    t0 = time.perf_counter()
    out = B.infer_full_graph(rowptr, col, None, split, layers, x, edge_chunk=1 << 28)
    torch.cuda.synchronize()
    say(f"GPU: infer_full_graph (first call, 2 layers, 8 chunks) {1e3 * (time.perf_counter() - t0):.1f} ms")
    verts = sample_vertices(np.random.default_rng(7), n, r, osplit)
    say(f"oracle: {len(verts)} sampled vertices, layer by layer")
    vt = torch.from_numpy(verts).cuda()
    agg1 = B.gather_layer(W.AGG_MEAN, rowptr, col, x, split)
    h1 = B.apply_layer(x, agg1, layers[0].w_self, layers[0].w_nbr, layers[0].bias, layers[0].act)
    a64 = oracle.gather(oracle.MEAN, r, c, w.x, verts=verts)
    ok, worst = tolerance_ok(B.to_numpy(agg1[vt]), a64, w.dtype)
    assert ok, f"layer 1 gather: {worst}"
    h1_host = B.to_numpy(h1)
    a64 = oracle.gather(oracle.MEAN, r, c, h1_host, verts=verts)
    agg2 = B.gather_layer(W.AGG_MEAN, rowptr, col, h1, split)
    ok, worst = tolerance_ok(B.to_numpy(agg2[vt]), a64, w.dtype)
    assert ok, f"layer 2 gather: {worst}"
    y64 = oracle.apply(h1_host[verts], B.to_numpy(agg2[vt]), w.layers[1].w_self, w.layers[1].w_nbr, w.layers[1].bias, w.layers[1].act)
    ok, worst = tolerance_ok(B.to_numpy(out[vt]), y64, w.dtype)
    assert ok, f"layer 2 apply (chunked infer_full_graph): {worst}"

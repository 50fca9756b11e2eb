#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A step = build_csr_by_dst + split_hubs + infer_full_graph (which is gcn_norm_scales + gcn_edge_coefficients + L x
(gather_layer + apply_layer)) over one synthetic graph whose edge list, features and weights are already resident in
HBM.  The layer loop records caller-provided HIP events at its stage boundaries (itb_set_layer_events), so the gather
kernel is timed live inside the timed region; `infer_full_graph_ms` additionally times the call back to back.

Prints ONE JSON line: metric / value (edges per second and layer over the whole step), `roofline` (the gather launch
with the longest duration: algorithmic bytes / measured time against the HBM peak, plus the hardware byte count recorded
under profiles/), `breakdown` (per-stage times and rates) and `cpu_baseline` (the CPU oracle timed on the host)."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="medium_uniform")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--threshold", default=None,
                    help="hub threshold override: an integer, or 'heuristic' = 0.1 * E / #CUs (Sec. IV-D rule of thumb)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget-s", type=float, default=25.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run the plain copy kernel (1 GiB, 5 launches): reference for byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2307_00228_amd import binding as B
    from paper_2307_00228_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = 1 << 30
        a = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
        b = torch.empty(n, dtype=torch.uint8, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        B.copy_bytes(a, b)
        e0.record()
        for _ in range(5):
            B.copy_bytes(a, b)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        print(json.dumps({"copy_bytes": n, "launches": 6, "avg_ms": ms, "GBps_read_plus_write": 2 * n / ms / 1e6}))
        return
    w = W.make(args.workload, args.scale)
    N, E, L = w.n_nodes, w.n_edges, len(w.layers)
    esz = 2 if w.dtype == W.BF16 else 4
    src, dst = torch.from_numpy(w.src).cuda(), torch.from_numpy(w.dst).cuda()
    x = B.to_device(w.x)
    layers = B.device_layers(w.layers)
    if args.threshold is not None:
        if args.threshold == "heuristic":
            w.threshold = B.hub_threshold_heuristic(E, torch.cuda.get_device_properties(0).multi_processor_count, 0.1)
        else:
            w.threshold = int(args.threshold)
    use_split = w.threshold < W.NO_SPLIT
    thr = w.threshold if use_split else (1 << 62)
    tdt = x.dtype

    for kv in os.environ.get("ITB_TUNING", "").split(","):       # e.g. ITB_TUNING=2:0 (measurement aid)
        if kv:
            B.set_tuning(int(kv.split(":")[0]), int(kv.split(":")[1]))

    from paper_2307_00228_amd import compose
    is_gat = [l.agg == W.AGG_GAT for l in w.layers]
    needs_deg_out = any(l.agg == W.AGG_GCN for l in w.layers)   # out-degrees enter the GCN coefficients only
    projected = compose.plan(layers, tdt)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    stamps = {"gather": [], "apply": [], "project": [], "csr": [], "split": []}
    out = torch.empty((N, w.layers[-1].d_out), dtype=tdt, device="cuda")
    state = {"ws": None}

    def fresh_events(k):
        evs = [ev() for _ in range(k)]
        for e in evs:
            e.record()              # creates the handle; the library records it again at its mark
        return evs

    # Events for every timed step are made beforehand: inside the timed region a step costs the three calls below
    # plus one call that hands the step's events to the library.
    layer_events = [fresh_events(4 * L) for _ in range(args.steps)]
    outer_events = [fresh_events(3) for _ in range(args.steps)]
    torch.cuda.synchronize()

    def step(k):
        """k: index of the timed step, or None for a warm-up step."""
        if k is not None:
            outer_events[k][0].record()
        rowptr, col, deg_out = B.build_csr_by_dst(N, src, dst, want_deg_out=needs_deg_out)
        if k is not None:
            outer_events[k][1].record()
        split = B.split_hubs(rowptr, thr)
        if k is not None:
            outer_events[k][2].record()
        sp = split if use_split else None
        if state["ws"] is None:
            state["ws"] = torch.empty(max(256, B.infer_workspace_bytes(N, E, sp, tdt, layers)), dtype=torch.uint8, device="cuda")
        B.set_layer_events(layer_events[k] if k is not None else [])
        B.infer_full_graph(rowptr, col, deg_out, sp, layers, x, out=out, workspace=state["ws"])
        return rowptr, col, deg_out, split

    for _ in range(args.warmup):
        graph = step(None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        graph = step(k)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    B.set_layer_events([])
    ms_per_step = elapsed * 1e3 / args.steps
    for k in range(args.steps):
        o, le = outer_events[k], layer_events[k]
        stamps["csr"].append((o[0], o[1]))
        stamps["split"].append((o[1], o[2]))
        for i in range(L):
            b, g0, g1, e1 = le[4 * i: 4 * i + 4]
            stamps["gather"].append((g0, g1))
            if is_gat[i]:               # projection first, the attention reduce ends the layer
                stamps["apply"].append((b, g0))
                stamps["project"].append(None)
            else:                       # optional projection, gather, update
                stamps["project"].append((b, g0))
                stamps["apply"].append((g1, e1))

    def avg_ms(pairs, sel=None):
        v = [p[0].elapsed_time(p[1]) if p is not None else 0.0 for p in pairs]
        if sel is not None:
            v = v[sel::L]
        return float(np.mean(v)) if v else 0.0

    g_ms = [avg_ms(stamps["gather"], i) for i in range(L)]
    a_ms = [avg_ms(stamps["apply"], i) for i in range(L)]
    p_ms = [avg_ms(stamps["project"], i) for i in range(L)]   # projection before the gather (0 where there is none)
    # algorithmic traffic of one gather launch: every in-edge reads its column index and its source row once,
    # every vertex reads its row pointer and writes its aggregate row once
    # (GAT: the row is the projected state of width d_out; plus the 4-byte source score of each head per edge, and per
    # vertex its own row and scores for the implicit self edge)
    # (a narrowing layer gathers rows already multiplied by W_nbr: width d_out)
    def gather_width(l, g, pf):
        return l.d_out if (g or pf) else l.d_in
    # (a GCN layer also reads the 4-byte source coefficient of each in-edge and the 4-byte destination scale of each vertex)
    g_bytes = [E * (4 + 4 * l.heads + l.d_out * esz) + N * (8 + 2 * l.d_out * esz + 8 * l.heads) if g
               else E * (4 + (4 if l.agg == W.AGG_GCN else 0) + gather_width(l, g, pf) * esz)
               + N * (8 + (4 if l.agg == W.AGG_GCN else 0) + gather_width(l, g, pf) * esz)
               for l, g, pf in zip(w.layers, is_gat, projected)]
    # flops of the final update launch of the layer (GAT: the projection; projected layers: the self product)
    a_flops = [(2.0 if (g or pf) else 4.0) * l.d_in * l.d_out * N for l, g, pf in zip(w.layers, is_gat, projected)]
    dom = int(np.argmax(g_ms))
    achieved = g_bytes[dom] / (g_ms[dom] * 1e-3) / 1e9

    # infer_full_graph itself (same kernels, one call)
    rowptr, col, deg_out, split = graph
    ws = state["ws"]
    for _ in range(2):
        B.infer_full_graph(rowptr, col, deg_out, split if use_split else None, layers, x, out=out, workspace=ws)
    i0, i1 = ev(), ev()
    i0.record()
    for _ in range(args.steps):
        B.infer_full_graph(rowptr, col, deg_out, split if use_split else None, layers, x, out=out, workspace=ws)
    i1.record()
    torch.cuda.synchronize()
    infer_ms = i0.elapsed_time(i1) / args.steps
    # the same call captured once into a HIP graph and replayed (the layer loop only enqueues work)
    hip_graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(hip_graph):
        B.infer_full_graph(rowptr, col, deg_out, split if use_split else None, layers, x, out=out, workspace=ws)
    hip_graph.replay()
    g0, g1 = ev(), ev()
    g0.record()
    for _ in range(args.steps):
        hip_graph.replay()
    g1.record()
    torch.cuda.synchronize()
    infer_graph_ms = g0.elapsed_time(g1) / args.steps

    # HBM-side traffic of the dominant kernel is measured offline with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, each
    # scaled by the plain copy kernel) and recorded with its provenance; null when no record covers this workload.
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath) and args.scale == 1.0:
        rec = json.load(open(tpath)).get(args.workload)
        if rec:
            traffic = rec["traffic_bytes_per_launch"]

    result = {
        "metric": "edges/sec per GNN layer (gather) + apply TFLOP/s; % of HBM/MFMA roofline",
        "value": E * L / (ms_per_step * 1e-3),
        "unit": "edges/s per layer, whole path incl. CSR build and hub split (E*L / step time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "scale": args.scale, "n_nodes": N, "n_edges": E,
                   "dims": [w.layers[0].d_in] + [l.d_out for l in w.layers], "aggregator": w.layers[0].agg,
                   "hub_threshold": w.threshold if use_split else None, "recipe": w.recipe},
        "roofline": {"bound": "hbm", "kernel": f"gather_layer (layer {dom + 1}, dim {gather_width(w.layers[dom], is_gat[dom], projected[dom])})",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "algorithmic_bytes": g_bytes[dom], "avg_ms": g_ms[dom]},
        "breakdown": {
            "csr_build_ms": avg_ms(stamps["csr"]), "split_hubs_ms": avg_ms(stamps["split"]),
            "gather_ms": g_ms, "apply_ms": a_ms, "infer_full_graph_ms": infer_ms, "infer_full_graph_replay_ms": infer_graph_ms,
            "gather_edges_per_s": [E / (t * 1e-3) for t in g_ms],
            "gather_GBps": [b / (t * 1e-3) / 1e9 for b, t in zip(g_bytes, g_ms)],
            "apply_TFLOPs": [f / (t * 1e-3) / 1e12 for f, t in zip(a_flops, a_ms)],
            "apply_frac_of_mfma_peak": [f / (t * 1e-3) / 1e12 / PEAK_TFLOPS[w.dtype] for f, t in zip(a_flops, a_ms)],
            "projected_before_gather": projected, "project_ms": p_ms,
            "nodes_per_s_per_layer": [N / ((g + a) * 1e-3) for g, a in zip(g_ms, a_ms)],
            "n_hubs": split.n_hubs, "n_shadows": split.n_shadows,
        },
    }

    if not args.no_cpu_baseline:
        import oracle
        cores = oracle.set_threads(0)
        # bounded sample: the whole path on the first `frac` of the workload's vertices/edges if the full one
        # would take much longer than the budget (estimated from a small probe)
        probe = W.make(args.workload, min(args.scale, 0.02 * args.scale if N > 200_000 else args.scale))
        t = time.perf_counter()
        r, c, d = oracle.build_csr(probe.n_nodes, probe.src, probe.dst)
        oracle.split_hubs(r, thr)
        oracle.infer_full_graph(r, c, d, probe.x, probe.layers, probe.dtype)
        probe_s = time.perf_counter() - t
        est_full = probe_s * (E / max(probe.n_edges, 1))
        frac = 1.0 if est_full <= args.cpu_budget_s else args.cpu_budget_s / est_full
        sw = w if frac == 1.0 else W.make(args.workload, args.scale * frac)
        t = time.perf_counter()
        r, c, d = oracle.build_csr(sw.n_nodes, sw.src, sw.dst)
        oracle.split_hubs(r, thr)
        oracle.infer_full_graph(r, c, d, sw.x, sw.layers, sw.dtype)
        cpu_s = time.perf_counter() - t
        result["cpu_baseline"] = {"value": sw.n_edges * L / cpu_s, "unit": "edges/s per layer, whole path",
                                  "cores": cores, "kind": "oracle",
                                  "sample": f"same workload at scale {args.scale * frac:.4g} "
                                            f"({sw.n_nodes} nodes, {sw.n_edges} edges, all {L} layers), {cpu_s:.1f} s"}
        # the same on one thread, on a sample sized for a few seconds
        one = W.make(args.workload, args.scale * frac / max(1.0, 0.25 * cores * cpu_s))
        oracle.set_threads(1)
        t = time.perf_counter()
        r, c, d = oracle.build_csr(one.n_nodes, one.src, one.dst)
        oracle.split_hubs(r, thr)
        oracle.infer_full_graph(r, c, d, one.x, one.layers, one.dtype)
        one_s = time.perf_counter() - t
        oracle.set_threads(cores)
        result["cpu_baseline"]["value_1_thread"] = one.n_edges * L / one_s
        result["cpu_baseline"]["sample_1_thread"] = f"{one.n_nodes} nodes, {one.n_edges} edges, {one_s:.1f} s"
    print(json.dumps(result))


if __name__ == "__main__":
    main()

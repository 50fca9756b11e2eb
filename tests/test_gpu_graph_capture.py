"""The layer loop only enqueues work (kernels, and the fork/join of its helper stream): it can be captured into a
HIP graph and replayed.  Every replay is checked against the eager result, with eager work and synchronisations of
the program in between."""
import numpy as np
import pytest

from paper_2307_00228_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,scale,chunks", [("tiny_powerlaw", 1.0, 1), ("hub_heavy", 0.002, 1), ("attention", 0.003, 1),
                                               ("huge_share", 0.0005, 3)])
def test_infer_full_graph_under_graph_capture(name, scale, chunks):
    """(huge_share: bf16 64-64-32, whose first update is chained into the second layer's projection, issued in three
    edge ranges with one fork of the helper stream per layer.)"""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2307_00228_amd import binding as B
    w = W.make(name, scale, bias_random=True)
    src = torch.from_numpy(np.ascontiguousarray(w.src)).cuda()
    dst = torch.from_numpy(np.ascontiguousarray(w.dst)).cuda()
    rowptr, col, deg_out = B.build_csr_by_dst(w.n_nodes, src, dst)
    split = B.split_hubs(rowptr, w.threshold) if w.threshold < W.NO_SPLIT else None
    if name != "tiny_powerlaw":
        assert split.n_hubs > 0                      # the captured region contains the helper-stream fork and join
    layers, x = B.device_layers(w.layers), B.to_device(w.x)
    chunk = 0 if chunks == 1 else (w.n_edges + chunks - 1) // chunks
    ws = torch.empty(max(256, B.infer_workspace_bytes(w.n_nodes, w.n_edges, split, x.dtype, layers, chunk)), dtype=torch.uint8,
                     device="cuda")
    out = torch.empty((w.n_nodes, w.layers[-1].d_out), dtype=x.dtype, device="cuda")
    view = torch.int16 if w.dtype == W.BF16 else torch.int32
    eager = B.infer_full_graph(rowptr, col, deg_out, split, layers, x, out=out, workspace=ws, edge_chunk=chunk).clone()   # also warms up
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.infer_full_graph(rowptr, col, deg_out, split, layers, x, out=out, workspace=ws, edge_chunk=chunk)
    for k in range(4):
        out.fill_(float("nan"))
        ws.random_(0, 255)                           # eager work between the replays, on the same buffers
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(view), eager.view(view)), f"replay {k}"
        again = B.infer_full_graph(rowptr, col, deg_out, split, layers, x)      # eager call between replays
        assert torch.equal(again.view(view), eager.view(view))

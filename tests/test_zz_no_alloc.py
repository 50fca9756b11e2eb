"""gather_layer_noalloc (the entry point for callers that cannot allocate) against gather_layer, through the C ABI.

Two calls in a row on the same GPU share the library's built-in scratch array, which keeps the previous call's
contents: the second call uses a smaller input, so stale list entries and partials would show."""
import numpy as np
import pytest

import oracle
from paper_2307_00228_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2307_00228_amd import binding
    return binding


def graph(B, seed, n, e, dim, dtype, hub, T):
    import torch
    src, dst, x = W.random_small_graph(seed, n, e, dim, dtype, hub)
    r, c, d = oracle.build_csr(n, src, dst)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    split = B.split_hubs(rp, T) if T else None
    return (r, c, d, x), rp, cl, split, B.to_device(x)


@pytest.mark.parametrize("kind", [W.AGG_MEAN, W.AGG_GCN, W.AGG_MAX, W.AGG_GAT])
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_noalloc_equals_gather_layer_two_calls_in_a_row(B, kind, dtype):
    import torch
    view = torch.int16 if dtype == W.BF16 else torch.int32
    B.set_tuning(3, 40)        # long-row limit 40: the work list in the scratch array is used by both calls
    try:
        # the larger input first (hubs -> partials, many long rows), then a smaller one with other sizes everywhere
        for seed, n, e, dim, hub, T in [(101, 9000, 200000, 128, 0.3, 300), (102, 700, 9000, 64, 0.2, 50)]:
            host, rp, cl, split, h = graph(B, seed, n, e, dim, dtype, hub, T)
            r, c, d, x = host
            kw = {}
            ss = sd = None
            if kind == W.AGG_GCN:
                ss, sd = B.gcn_norm_scales(rp, torch.from_numpy(d).cuda())
            if kind == W.AGG_GAT:
                rng = np.random.default_rng(seed)
                ss = torch.from_numpy(rng.standard_normal((n, 4)).astype(np.float32)).cuda()
                sd = torch.from_numpy(rng.standard_normal((n, 4)).astype(np.float32)).cuda()
                kw = dict(heads=4, leaky_slope=0.2)
            want = B.gather_layer(kind, rp, cl, h, split, ss, sd, **kw)
            out = torch.full_like(want, float("nan"))
            B.gather_layer_noalloc(kind, rp, cl, h, out, split, ss, sd, **kw)
            torch.cuda.synchronize()
            assert torch.equal(out.view(view), want.view(view)), f"n={n}"
            # and, like gather_layer itself, to the oracle's bar
            got = W.as_f32(B.to_numpy(out)).astype(np.float64)
            if kind == W.AGG_GAT:
                o64 = oracle.gat_gather(r, c, x, ss.cpu().numpy(), sd.cpu().numpy(), 4, 0.2)
            else:
                o64 = oracle.gather(kind, r, c, x, deg_out=d)
            if kind == W.AGG_MAX:
                assert (got == o64).all()
            elif dtype == W.F32:
                assert np.abs(got - o64).max() <= 1e-4
            else:
                assert (np.abs(got - o64) <= 2e-2 * (np.abs(o64) + np.sqrt(np.mean(o64 ** 2)))).all()
    finally:
        B.set_tuning(3, 512)


def test_noalloc_rejects_sizes_beyond_its_scratch(B):
    import torch
    n = 1 << 23                      # the work list alone (4 bytes per vertex) exceeds the 16 MiB array
    rp = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
    cl = torch.zeros(0, dtype=torch.int32, device="cuda")
    h = torch.zeros((n, 4), dtype=torch.float32, device="cuda")
    out = torch.empty_like(h)
    with pytest.raises(B.InferTurboError, match="WORKSPACE"):
        B.gather_layer_noalloc(W.AGG_SUM, rp, cl, h, out)
    torch.cuda.synchronize()

"""Parity of the HIP path against the CPU oracle, through the C ABI (needs an MI355X).

Integer results (CSR, hub split) must be bit-exact.  Features: fp32 within max-abs 1e-4;
for the un-normalised SUM aggregator, whose terms do not shrink with the in-degree, element
by element 1e-4 * max(1, |oracle value|, root-sum-square of the element's own terms): the
rounding of an fp32 sum scales with the magnitude of what is summed, and a hub's element may
be small only by cancellation; an element next to a hub gets no slack from the hub.
bf16 storage with fp32 accumulation within |g-o| <= 2e-2 * (|o| + rms(o)).
Whole layers are held to Eq. (1) without intermediate rounding; where the path under test
stores agg(h) in bf16 between gather and update, the bound is widened by what that one
rounding can move the result at most (agg_rounding_slack)."""
import numpy as np
import pytest

import oracle
from paper_2307_00228_amd import workloads as W

pytestmark = pytest.mark.gpu

FP32_ATOL = 1e-4
BF16_RTOL = 2e-2


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2307_00228_amd import binding
    return binding


def dev_i32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def sum_scale(graph, x_st, edge_w=None):
    """Root-sum-square of the terms of every element of an un-normalised sum over in-edges (CSR rowptr, col)."""
    import scipy.sparse as sp
    r, c = graph[0], graph[1]
    n = len(r) - 1
    w2 = np.ones(len(c)) if edge_w is None else np.asarray(edge_w, dtype=np.float64) ** 2
    return np.sqrt(sp.csr_matrix((w2, c, r), shape=(n, n)) @ (W.as_f32(x_st).astype(np.float64) ** 2))


def check_features(got_st, want64, dtype, what="", sum_terms=None, slack=0.0):
    """`sum_terms`: for an un-normalised SUM, the root-sum-square of every element's terms (see sum_scale)."""
    got = W.as_f32(got_st).astype(np.float64)
    want64 = np.asarray(want64, dtype=np.float64)
    assert got.shape == want64.shape, (got.shape, want64.shape)
    if got.size == 0:
        return
    err = np.abs(got - want64)
    if dtype == W.F32:
        atol = FP32_ATOL * (np.maximum(np.maximum(1.0, np.abs(want64)), sum_terms) if sum_terms is not None
                            else np.ones_like(want64))
        bad = err > atol
        assert not bad.any(), f"{what}: fp32 abs err {err[bad].max():.3e} at {np.argwhere(bad)[0]} (tol {atol[bad].min():.1e})"
    else:
        tol = BF16_RTOL * (np.abs(want64) + np.sqrt(np.mean(want64 ** 2))) + slack
        bad = err > tol
        assert not bad.any(), f"{what}: bf16 err {err[bad].max():.3e} at {np.argwhere(bad)[0]} (tol {tol[bad].min():.3e})"


def agg_rounding_slack(a64, w_nbr, dtype):
    """What storing agg(h) in bf16 between gather and update can move the update by: round-to-nearest-even changes
    an element by at most 2^-9 relative, so output j moves by at most 2^-9 * sum_k |agg_k| |W_kj|."""
    if dtype == W.F32 or a64 is None:
        return 0.0
    return 2.0 ** -9 * (np.abs(a64) @ np.abs(W.as_f32(w_nbr).astype(np.float64)))


def check_layer(B, tr, r, c, d, h, lay, dtype, what):
    """One dense layer's stored output against Eq. (1) evaluated from the stored input `h`."""
    _, y64, a64 = oracle.dense_layer(r, c, d, h, lay, dtype, return_agg64=True)
    exact_agg = tr.projected or lay.agg in (W.AGG_MAX, W.AGG_MIN, W.AGG_NONE)     # nothing rounded between the steps
    check_features(B.to_numpy(tr.out), y64, dtype, what, slack=0.0 if exact_agg else agg_rounding_slack(a64, lay.w_nbr, dtype))


# ------------------------------------------------------------------------------------------ CSR build
CSR_CASES = [
    ("empty_graph", 0, 0, 0.0), ("nodes_no_edges", 17, 0, 0.0), ("one_node_self_loops", 1, 9, 0.0),
    ("two_nodes", 2, 5, 0.0), ("tiny", 10, 37, 0.3), ("one_tile_ragged", 1000, 4095, 0.2),
    ("tile_plus_one", 300, 4097, 0.5), ("several_tiles", 70000, 300001, 0.1), ("all_to_one", 5000, 50000, 1.0),
    ("wide_ids_3_passes", 1 << 17, 200000, 0.05), ("sparse_rows", 1_000_000, 4000, 0.0),
]


@pytest.mark.parametrize("name,n,e,hub", CSR_CASES, ids=[c[0] for c in CSR_CASES])
def test_build_csr_bit_exact(B, name, n, e, hub):
    src, dst, _ = W.random_small_graph(n % 997 + e % 991, n, e, 1, W.F32, hub)
    if n == 0:
        src, dst = src[:0], dst[:0]
    rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
    r, c, d = oracle.build_csr(n, src, dst)
    assert np.array_equal(rowptr.cpu().numpy(), r), "rowptr"
    assert np.array_equal(col.cpu().numpy(), c), "col (stable order)"
    assert np.array_equal(deg_out.cpu().numpy(), d), "deg_out"


@pytest.mark.parametrize("bits", [1, 2, 4, 5, 6, 7, 8, 9, 12, 15, 16, 17, 21, 24, 25])
def test_build_csr_every_digit_width_and_pass_count(B, bits):
    """The key width decides the number of radix passes (1 to 4) and the digit width of each (1..8 bits; 5..8 have code
    of their own).  Row pointers come from the runs of the last pass, so the cases also put the edges into a few far-apart
    vertex ids (long stretches of empty (digit, tile) runs and of empty rows), and use a ragged last tile."""
    n = (1 << bits) - (3 if bits > 2 else 0)          # not a power of two: the top digit is not full
    e = 5 * 8192 + 123
    rng = np.random.default_rng(bits)
    src = rng.integers(0, n, e).astype(np.int32)
    for spread in ("uniform", "clustered"):
        if spread == "uniform":
            dst = rng.integers(0, n, e).astype(np.int32)
        else:
            few = np.unique(np.concatenate([[0, n - 1, n // 2], rng.integers(0, n, 5)])).astype(np.int32)
            dst = few[rng.integers(0, len(few), e)]
        r, c, d = oracle.build_csr(n, src, dst)
        for want_deg in (False, True):
            rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst), want_deg_out=want_deg)
            assert np.array_equal(rowptr.cpu().numpy(), r), (spread, want_deg, "rowptr")
            assert np.array_equal(col.cpu().numpy(), c), (spread, want_deg, "col")
            if want_deg:
                assert np.array_equal(deg_out.cpu().numpy(), d), (spread, "deg_out")


@pytest.mark.parametrize("n,e,hub", [(5000, 700000, 0.6), (1, 9, 0.0), (17, 100, 0.5), (1 << 17, 200000, 0.1),
                                     (5_000_000, 100000, 0.2), (3000, 0, 0.0)])
def test_out_degrees_both_strategies(B, n, e, hub):
    """deg_out comes from a partition + per-bucket count (ids up to 2^22; a source with more than 2^18 out-edges
    spans several slices of its bucket) or from the keys-only sort (wider ids, or forced): both exact."""
    import torch
    dst, src, _ = W.random_small_graph(n + e + 5, n, e, 4, W.F32, hub)      # swapped: the hub is a SOURCE here
    want = np.bincount(src, minlength=n).astype(np.int32)
    assert np.array_equal(oracle.build_csr(n, src, dst)[2], want)
    for forced_sort in (0, 1):
        B.set_tuning(5, forced_sort)
        try:
            rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
            torch.cuda.synchronize()
        finally:
            B.set_tuning(5, 0)
        assert np.array_equal(deg_out.cpu().numpy(), want), f"forced_sort={forced_sort}"
        r, c, _ = oracle.build_csr(n, src, dst)
        assert np.array_equal(rowptr.cpu().numpy(), r) and np.array_equal(col.cpu().numpy(), c)


def test_build_csr_range_error(B):
    src = np.array([0, 1, 2, 3], np.int32)
    for bad_dst in (np.array([1, 4, 0, 0], np.int32), np.array([1, -1, 0, 0], np.int32)):
        with pytest.raises(B.InferTurboError) as ei:
            B.build_csr_by_dst(4, dev_i32(src), dev_i32(bad_dst))
        assert ei.value.code == -3
    # a bad source is found with and without out-degrees (two different kernels look at the source column), also when
    # it sits in the ragged last tile of a multi-tile table, and a table of valid ids right at the limit passes
    for want_deg in (True, False):
        with pytest.raises(B.InferTurboError) as ei:
            B.build_csr_by_dst(4, dev_i32(np.array([7, 1, 2, 3], np.int32)), dev_i32(src), want_deg_out=want_deg)
        assert ei.value.code == -3
        n, e = 1000, 3 * 8192 + 77
        rng = np.random.default_rng(3)
        s_ok, d_ok = rng.integers(0, n, e).astype(np.int32), rng.integers(0, n, e).astype(np.int32)
        s_ok[5], d_ok[9] = n - 1, n - 1
        B.build_csr_by_dst(n, dev_i32(s_ok), dev_i32(d_ok), want_deg_out=want_deg)
        for where in (0, 8191, 8192, e - 1):
            for bad in (n, -1):
                s_bad = s_ok.copy()
                s_bad[where] = bad
                with pytest.raises(B.InferTurboError) as ei:
                    B.build_csr_by_dst(n, dev_i32(s_bad), dev_i32(d_ok), want_deg_out=want_deg)
                assert ei.value.code == -3, (want_deg, where, bad)


@pytest.mark.parametrize("name,scale", [("tiny_powerlaw", 1.0), ("hub_heavy", 0.01), ("attention", 0.01),
                                        ("huge_share", 0.0005), ("medium_uniform", 0.05)])
def test_build_csr_workloads(B, name, scale):
    w = W.make(name, scale, features=False)
    rowptr, col, deg_out = B.build_csr_by_dst(w.n_nodes, dev_i32(w.src), dev_i32(w.dst))
    r, c, d = oracle.build_csr(w.n_nodes, w.src, w.dst)
    assert np.array_equal(rowptr.cpu().numpy(), r)
    assert np.array_equal(col.cpu().numpy(), c)
    assert np.array_equal(deg_out.cpu().numpy(), d)


# ------------------------------------------------------------------------------------------ hub split
def assert_split_equal(sp, want):
    assert sp.n_hubs == want["n_hubs"] and sp.n_shadows == want["n_shadows"]
    assert np.array_equal(sp.hub_ids.cpu().numpy(), want["hub_ids"])
    assert np.array_equal(sp.hub_shadow_off.cpu().numpy(), want["hub_shadow_off"])
    assert np.array_equal(sp.shadow_begin.cpu().numpy(), want["shadow_begin"])
    assert np.array_equal(sp.shadow_end.cpu().numpy(), want["shadow_end"])
    assert np.array_equal(sp.shadow_owner.cpu().numpy(), want["shadow_owner"])


@pytest.mark.parametrize("T", [1, 2, 3, 7, 64, 999, 1000, 1001, 10 ** 9, 1 << 31, 1 << 62])
def test_split_hubs_bit_exact(B, T):
    import torch
    n, e = 5000, 60000
    src, dst, _ = W.random_small_graph(7, n, e, 1, W.F32, 0.3)
    dst[:1000] = 4999                                   # in-degree of the last vertex >= 1000
    r, c, _ = oracle.build_csr(n, src, dst)
    sp = B.split_hubs(torch.from_numpy(r).cuda(), T)
    assert_split_equal(sp, oracle.split_hubs(r, T))


def test_split_hubs_threshold_boundary_and_empty(B):
    import torch
    src = np.arange(1, 9, dtype=np.int32)
    r, _, _ = oracle.build_csr(9, src, np.zeros(8, np.int32))
    rp = torch.from_numpy(r).cuda()
    assert B.split_hubs(rp, 8).n_hubs == 0              # in-degree == threshold is not a hub
    s7 = B.split_hubs(rp, 7)
    assert s7.n_hubs == 1 and s7.n_shadows == 2
    assert_split_equal(s7, oracle.split_hubs(r, 7))
    empty = B.split_hubs(torch.zeros(1, dtype=torch.int64, device="cuda"), 4)
    assert empty.n_hubs == 0 and empty.n_shadows == 0 and empty.hub_shadow_off.cpu().tolist() == [0]


@pytest.mark.parametrize("name,scale", [("hub_heavy", 0.01), ("attention", 0.01), ("huge_share", 0.0005)])
def test_split_hubs_workloads(B, name, scale):
    import torch
    w = W.make(name, scale, features=False)
    r, _, _ = oracle.build_csr(w.n_nodes, w.src, w.dst)
    sp = B.split_hubs(torch.from_numpy(r).cuda(), w.threshold)
    want = oracle.split_hubs(r, w.threshold)
    assert want["n_hubs"] > 0
    assert_split_equal(sp, want)


# ------------------------------------------------------------------------------------------ gather
def run_gather(B, kind, n, src, dst, x_st, dtype, T=None, out_f32=False, chunk=None):
    import torch
    r, c, d = oracle.build_csr(n, src, dst)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    split = B.split_hubs(rp, T) if T is not None else None
    h = B.to_device(x_st)
    ss = sd = None
    if kind == W.AGG_GCN:
        ss, sd = B.gcn_norm_scales(rp, torch.from_numpy(d).cuda())
    out_dtype = torch.float32 if out_f32 else None
    if chunk is None:
        out = B.gather_layer(kind, rp, cl, h, split, ss, sd, out_dtype=out_dtype)
    else:
        out = torch.full((n, x_st.shape[1]), float("nan"), dtype=out_dtype or h.dtype, device="cuda")
        e = len(src)
        lo = 0
        while True:
            hi = lo + chunk
            last = hi >= e
            B.gather_layer(kind, rp, cl, h, split, ss, sd, out_dtype=out_dtype, edge_lo=lo,
                           edge_hi=B.INT64_MAX if last else hi, out=out)
            if last:
                break
            lo = hi
    want = oracle.gather(kind, r, c, x_st, deg_out=d)
    return B.to_numpy(out), want, (r, c, d)


GATHER_DIMS = {W.F32: [4, 16, 64, 100, 128, 260], W.BF16: [8, 64, 128, 256, 520]}


@pytest.mark.parametrize("kind", [W.AGG_SUM, W.AGG_MEAN, W.AGG_GCN])
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_gather_dims_no_split(B, kind, dtype):
    for dim in GATHER_DIMS[dtype]:
        n, e = 3000, 40000
        src, dst, x = W.random_small_graph(dim, n, e, dim, dtype, 0.15)
        got, want, g = run_gather(B, kind, n, src, dst, x, dtype)
        check_features(got, want, dtype, f"dim={dim}", sum_terms=sum_scale(g, x) if kind == W.AGG_SUM else None)


@pytest.mark.parametrize("kind", [W.AGG_SUM, W.AGG_MEAN, W.AGG_GCN])
@pytest.mark.parametrize("dtype,dim", [(W.F32, 64), (W.F32, 128), (W.BF16, 64), (W.BF16, 128), (W.BF16, 256)])
@pytest.mark.parametrize("T", [1, 5, 64, 1000])
def test_gather_with_hub_split(B, kind, dtype, dim, T):
    n, e = 2000, 30000
    src, dst, x = W.random_small_graph(T + dim, n, e, dim, dtype, 0.35)
    got, want, g = run_gather(B, kind, n, src, dst, x, dtype, T=T)
    check_features(got, want, dtype, f"T={T}", sum_terms=sum_scale(g, x) if kind == W.AGG_SUM else None)


def test_gather_edge_cases(B):
    # no edges at all; a single vertex; isolated vertices next to a hub; in-degree == T and T+1
    for n, e, hub in [(5, 0, 0.0), (1, 0, 0.0), (1, 300, 0.0), (64, 64, 1.0), (65, 4000, 0.9), (129, 1, 0.0)]:
        src, dst, x = W.random_small_graph(n + e, n, e, 64, W.F32, hub)
        for T in (None, 16):
            for kind in (W.AGG_SUM, W.AGG_MEAN, W.AGG_GCN):
                got, want, g = run_gather(B, kind, n, src, dst, x, W.F32, T=T)
                check_features(got, want, W.F32, f"n={n} e={e} T={T} kind={kind}",
                               sum_terms=sum_scale(g, x) if kind == W.AGG_SUM else None)
    src = np.concatenate([np.arange(16), np.arange(17)]).astype(np.int32)
    dst = np.concatenate([np.zeros(16), np.ones(17)]).astype(np.int32)
    _, _, x = W.random_small_graph(3, 20, 0, 32, W.BF16)
    got, want, _ = run_gather(B, W.AGG_MEAN, 20, src, dst, x, W.BF16, T=16)
    check_features(got, want, W.BF16)
    assert not W.as_f32(got)[2:].any()                  # isolated vertices aggregate to exactly zero


def test_gather_bf16_in_fp32_out(B):
    n, e, dim = 4000, 50000, 128
    src, dst, x = W.random_small_graph(11, n, e, dim, W.BF16, 0.3)
    got, want, _ = run_gather(B, W.AGG_MEAN, n, src, dst, x, W.BF16, T=100, out_f32=True)
    assert got.dtype == np.float32
    assert np.abs(got.astype(np.float64) - want).max() <= 1e-4   # fp32 accumulation of exact bf16 inputs


def test_gather_chunked_equals_unchunked_and_is_deterministic(B):
    n, e, dim = 6000, 90000, 64
    src, dst, x = W.random_small_graph(13, n, e, dim, W.F32, 0.3)
    full, want, _ = run_gather(B, W.AGG_GCN, n, src, dst, x, W.F32, T=50)
    again, _, _ = run_gather(B, W.AGG_GCN, n, src, dst, x, W.F32, T=50)
    assert np.array_equal(full, again)                  # bitwise run-to-run
    chunked, _, _ = run_gather(B, W.AGG_GCN, n, src, dst, x, W.F32, T=50, chunk=7001)
    assert np.array_equal(full, chunked)                # every row produced exactly once, same order of sums
    check_features(full, want, W.F32)


@pytest.mark.parametrize("dtype,dim", [(W.F32, 64), (W.F32, 128), (W.BF16, 128), (W.BF16, 40)])
@pytest.mark.parametrize("T", [None, 50])
def test_gcn_gather_with_per_edge_coefficients(B, dtype, dim, T):
    """The source coefficient laid out per in-edge (read beside the column index) gives bitwise the result of the
    per-source look-up, and both match the oracle; the layout itself is col-gathered src_scale."""
    import torch
    n, e = 5000, 80000
    src, dst, x = W.random_small_graph(dim + 9, n, e, dim, dtype, 0.3)
    r, c, d = oracle.build_csr(n, src, dst)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    ss, sd = B.gcn_norm_scales(rp, torch.from_numpy(d).cuda())
    coef = B.gcn_edge_coefficients(cl, ss)
    assert np.array_equal(coef.cpu().numpy(), ss.cpu().numpy()[c])
    split = B.split_hubs(rp, T) if T else None
    h = B.to_device(x)
    by_lookup = B.gather_layer(W.AGG_GCN, rp, cl, h, split, ss, sd)
    by_edge = B.gather_layer(W.AGG_GCN, rp, cl, h, split, None, sd, edge_coef=coef)
    view = torch.int16 if dtype == W.BF16 else torch.int32
    assert torch.equal(by_lookup.view(view), by_edge.view(view))
    check_features(B.to_numpy(by_edge), oracle.gather(W.AGG_GCN, r, c, x, deg_out=d), dtype)
    chunked = torch.full_like(by_edge, float("nan"))
    for lo in range(0, e, 9001):
        B.gather_layer(W.AGG_GCN, rp, cl, h, split, None, sd, edge_coef=coef, edge_lo=lo,
                       edge_hi=B.INT64_MAX if lo + 9001 >= e else lo + 9001, out=chunked)
    assert torch.equal(chunked.view(view), by_edge.view(view))


@pytest.mark.parametrize("kind", [W.AGG_SUM, W.AGG_MEAN])
@pytest.mark.parametrize("dtype,dim", [(W.F32, 64), (W.BF16, 128), (W.F32, 260)])
@pytest.mark.parametrize("T", [None, 40])
def test_edge_weighted_gather(B, kind, dtype, dim, T):
    """Messages w_e * h[u] with one scalar per in-edge (CSR order), through rows, long rows and hub partials."""
    import torch
    n, e = 3000, 50000
    src, dst, x = W.random_small_graph(dim + 13, n, e, dim, dtype, 0.3)
    r, c, _ = oracle.build_csr(n, src, dst)
    w = np.random.default_rng(dim).uniform(-1.0, 1.0, e).astype(np.float32)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    split = B.split_hubs(rp, T) if T else None
    out = B.gather_layer(kind, rp, cl, B.to_device(x), split, edge_coef=torch.from_numpy(w).cuda())
    want = oracle.gather_weighted(kind, r, c, x, w)
    check_features(B.to_numpy(out), want, dtype, sum_terms=sum_scale((r, c), x, w) if kind == W.AGG_SUM else None)
    ones = torch.ones(e, dtype=torch.float32, device="cuda")
    plain = B.gather_layer(kind, rp, cl, B.to_device(x), split)
    view = torch.int16 if dtype == W.BF16 else torch.int32
    assert torch.equal(B.gather_layer(kind, rp, cl, B.to_device(x), split, edge_coef=ones).view(view), plain.view(view))


def test_gather_from_two_host_threads(B):
    """Two host threads, each on its own stream, call gather_layer with a hub split at the same time: the helper
    stream's fork/join sequences must not interleave (bitwise the single-threaded results)."""
    import threading
    import torch
    n, e, dim = 20000, 400000, 64
    graphs = []
    for seed in (41, 42):
        src, dst, x = W.random_small_graph(seed, n, e, dim, W.F32, 0.3)
        r, c, d = oracle.build_csr(n, src, dst)
        rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
        sp = B.split_hubs(rp, 64)
        h = B.to_device(x)
        ref = B.gather_layer(W.AGG_MEAN, rp, cl, h, sp)
        graphs.append((rp, cl, sp, h, ref))
    torch.cuda.synchronize()
    errors = []

    def worker(k):
        rp, cl, sp, h, ref = graphs[k]
        st = torch.cuda.Stream()
        try:
            with torch.cuda.stream(st):
                for _ in range(25):
                    out = B.gather_layer(W.AGG_MEAN, rp, cl, h, sp)
                    st.synchronize()
                    if not torch.equal(out.view(torch.int32), ref.view(torch.int32)):
                        errors.append(k)
                        return
        except Exception as ex:          # noqa: BLE001 - reported below
            errors.append(repr(ex))

    threads = [threading.Thread(target=worker, args=(k,)) for k in (0, 1)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_bf16_store_rounding_is_nearest_even_bit_exact(B):
    """Stores to bf16 go through the hardware float-pair conversion: with W = identity the update's accumulator is
    exactly x + bias (one fp32 addition), so the stored bits must equal round-to-nearest-even of that sum, ties included."""
    import torch
    d, n = 64, 4096
    rng = np.random.default_rng(77)
    x = W.store(rng.standard_normal((n, d)).astype(np.float32), W.BF16)
    bias = rng.standard_normal(d).astype(np.float32) * np.float32(0.37)
    xf = W.as_f32(x).copy()
    # exact ties: 1 + 2^-8 -> 1 (even), 1.0078125 + 2^-8 -> 1.015625 (odd mantissa rounds up), and their negatives
    xf[0, :] = 1.0
    xf[1, :] = 1.0078125
    xf[2, :] = -1.0
    xf[3, :] = -1.0078125
    bias[:8] = np.float32(2.0 ** -8)
    bias[8:16] = np.float32(-(2.0 ** -8))
    x = W.store(xf, W.BF16)
    eye = W.store(np.eye(d, dtype=np.float32), W.BF16)
    out = B.apply_layer(None, B.to_device(x), None, B.to_device(eye), torch.from_numpy(bias).cuda(), W.ACT_NONE)
    want = oracle.round_store((W.as_f32(x) + bias[None, :]).astype(np.float64), W.BF16)   # fp32 sum, then RNE
    got = B.to_numpy(out)
    assert np.array_equal(got, want), np.argwhere(got != want)[:5]
    assert W.as_f32(got)[0, 0] == 1.0 and W.as_f32(got)[1, 0] == 1.015625
    assert W.as_f32(got)[2, 8] == -1.0 and W.as_f32(got)[3, 8] == -1.015625


# ------------------------------------------------------------------------------------------ max / min
def assert_same_values(got_st, want64, what=""):
    """Extrema select one of the stored inputs: the result must equal the oracle's value exactly (as numbers:
    -0.0 == 0.0)."""
    got = W.as_f32(got_st).astype(np.float64)
    assert got.shape == want64.shape
    bad = got != want64
    assert not bad.any(), f"{what}: {int(bad.sum())} mismatches, first at {np.argwhere(bad)[0]}"


@pytest.mark.parametrize("kind", [W.AGG_MAX, W.AGG_MIN])
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_extremum_gather_dims_no_split(B, kind, dtype):
    for dim in GATHER_DIMS[dtype]:
        n, e = 3000, 40000
        src, dst, x = W.random_small_graph(dim + 1, n, e, dim, dtype, 0.15)
        got, want, _ = run_gather(B, kind, n, src, dst, x, dtype)
        assert_same_values(got, want, f"dim={dim}")


@pytest.mark.parametrize("kind", [W.AGG_MAX, W.AGG_MIN])
@pytest.mark.parametrize("dtype,dim", [(W.F32, 64), (W.F32, 128), (W.BF16, 64), (W.BF16, 128), (W.BF16, 256)])
@pytest.mark.parametrize("T", [1, 5, 64, 1000])
def test_extremum_gather_with_hub_split(B, kind, dtype, dim, T):
    n, e = 2000, 30000
    src, dst, x = W.random_small_graph(T + dim + 2, n, e, dim, dtype, 0.35)
    got, want, (r, _, _) = run_gather(B, kind, n, src, dst, x, dtype, T=T)
    assert_same_values(got, want, f"T={T}")
    assert (np.diff(r) > max(T, 512)).any()              # a hub went through partials (and beyond the long-row limit)


def test_extremum_gather_edge_cases(B):
    for n, e, hub in [(5, 0, 0.0), (1, 0, 0.0), (1, 300, 0.0), (64, 64, 1.0), (65, 4000, 0.9), (129, 1, 0.0)]:
        src, dst, x = W.random_small_graph(n + e + 1, n, e, 64, W.F32, hub)
        x = (x - np.float32(5.0)).astype(np.float32)        # all-negative rows: a zero-initialised maximum would show
        for T in (None, 16):
            for kind in (W.AGG_MAX, W.AGG_MIN):
                got, want, (r, _, _) = run_gather(B, kind, n, src, dst, x, W.F32, T=T)
                assert_same_values(got, want, f"n={n} e={e} T={T} kind={kind}")
                assert not got[np.diff(r) == 0].any()       # no in-edge: exactly zero
    # bf16 in, fp32 out and chunked launches: still the same numbers
    n, e, dim = 4000, 50000, 128
    src, dst, x = W.random_small_graph(12, n, e, dim, W.BF16, 0.3)
    got, want, _ = run_gather(B, W.AGG_MAX, n, src, dst, x, W.BF16, T=100, out_f32=True)
    assert got.dtype == np.float32
    assert_same_values(got, want)
    got, want, _ = run_gather(B, W.AGG_MIN, n, src, dst, x, W.BF16, T=100, chunk=7001)
    assert_same_values(got, want)


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_infer_with_encoder_extremum_layers_and_head(B, dtype):
    """Encoder (no gather) -> max -> min -> GCN -> mean -> prediction head (no gather), one infer_full_graph call."""
    n, e = 5000, 80000
    src, dst, x = W.random_small_graph(31, n, e, 48, dtype, 0.3)
    kinds = [W.AGG_NONE, W.AGG_MAX, W.AGG_MIN, W.AGG_GCN, W.AGG_MEAN, W.AGG_NONE]
    layers = W.dense_layers(np.random.default_rng(32), kinds, (48, 64, 64, 32, 64, 32, 8), dtype, bias_random=True)
    rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
    r, c, d = oracle.build_csr(n, src, dst)
    want = oracle.infer_full_graph(r, c, d, x, layers, dtype)
    from paper_2307_00228_amd import compose
    import torch
    for T in (None, 40):
        split = B.split_hubs(rowptr, T) if T else None
        dl, xd = B.device_layers(layers), B.to_device(x)
        out = B.infer_full_graph(rowptr, col, deg_out, split, dl, xd)
        if dtype == W.F32:
            check_features(B.to_numpy(out), W.as_f32(want), dtype, f"T={T}")
        view = torch.int16 if dtype == W.BF16 else torch.int32
        again = B.infer_full_graph(rowptr, col, deg_out, split, dl, xd, edge_chunk=9000)
        assert torch.equal(out.view(view), again.view(view))
        steps = compose.run_layers(rowptr, col, deg_out, split, dl, xd)
        assert torch.equal(out.view(view), steps[-1].out.view(view))
        # every layer on its own, from the state the GPU stored for the previous one (six bf16 roundings in a row,
        # two of them through an extremum that picks the worst case, do not average out end to end)
        h = x
        for i, (lay, tr) in enumerate(zip(layers, steps)):
            check_layer(B, tr, r, c, d, h, lay, dtype, f"T={T} layer {i}")
            if lay.agg in (W.AGG_MAX, W.AGG_MIN):
                assert_same_values(B.to_numpy(tr.agg), oracle.gather(lay.agg, r, c, h), f"T={T} layer {i} aggregate")
            h = B.to_numpy(tr.out)


# ------------------------------------------------------------------------------------------ apply
APPLY_CASES = [(W.F32, 64, 64), (W.F32, 64, 16), (W.F32, 128, 128), (W.F32, 128, 64), (W.F32, 8, 1), (W.F32, 256, 256),
               (W.F32, 40, 100), (W.BF16, 128, 128), (W.BF16, 64, 64), (W.BF16, 64, 32), (W.BF16, 256, 256),
               (W.BF16, 16, 7), (W.BF16, 48, 200),
               # widths that are not whole k-chunks (padded k range), and output widths beyond one pass of column tiles
               (W.F32, 100, 47), (W.F32, 200, 64), (W.F32, 12, 300), (W.F32, 52, 8), (W.BF16, 200, 64), (W.BF16, 40, 24),
               (W.BF16, 104, 512), (W.BF16, 8, 8)]


@pytest.mark.parametrize("dtype,d_in,d_out", APPLY_CASES)
@pytest.mark.parametrize("n", [1, 31, 257, 5000])
def test_apply_layer(B, dtype, d_in, d_out, n):
    rng = np.random.default_rng(d_in * 1000 + d_out + n)
    h = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    a = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    lay = W.dense_layers(rng, W.AGG_MEAN, (d_in, d_out, d_out), dtype, bias_random=True)[0]
    for act, with_self, with_bias in [(W.ACT_RELU, True, True), (W.ACT_NONE, False, False)]:
        out = B.apply_layer(B.to_device(h) if with_self else None, B.to_device(a),
                            B.to_device(lay.w_self) if with_self else None, B.to_device(lay.w_nbr),
                            B.to_device(lay.bias) if with_bias else None, act)
        want = oracle.apply(h if with_self else None, a, lay.w_self if with_self else None, lay.w_nbr,
                            lay.bias if with_bias else None, act)
        check_features(B.to_numpy(out), want, dtype, f"act={act} self={with_self}")


@pytest.mark.parametrize("dtype,d_in,d_out", [(W.F32, 768, 96), (W.BF16, 768, 256), (W.BF16, 1000, 40), (W.F32, 600, 7)])
def test_apply_wide_input_without_self_term(B, dtype, d_in, d_out):
    """Encoder-style layers: input widths of raw features (hundreds), no self matrix; and the widths that do not fit are
    refused with a status, not attempted."""
    n = 3000
    rng = np.random.default_rng(d_in + d_out)
    a = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    lay = W.dense_layers(rng, W.AGG_NONE, (d_in, d_out, d_out), dtype, bias_random=True)[0]
    out = B.apply_layer(None, B.to_device(a), None, B.to_device(lay.w_nbr), B.to_device(lay.bias), W.ACT_RELU)
    want = oracle.apply(None, a, None, lay.w_nbr, lay.bias, W.ACT_RELU)
    check_features(B.to_numpy(out), want, dtype)
    if dtype == W.F32 and d_in == 768:      # with a self matrix the 2 x 768 x 32 fp32 panel alone exceeds the LDS
        wide = W.dense_layers(rng, W.AGG_MEAN, (d_in, d_out, d_out), dtype)[0]
        with pytest.raises(B.InferTurboError, match="UNSUPPORTED"):
            B.apply_layer(B.to_device(a), B.to_device(a), B.to_device(wide.w_self), B.to_device(wide.w_nbr), None, W.ACT_NONE)
    with pytest.raises(B.InferTurboError, match="UNSUPPORTED"):      # rows must be whole 16-byte pieces
        bad = 6 if dtype == W.F32 else 12
        x = B.to_device(W.store(np.zeros((4, bad), np.float32), dtype))
        B.apply_layer(None, x, None, B.to_device(W.store(np.zeros((bad, 8), np.float32), dtype)), None, W.ACT_NONE)


@pytest.mark.parametrize("dtype,d_in,d_out", [(W.F32, 64, 64), (W.F32, 128, 40), (W.BF16, 64, 128), (W.BF16, 32, 16)])
@pytest.mark.parametrize("n", [5, 300, 4001])
def test_apply_message_output_and_scale_rows(B, dtype, d_in, d_out, n):
    """The scatter-side message h' * c(v): second output of the update, and scale_rows for the input features."""
    import torch
    rng = np.random.default_rng(n + d_in)
    h = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    a = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    scale = rng.uniform(0.05, 1.0, n).astype(np.float32)
    lay = W.dense_layers(rng, W.AGG_GCN, (d_in, d_out, d_out), dtype, bias_random=True)[0]
    msg = torch.empty((n, d_out), dtype=B.to_device(h).dtype, device="cuda")
    out = B.apply_layer(B.to_device(h), B.to_device(a), B.to_device(lay.w_self), B.to_device(lay.w_nbr), B.to_device(lay.bias),
                        W.ACT_RELU, msg_scale=torch.from_numpy(scale).cuda(), msg_out=msg)
    y64 = oracle.apply(h, a, lay.w_self, lay.w_nbr, lay.bias, oracle.ACT_RELU)
    check_features(B.to_numpy(out), y64, dtype)
    check_features(B.to_numpy(msg), y64 * scale[:, None].astype(np.float64), dtype)
    xs = B.scale_rows(B.to_device(h), torch.from_numpy(scale).cuda())
    check_features(B.to_numpy(xs), W.as_f32(h).astype(np.float64) * scale[:, None].astype(np.float64), dtype)


@pytest.mark.parametrize("dtype,dims", [(W.F32, (64, 32, 32)), (W.F32, (48, 48, 16)), (W.BF16, (128, 64, 32)), (W.BF16, (64, 128, 128))])
def test_gcn_stack(B, dtype, dims):
    """GCN layers: the first one has no message rows yet (scale_rows makes them), later ones read the rows the previous
    update left; narrowing layers apply W_nbr before the gather."""
    import torch
    from paper_2307_00228_amd import compose
    n, e = 6000, 90000
    src, dst, x = W.random_small_graph(sum(dims), n, e, dims[0], dtype, 0.3)
    layers = W.dense_layers(np.random.default_rng(dims[1]), W.AGG_GCN, dims, dtype, bias_random=True)
    rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
    r, c, d = oracle.build_csr(n, src, dst)
    dl, xd = B.device_layers(layers), B.to_device(x)
    assert compose.plan(dl, xd.dtype) == [dims[i + 1] < dims[i] for i in range(len(dims) - 1)]
    for T in (None, 60):
        split = B.split_hubs(rowptr, T) if T else None
        steps = compose.run_layers(rowptr, col, deg_out, split, dl, xd)
        out = B.infer_full_graph(rowptr, col, deg_out, split, dl, xd)
        view = torch.int16 if dtype == W.BF16 else torch.int32
        assert torch.equal(out.view(view), steps[-1].out.view(view))
        h = x
        for i, (lay, tr) in enumerate(zip(layers, steps)):
            check_layer(B, tr, r, c, d, h, lay, dtype, f"T={T} layer {i}")
            h = B.to_numpy(tr.out)


@pytest.mark.parametrize("dtype,d_in,d_out", [(W.F32, 64, 16), (W.F32, 128, 64), (W.BF16, 64, 32), (W.BF16, 128, 40),
                                              (W.F32, 64, 47), (W.BF16, 64, 20), (W.BF16, 200, 300)])
@pytest.mark.parametrize("n", [7, 1000, 4100])
def test_apply_with_addend(B, dtype, d_in, d_out, n):
    """h_out = act(h . W + addend + bias), optionally with the message output."""
    import torch
    rng = np.random.default_rng(n + d_out)
    h = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    add = W.store(rng.standard_normal((n, d_out)).astype(np.float32), dtype)
    scale = rng.uniform(0.1, 1.0, n).astype(np.float32)
    lay = W.dense_layers(rng, W.AGG_MEAN, (d_in, d_out, d_out), dtype, bias_random=True)[0]
    y64 = oracle.apply(None, h, None, lay.w_self, lay.bias, oracle.ACT_NONE) + W.as_f32(add).astype(np.float64)
    want = np.maximum(y64, 0.0)
    out = B.apply_layer(None, B.to_device(h), None, B.to_device(lay.w_self), B.to_device(lay.bias), W.ACT_RELU,
                        addend=B.to_device(add))
    check_features(B.to_numpy(out), want, dtype)
    msg = torch.empty_like(out)
    out2 = B.apply_layer(None, B.to_device(h), None, B.to_device(lay.w_self), B.to_device(lay.bias), W.ACT_RELU,
                         addend=B.to_device(add), msg_scale=torch.from_numpy(scale).cuda(), msg_out=msg)
    assert torch.equal(out2.view(torch.int16 if dtype == W.BF16 else torch.int32), out.view(torch.int16 if dtype == W.BF16 else torch.int32))
    check_features(B.to_numpy(msg), want * scale[:, None].astype(np.float64), dtype)


@pytest.mark.parametrize("dtype,d_in,d_out", [(W.F32, 128, 64), (W.F32, 64, 16), (W.BF16, 64, 32), (W.BF16, 128, 64),
                                              (W.BF16, 200, 40), (W.F32, 100, 4), (W.BF16, 256, 128), (W.F32, 64, 200)])
@pytest.mark.parametrize("n", [3, 1000, 4100])
def test_apply_second_product(B, dtype, d_in, d_out, n):
    """Two products of the same rows in one launch: out = act(x W1 + b), out_second = x W2 (plain)."""
    import torch
    rng = np.random.default_rng(n + d_in + d_out)
    x = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    lay = W.dense_layers(rng, W.AGG_MEAN, (d_in, d_out, d_out), dtype, bias_random=True)[0]
    xd = B.to_device(x)
    out, second = B.apply_layer(None, xd, None, B.to_device(lay.w_nbr), B.to_device(lay.bias), W.ACT_RELU,
                                w_second=B.to_device(lay.w_self))
    check_features(B.to_numpy(out), oracle.apply(None, x, None, lay.w_nbr, lay.bias, oracle.ACT_RELU), dtype, "first")
    check_features(B.to_numpy(second), oracle.apply(None, x, None, lay.w_self, None, oracle.ACT_NONE), dtype, "second")
    # each product bitwise equal to the single-product launch
    view = torch.int16 if dtype == W.BF16 else torch.int32
    alone1 = B.apply_layer(None, xd, None, B.to_device(lay.w_nbr), B.to_device(lay.bias), W.ACT_RELU)
    alone2 = B.apply_layer(None, xd, None, B.to_device(lay.w_self), None, W.ACT_NONE)
    assert torch.equal(out.view(view), alone1.view(view)) and torch.equal(second.view(view), alone2.view(view))


@pytest.mark.parametrize("d_in,with_self", [(64, True), (64, False), (128, True), (256, True), (320, False), (448, True)])
@pytest.mark.parametrize("dc", [32, 16, 8, 24])
@pytest.mark.parametrize("n", [1, 37, 1000, 4100])
def test_apply_chained_projection(B, d_in, with_self, dc, n):
    """The finished rows of an update (bf16, 64 columns) multiplied by two more matrices in the same launch:
    y = act(h W_self + agg W_nbr + b), out_first = round(y) W_c1, out_second = round(y) W_c2 -- the oracle applies the
    two steps one after the other with the stored rounding in between; the chained launch gives the same bits as the
    two separate launches, with and without storing y."""
    import torch
    rng = np.random.default_rng(n + d_in + dc)
    dtype = W.BF16
    h = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    agg = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    lay = W.dense_layers(rng, W.AGG_MEAN, (d_in, 64, 64), dtype, bias_random=True)[0]
    nxt = W.dense_layers(rng, W.AGG_MEAN, (64, dc, dc), dtype)[0]
    hd, ad = B.to_device(h), B.to_device(agg)
    ws = B.to_device(lay.w_self) if with_self else None
    wn, bias = B.to_device(lay.w_nbr), B.to_device(lay.bias)
    c1, c2 = B.to_device(nxt.w_nbr), B.to_device(nxt.w_self)
    y, p1, p2 = B.apply_layer(hd if with_self else None, ad, ws, wn, bias, W.ACT_RELU, chain=(c1, c2))
    y64 = oracle.apply(h if with_self else None, agg, lay.w_self if with_self else None, lay.w_nbr, lay.bias, oracle.ACT_RELU)
    check_features(B.to_numpy(y), y64, dtype, "y")
    y_st = oracle.round_store(y64, dtype)
    check_features(B.to_numpy(p1), oracle.apply(None, y_st, None, nxt.w_nbr, None, oracle.ACT_NONE), dtype, "first")
    check_features(B.to_numpy(p2), oracle.apply(None, y_st, None, nxt.w_self, None, oracle.ACT_NONE), dtype, "second")
    # the same bits as update and projection issued one after the other
    y_alone = B.apply_layer(hd if with_self else None, ad, ws, wn, bias, W.ACT_RELU)
    q1, q2 = B.apply_layer(None, y_alone, None, c1, None, W.ACT_NONE, w_second=c2)
    view = torch.int16
    assert torch.equal(y.view(view), y_alone.view(view))
    assert torch.equal(p1.view(view), q1.view(view)) and torch.equal(p2.view(view), q2.view(view))
    # and without ever storing y
    none, r1, r2 = B.apply_layer(hd if with_self else None, ad, ws, wn, bias, W.ACT_RELU, chain=(c1, c2), store_out=False)
    assert none is None and torch.equal(r1.view(view), p1.view(view)) and torch.equal(r2.view(view), p2.view(view))


@pytest.mark.parametrize("dims,kinds", [((64, 64, 32), (W.AGG_MEAN, W.AGG_MEAN)), ((64, 64, 16), (W.AGG_GCN, W.AGG_SUM)),
                                        ((64, 64, 32, 8), (W.AGG_MEAN, W.AGG_MEAN, W.AGG_MEAN)),
                                        ((64, 64, 64, 32), (W.AGG_MAX, W.AGG_MEAN, W.AGG_GCN))])
@pytest.mark.parametrize("chunk", [0, 9000])
def test_layer_loop_chains_an_update_into_the_next_projection(B, dims, kinds, chunk):
    """bf16 stacks in which a 64-wide gather -> update layer is followed by a narrowing layer: the plan reports the
    chaining, the single call matches the oracle and equals, bit for bit, the same model with chaining switched off and
    the call-by-call composition."""
    import torch
    from paper_2307_00228_amd import compose
    dtype = W.BF16
    n, e = 5000, 60000
    src, dst, x = W.random_small_graph(sum(dims), n, e, dims[0], dtype, 0.3)
    rng = np.random.default_rng(dims[-1])
    layers = []
    for i, kind in enumerate(kinds):
        lay = W.dense_layers(rng, kind, (dims[i], dims[i + 1], dims[i + 1]), dtype, bias_random=True)[0]
        lay.act = W.ACT_RELU if i + 1 < len(kinds) else W.ACT_NONE
        layers.append(lay)
    r, c, d = oracle.build_csr(n, src, dst)
    rp, cl, dg = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda(), torch.from_numpy(d).cuda()
    split = B.split_hubs(rp, 1500)
    dl = B.device_layers(layers)
    plan = B.infer_layer_plan(dl, torch.bfloat16)
    assert B.PLAN_GATHER_UPDATE_CHAINED in plan
    for i, pl in enumerate(plan):
        if pl == B.PLAN_GATHER_UPDATE_CHAINED:
            assert plan[i + 1] == B.PLAN_PROJECT_GATHER and dims[i + 1] == 64
    xd = B.to_device(x)
    got = B.infer_full_graph(rp, cl, dg, split, dl, xd, edge_chunk=chunk)
    torch.cuda.synchronize()
    tr = compose.run_layers(rp, cl, dg, split, dl, xd)
    assert torch.equal(tr[-1].out.view(torch.int16), got.view(torch.int16))
    assert any(t.out is None for t in tr)
    B.set_tuning(9, 0)
    try:
        assert B.PLAN_GATHER_UPDATE_CHAINED not in B.infer_layer_plan(dl, torch.bfloat16)
        plain = B.infer_full_graph(rp, cl, dg, split, dl, xd, edge_chunk=chunk)
        steps = compose.run_layers(rp, cl, dg, split, dl, xd)
        torch.cuda.synchronize()
    finally:
        B.set_tuning(9, 1)
    # every layer of the unchained run against Eq. (1) from the state stored for the layer before; the chained run
    # must then give the same bits
    h = x
    for i, (lay, st) in enumerate(zip(layers, steps)):
        check_layer(B, st, r, c, d, h, lay, dtype, f"layer {i} of {kinds} {dims}")
        h = B.to_numpy(st.out)
    assert torch.equal(steps[-1].out.view(torch.int16), got.view(torch.int16))
    assert torch.equal(plain.view(torch.int16), got.view(torch.int16))


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("rows,cin,cout", [(1, 1, 8), (37, 47, 48), (1000, 48, 47), (5, 10, 10), (4099, 3, 16), (64, 130, 7)])
def test_copy_columns_bit_exact(B, dtype, rows, cin, cout):
    import torch
    rng = np.random.default_rng(rows + cin + cout)
    a = W.store(rng.standard_normal((rows, cin)).astype(np.float32), dtype)
    got = B.to_numpy(B.copy_columns(B.to_device(a), cout))
    want = np.zeros((rows, cout), dtype=a.dtype)
    k = min(cin, cout)
    want[:, :k] = a[:, :k]
    assert got.shape == want.shape and np.array_equal(np.asarray(got).view(np.uint8), want.view(np.uint8))


@pytest.mark.parametrize("dtype,dims", [(W.BF16, (64, 64, 47)), (W.BF16, (128, 41)), (W.BF16, (64, 64, 3)), (W.F32, (128, 64, 10)),
                                        (W.F32, (64, 47)), (W.F32, (32, 16, 5))])
@pytest.mark.parametrize("kind", [W.AGG_MEAN, W.AGG_GCN])
def test_last_layer_of_any_width_is_projected_through_padding(B, dtype, dims, kind):
    """A narrowing last layer whose width is not whole 16-byte pieces (47 classes, say) still takes W_nbr before its
    gather: on zero-padded copies of its matrices, the padding dropped when the output is stored.  Plan, every layer
    against Eq. (1), bitwise equality of the single call (chunked or not) with the call-by-call composition, and -- for
    bf16 stacks with a 64-wide layer in front -- with the chained update switched off."""
    import torch
    from dataclasses import replace
    from paper_2307_00228_amd import compose
    n, e = 4000, 50000
    src, dst, x = W.random_small_graph(sum(dims) + kind, n, e, dims[0], dtype, 0.3)
    rng = np.random.default_rng(dims[-1] + kind)
    layers = []
    for i in range(len(dims) - 1):
        lay = W.dense_layers(rng, kind, (dims[i], dims[i + 1], dims[i + 1]), dtype, bias_random=True)[0]
        layers.append(replace(lay, act=W.ACT_RELU if i + 2 < len(dims) else W.ACT_NONE))
    r, c, d = oracle.build_csr(n, src, dst)
    rp, cl, dg = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda(), torch.from_numpy(d).cuda()
    split = B.split_hubs(rp, 900)
    dl, xd = B.device_layers(layers), B.to_device(x)
    tdt = torch.bfloat16 if dtype == W.BF16 else torch.float32
    plan = B.infer_layer_plan(dl, tdt)
    assert plan[-1] == B.PLAN_PROJECT_GATHER
    view = torch.int16 if dtype == W.BF16 else torch.int32
    got = B.infer_full_graph(rp, cl, dg, split, dl, xd)
    assert tuple(got.shape) == (n, dims[-1])
    chunked = B.infer_full_graph(rp, cl, dg, split, dl, xd, edge_chunk=e // 3)
    assert torch.equal(got.view(view), chunked.view(view))
    B.set_tuning(9, 0)
    try:
        steps = compose.run_layers(rp, cl, dg, split, dl, xd)
        plain = B.infer_full_graph(rp, cl, dg, split, dl, xd)
        torch.cuda.synchronize()
    finally:
        B.set_tuning(9, 1)
    assert torch.equal(got.view(view), plain.view(view)) and torch.equal(got.view(view), steps[-1].out.view(view))
    tr = compose.run_layers(rp, cl, dg, split, dl, xd)
    assert torch.equal(got.view(view), tr[-1].out.view(view))
    h = x
    for i, (lay, st) in enumerate(zip(layers, steps)):
        check_layer(B, st, r, c, d, h, lay, dtype, f"layer {i} of {dims}")
        h = B.to_numpy(st.out)


@pytest.mark.parametrize("kind", [W.AGG_SUM, W.AGG_MEAN, W.AGG_GCN])
@pytest.mark.parametrize("dtype,dim", [(W.F32, 64), (W.F32, 16), (W.BF16, 32), (W.BF16, 64), (W.BF16, 520)])
@pytest.mark.parametrize("T", [None, 40])
def test_gather_with_fused_update(B, kind, dtype, dim, T):
    """The update in the gather's row epilogue: out = act(agg + addend + bias), through short rows, whole-wavefront
    rows, long rows (limit lowered), hub partials + combine, and edge-range chunks."""
    import torch
    n, e = 3000, 50000
    src, dst, x = W.random_small_graph(dim + 21, n, e, dim, dtype, 0.3)
    r, c, d = oracle.build_csr(n, src, dst)
    rng = np.random.default_rng(dim + 22)
    add = W.store(rng.standard_normal((n, dim)).astype(np.float32), dtype)
    bias = rng.uniform(-0.5, 0.5, dim).astype(np.float32)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    split = B.split_hubs(rp, T) if T else None
    ss = sd = None
    if kind == W.AGG_GCN:
        ss, sd = B.gcn_norm_scales(rp, torch.from_numpy(d).cuda())
    h, addd, biasd = B.to_device(x), B.to_device(add), torch.from_numpy(bias).cuda()
    a64 = oracle.gather(kind, r, c, x, deg_out=d)
    want = np.maximum(a64 + W.as_f32(add).astype(np.float64) + bias, 0.0)
    view = torch.int16 if dtype == W.BF16 else torch.int32
    B.set_tuning(3, 40)
    try:
        out = B.gather_layer(kind, rp, cl, h, split, ss, sd, addend=addd, bias=biasd, act=W.ACT_RELU)
        chunked = torch.full_like(out, float("nan"))
        for lo in range(0, e, 7001):
            B.gather_layer(kind, rp, cl, h, split, ss, sd, addend=addd, bias=biasd, act=W.ACT_RELU, edge_lo=lo,
                           edge_hi=B.INT64_MAX if lo + 7001 >= e else lo + 7001, out=chunked)
        torch.cuda.synchronize()
    finally:
        B.set_tuning(3, 512)
    check_features(B.to_numpy(out), want, dtype, sum_terms=sum_scale((r, c), x) if kind == W.AGG_SUM else None)
    assert torch.equal(out.view(view), chunked.view(view))
    # bias alone, and no activation
    out2 = B.gather_layer(kind, rp, cl, h, split, ss, sd, bias=biasd)
    check_features(B.to_numpy(out2), a64 + bias, dtype, sum_terms=sum_scale((r, c), x) if kind == W.AGG_SUM else None)


# ------------------------------------------------------------------------------------------ edge feature vectors
def edge_case(seed, n, e, d, d_e, dtype, hub=0.3):
    src, dst, x = W.random_small_graph(seed, n, e, d, dtype, hub)
    rng = np.random.default_rng(seed + 1)
    ef = W.store(rng.standard_normal((e, d_e)).astype(np.float32), dtype)       # per in-edge, CSR order
    return src, dst, x, ef, rng


@pytest.mark.parametrize("kind", [W.AGG_SUM, W.AGG_MEAN, W.AGG_GCN])
@pytest.mark.parametrize("dtype,d_e", [(W.F32, 4), (W.F32, 16), (W.F32, 36), (W.BF16, 8), (W.BF16, 16), (W.BF16, 72)])
@pytest.mark.parametrize("T", [None, 40])
def test_aggregate_edge_features(B, kind, dtype, d_e, T):
    """Per-destination reduce of the per-edge feature table (streamed in CSR order), through short rows, long rows and
    hub partials; against the oracle's per-edge message gather with zero states and W_e = identity."""
    import torch
    n, e = 3000, 50000
    src, dst, x, ef, _ = edge_case(d_e + 31, n, e, d_e, d_e, dtype)
    r, c, d = oracle.build_csr(n, src, dst)
    rp = torch.from_numpy(r).cuda()
    split = B.split_hubs(rp, T) if T else None
    coef = sd = None
    if kind == W.AGG_GCN:
        ss, sd = B.gcn_norm_scales(rp, torch.from_numpy(d).cuda())
        coef = B.gcn_edge_coefficients(torch.from_numpy(c).cuda(), ss)
    B.set_tuning(3, 40)
    try:
        got = B.aggregate_edge_features(kind, rp, B.to_device(ef), split, edge_coef=coef, dst_scale=sd)
        torch.cuda.synchronize()
    finally:
        B.set_tuning(3, 512)
    want = oracle.gather_edge_features(kind, r, c, np.zeros((n, d_e), np.float32), ef, np.eye(d_e, dtype=np.float32), deg_out=d)
    check_features(B.to_numpy(got), want, dtype, sum_terms=sum_scale_edges(r, ef) if kind == W.AGG_SUM else None)


def sum_scale_edges(r, ef):
    """Root-sum-square of the terms of every element of a per-destination sum of per-edge rows."""
    import scipy.sparse as sp
    n, e = len(r) - 1, len(ef)
    return np.sqrt(sp.csr_matrix((np.ones(e), np.arange(e), r), shape=(n, e)) @ (W.as_f32(ef).astype(np.float64) ** 2))


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("kinds", [(W.AGG_MEAN, W.AGG_MEAN), (W.AGG_GCN, W.AGG_SUM), (W.AGG_SUM, W.AGG_MAX)])
def test_layers_with_edge_features(B, dtype, kinds):
    """Layers whose messages carry an edge feature vector, m_e = h[u] + ef[e] W_e, through infer_full_graph: equal to the
    call-by-call loop bitwise, chunked or not, and every layer within its bar of Eq. (1) with those messages."""
    import torch
    from dataclasses import replace
    from paper_2307_00228_amd import compose
    n, e, d_e = 4000, 60000, 8
    dims = (32, 64, 32)             # the second layer narrows: with an edge matrix it still runs gather -> update
    src, dst, x, ef, rng = edge_case(51, n, e, dims[0], d_e, dtype)
    layers = W.dense_layers(rng, list(kinds), dims, dtype, bias_random=True)
    # edge matrices on every linear layer (the extremum layer, if any, takes plain states)
    layers = [replace(l, w_edge=W.store(rng.uniform(-0.4, 0.4, (d_e, l.d_in)).astype(np.float32), dtype))
              if l.agg in (W.AGG_SUM, W.AGG_MEAN, W.AGG_GCN) else l for l in layers]
    rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
    r, c, d = oracle.build_csr(n, src, dst)
    dl, xd, efd = B.device_layers(layers), B.to_device(x), B.to_device(ef)
    assert compose.plan(dl, xd.dtype) == [False, False]
    view = torch.int16 if dtype == W.BF16 else torch.int32
    for T in (None, 50):
        split = B.split_hubs(rowptr, T) if T else None
        out = B.infer_full_graph(rowptr, col, deg_out, split, dl, xd, edge_feat=efd)
        chunked = B.infer_full_graph(rowptr, col, deg_out, split, dl, xd, edge_feat=efd, edge_chunk=e // 4)
        steps = compose.run_layers(rowptr, col, deg_out, split, dl, xd, edge_feat=efd)
        assert torch.equal(out.view(view), chunked.view(view)) and torch.equal(out.view(view), steps[-1].out.view(view))
        h = x
        for i, (lay, tr) in enumerate(zip(layers, steps)):
            _, y64, a64 = oracle.dense_layer(r, c, d, h, lay, dtype, return_agg64=True, edge_feat=ef)
            slack = 0.0 if lay.agg == W.AGG_MAX else agg_rounding_slack(a64, lay.w_nbr, dtype)
            if dtype == W.BF16 and lay.w_edge is not None:
                # the edge term (reduced edge features, then their product with W_e) is stored in bf16 twice on its way
                # into the aggregate: each rounding moves it by at most 2^-9 relative
                et = np.abs(W.as_f32(B.to_numpy(tr.edge_term)).astype(np.float64))
                slack = slack + 2.0 ** -8 * (et @ np.abs(W.as_f32(lay.w_nbr).astype(np.float64)))
            # an un-normalised sum makes states in the hundreds on the hub: fp32 holds 1e-4 relative to the magnitude there
            unnormalised = W.AGG_SUM in kinds
            check_features(B.to_numpy(tr.out), y64, dtype, f"T={T} layer {i}", slack=slack,
                           sum_terms=np.abs(y64) if unnormalised else None)
            h = B.to_numpy(tr.out)
    # what the reading does not cover is refused: an edge matrix on a max layer, a feature width that is not whole 16-byte rows
    bad = [replace(layers[0], agg=W.AGG_MAX)]
    with pytest.raises(B.InferTurboError, match="UNSUPPORTED"):
        B.infer_full_graph(rowptr, col, deg_out, None, B.device_layers(bad), xd, edge_feat=efd)
    with pytest.raises(B.InferTurboError, match="UNSUPPORTED"):
        B.infer_full_graph(rowptr, col, deg_out, None, dl[:1], xd, edge_feat=efd[:, :3].contiguous())


def test_gcn_gather_of_prescaled_rows(B):
    import torch
    n, e, dim = 5000, 80000, 128
    src, dst, x = W.random_small_graph(321, n, e, dim, W.F32, 0.25)
    r, c, d = oracle.build_csr(n, src, dst)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    ss, sd = B.gcn_norm_scales(rp, torch.from_numpy(d).cuda())
    want = oracle.gather(oracle.GCN, r, c, x, deg_out=d)
    for T in (None, 100):
        split = B.split_hubs(rp, T) if T else None
        out = B.gather_layer(W.AGG_GCN, rp, cl, B.scale_rows(B.to_device(x), ss), split, None, sd)
        check_features(B.to_numpy(out), want, W.F32, f"T={T}")


# ------------------------------------------------------------------------------------------ GAT
@pytest.mark.parametrize("dtype,heads,dh", [(W.F32, 4, 16), (W.F32, 1, 64), (W.BF16, 4, 64), (W.BF16, 2, 8), (W.BF16, 8, 32)])
@pytest.mark.parametrize("T", [None, 7, 300])
def test_gat_gather(B, dtype, heads, dh, T):
    import torch
    n, e, dim = 2500, 36000, heads * dh
    src, dst, z = W.random_small_graph(heads * 100 + dh, n, e, dim, dtype, 0.3)
    dst[dst == 5] = 6                                   # vertex 5 is isolated: attends to itself only
    rng = np.random.default_rng(dim)
    s_src = (rng.standard_normal((n, heads)) * 2).astype(np.float32)
    s_dst = (rng.standard_normal((n, heads)) * 2).astype(np.float32)
    bias = rng.uniform(-0.5, 0.5, dim).astype(np.float32)
    r, c, _ = oracle.build_csr(n, src, dst)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    split = B.split_hubs(rp, T) if T is not None else None
    for act, b in ((W.ACT_NONE, None), (W.ACT_RELU, bias)):
        out = B.gather_layer(W.AGG_GAT, rp, cl, B.to_device(z), split, torch.from_numpy(s_src).cuda(),
                             torch.from_numpy(s_dst).cuda(), heads=heads, leaky_slope=0.2, act=act,
                             bias=None if b is None else torch.from_numpy(b).cuda())
        want = oracle.gat_gather(r, c, z, s_src, s_dst, heads, 0.2)
        if b is not None:
            want = np.maximum(want + b, 0.0)
        check_features(B.to_numpy(out), want, dtype, f"act={act}")
        if b is None:
            np.testing.assert_allclose(W.as_f32(B.to_numpy(out))[5], W.as_f32(z)[5], rtol=1e-6)


@pytest.mark.parametrize("dtype,d_in,heads,dh", [(W.F32, 64, 4, 32), (W.BF16, 256, 4, 64), (W.BF16, 64, 1, 64), (W.BF16, 32, 3, 64),
                                                 (W.BF16, 128, 2, 128), (W.BF16, 64, 1, 256), (W.F32, 96, 8, 4), (W.BF16, 48, 16, 8),
                                                 (W.F32, 200, 2, 16), (W.BF16, 64, 3, 24), (W.F32, 32, 1, 32), (W.BF16, 512, 2, 64)])
@pytest.mark.parametrize("n", [1, 33, 3000])
def test_apply_projection_with_scores(B, dtype, d_in, heads, dh, n):
    """z = h W and the attention scores of every head from the unrounded z.  The scores come out of the epilogue where
    the head width is a power of two inside one column block (by default only for d_in >= 256, where it is faster), else out
    of an extra score tile: both ways are forced in turn and held to the same bar; z is the same bits either way."""
    import torch
    rng = np.random.default_rng(d_in + heads + n)
    h = W.store(rng.standard_normal((n, d_in)).astype(np.float32), dtype)
    lay = W.gat_layers(rng, (d_in, heads * dh), heads, dtype)[0]
    z64 = oracle.apply(None, h, None, lay.w_nbr, None, oracle.ACT_NONE)
    outs = []
    try:
        for epilogue in (2, 0):
            B.set_tuning(10, epilogue)
            out, s_src, s_dst = B.apply_layer(None, B.to_device(h), None, B.to_device(lay.w_nbr), None, W.ACT_NONE, heads=heads,
                                              att_src=B.to_device(lay.att_src), att_dst=B.to_device(lay.att_dst))
            torch.cuda.synchronize()
            check_features(B.to_numpy(out), z64, dtype, f"epilogue={epilogue}")
            for got, att in ((s_src, lay.att_src), (s_dst, lay.att_dst)):
                want = oracle.gat_scores(z64, att)
                assert np.abs(got.cpu().numpy() - want).max() <= 1e-4 * max(1.0, np.abs(want).max()), f"epilogue={epilogue}"
            outs.append(out)
    finally:
        B.set_tuning(10, 1)
    view = torch.int16 if dtype == W.BF16 else torch.int32
    assert torch.equal(outs[0].view(view), outs[1].view(view))


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_gat_layers_small_graph(B, dtype):
    import torch
    n, e = 3000, 30000
    src, dst, x = W.random_small_graph(77, n, e, 64, dtype, 0.3)
    rng = np.random.default_rng(78)
    layers = W.gat_layers(rng, (64, 128, 64), 2, dtype, bias_random=True)
    rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
    r, c, d = oracle.build_csr(n, src, dst)
    want = oracle.infer_full_graph(r, c, d, x, layers, dtype)
    for T in (None, 50):
        split = B.split_hubs(rowptr, T) if T else None
        out = B.infer_full_graph(rowptr, col, deg_out, split, B.device_layers(layers), B.to_device(x))
        check_features(B.to_numpy(out), W.as_f32(want), dtype, f"T={T}")


# ------------------------------------------------------------------------------------------ whole path
@pytest.mark.parametrize("name,scale", [("tiny_powerlaw", 1.0), ("medium_uniform", 0.02), ("hub_heavy", 0.005),
                                        ("hub_heavy_uniform_control", 0.005), ("huge_share", 0.0003),
                                        ("attention", 0.005)])
def test_infer_full_graph_matches_oracle(B, name, scale):
    import torch
    w = W.make(name, scale, bias_random=True)
    rowptr, col, deg_out = B.build_csr_by_dst(w.n_nodes, dev_i32(w.src), dev_i32(w.dst))
    split = B.split_hubs(rowptr, w.threshold) if w.threshold < W.NO_SPLIT else None
    layers = B.device_layers(w.layers)
    x = B.to_device(w.x)
    out = B.infer_full_graph(rowptr, col, deg_out, split, layers, x)
    r, c, d = oracle.build_csr(w.n_nodes, w.src, w.dst)
    assert np.array_equal(rowptr.cpu().numpy(), r) and np.array_equal(col.cpu().numpy(), c)
    if split is not None and name == "hub_heavy":
        assert split.n_hubs >= 16
    want = oracle.infer_full_graph(r, c, d, w.x, w.layers, w.dtype)
    check_features(B.to_numpy(out), W.as_f32(want), w.dtype, name)
    # bitwise reproducible, also through the chunked launch path
    out2 = B.infer_full_graph(rowptr, col, deg_out, split, layers, x, edge_chunk=max(1, w.n_edges // 5))
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16 if w.dtype == W.BF16 else torch.int32),
                       out2.view(torch.int16 if w.dtype == W.BF16 else torch.int32))


def test_infer_split_equals_unsplit(B):
    """Shadow split + partial-gather leaves the result unchanged (within fp32 reassociation)."""
    w = W.make("tiny_powerlaw", 1.0)
    rowptr, col, deg_out = B.build_csr_by_dst(w.n_nodes, dev_i32(w.src), dev_i32(w.dst))
    layers, x = B.device_layers(w.layers), B.to_device(w.x)
    whole = B.infer_full_graph(rowptr, col, deg_out, None, layers, x)
    for T in (64, 4096):
        parts = B.infer_full_graph(rowptr, col, deg_out, B.split_hubs(rowptr, T), layers, x)
        assert (whole - parts).abs().max().item() <= 1e-5


# ------------------------------------------------------------------------------------------ randomised sweep
@pytest.mark.parametrize("seed", range(48))
def test_random_configurations(B, seed):
    """Random small graphs, widths, aggregators, thresholds and chunk sizes through the whole path step by step:
    CSR and split bit-exact, every aggregate to its bar (extrema exactly), chunked == unchunked bitwise."""
    import torch
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.choice([1, 2, 63, 64, 65, 500, 3000, 7000]))
    e = int(rng.choice([0, 1, 5, 100, 4096, 4097, 30000, 70000]))
    dtype = W.F32 if rng.random() < 0.5 else W.BF16
    dim = int(rng.choice([4, 8, 20, 64, 100, 128, 132, 260] if dtype == W.F32 else [8, 16, 40, 64, 128, 200, 256, 264]))
    hub = float(rng.choice([0.0, 0.1, 0.5, 0.95]))
    kind = int(rng.choice([W.AGG_SUM, W.AGG_MEAN, W.AGG_GCN, W.AGG_MAX, W.AGG_MIN]))
    T = [None, 1, 3, 17, 100, 700][int(rng.integers(0, 6))]
    src, dst, x = W.random_small_graph(5000 + seed, n, e, dim, dtype, hub)
    rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
    r, c, d = oracle.build_csr(n, src, dst)
    assert np.array_equal(rowptr.cpu().numpy(), r) and np.array_equal(col.cpu().numpy(), c)
    assert np.array_equal(deg_out.cpu().numpy(), d)
    if T is not None:
        assert_split_equal(B.split_hubs(rowptr, T), oracle.split_hubs(r, T))
    got, want, g = run_gather(B, kind, n, src, dst, x, dtype, T=T)
    what = f"n={n} e={e} dim={dim} {dtype} kind={kind} T={T} hub={hub}"
    if kind in (W.AGG_MAX, W.AGG_MIN):
        assert_same_values(got, want, what)
    else:
        check_features(got, want, dtype, what, sum_terms=sum_scale(g, x) if kind == W.AGG_SUM else None)
    if e > 10:
        chunk = int(rng.integers(1, e))
        chunked, _, _ = run_gather(B, kind, n, src, dst, x, dtype, T=T, chunk=chunk)
        assert np.array_equal(np.asarray(got).view(np.uint8), np.asarray(chunked).view(np.uint8)), what + f" chunk={chunk}"


@pytest.mark.parametrize("seed", range(16))
def test_random_layer_stacks(B, seed):
    """Random stacks of every layer kind (no-gather, mean, GCN, max, min, GAT) and widths through infer_full_graph:
    bitwise equal to the call-by-call loop, chunked or not, and every layer within its bar of the oracle evaluated
    from the state the GPU stored for the previous layer."""
    import torch
    from dataclasses import replace
    from paper_2307_00228_amd import compose
    rng = np.random.default_rng(2000 + seed)
    dtype = W.F32 if seed % 2 == 0 else W.BF16
    n, e = int(rng.choice([300, 2000, 6000])), int(rng.choice([2000, 30000, 60000]))
    hub = float(rng.choice([0.0, 0.3]))
    L = int(rng.integers(1, 5))
    widths = [int(rng.choice([16, 32, 64, 128])) for _ in range(L + 1)]
    kinds = [int(rng.choice([W.AGG_NONE, W.AGG_MEAN, W.AGG_GCN, W.AGG_MAX, W.AGG_MIN, W.AGG_GAT])) for _ in range(L)]
    if kinds[-1] != W.AGG_GAT and seed % 3 == 0:
        widths[-1] = int(rng.choice([3, 10, 47, 100]))      # an output width that is not whole 16-byte pieces
    layers = []
    for i, kind in enumerate(kinds):
        dims = (widths[i], widths[i + 1], widths[i + 1])
        if kind == W.AGG_GAT:
            lay = W.gat_layers(rng, dims, int(rng.choice([1, 2])), dtype, bias_random=True)[0]
        else:
            lay = W.dense_layers(rng, kind, dims, dtype, bias_random=True)[0]
        layers.append(replace(lay, act=W.ACT_RELU if i < L - 1 else W.ACT_NONE))
    src, dst, x = W.random_small_graph(7000 + seed, n, e, widths[0], dtype, hub)
    rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
    r, c, d = oracle.build_csr(n, src, dst)
    T = [None, 9, 200][seed % 3]
    split = B.split_hubs(rowptr, T) if T else None
    dl, xd = B.device_layers(layers), B.to_device(x)
    out = B.infer_full_graph(rowptr, col, deg_out, split, dl, xd)
    view = torch.int16 if dtype == W.BF16 else torch.int32
    chunked = B.infer_full_graph(rowptr, col, deg_out, split, dl, xd, edge_chunk=max(1, e // 3))
    assert torch.equal(out.view(view), chunked.view(view))
    steps = compose.run_layers(rowptr, col, deg_out, split, dl, xd)
    assert torch.equal(out.view(view), steps[-1].out.view(view))
    if any(t.out is None for t in steps):
        # a chained update never stores its layer's state: take the per-layer states from the same model with chaining
        # switched off, which must end in the same bits
        B.set_tuning(9, 0)
        try:
            steps = compose.run_layers(rowptr, col, deg_out, split, dl, xd)
            torch.cuda.synchronize()
        finally:
            B.set_tuning(9, 1)
        assert torch.equal(out.view(view), steps[-1].out.view(view))
    h = x
    for i, (lay, tr) in enumerate(zip(layers, steps)):
        what = f"layer {i} kinds={kinds} widths={widths} T={T}"
        if lay.agg == W.AGG_GAT:
            check_features(B.to_numpy(tr.out), oracle.gat_layer(r, c, h, lay, dtype)[3], dtype, what)
        else:
            check_layer(B, tr, r, c, d, h, lay, dtype, what)
        h = B.to_numpy(tr.out)


def test_layer_events_bracket_the_stages(B):
    """Stage events: four events per layer recorded by infer_full_graph on its stream, in order; the result is
    unchanged and a call without them leaves the events alone (the library keeps no handle after the call)."""
    import torch
    w = W.make("medium_uniform", 0.02)
    rowptr, col, deg_out = B.build_csr_by_dst(w.n_nodes, dev_i32(w.src), dev_i32(w.dst))
    layers, x = B.device_layers(w.layers), B.to_device(w.x)
    ref = B.infer_full_graph(rowptr, col, deg_out, None, layers, x)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(4 * len(layers))]
    for e in evs:
        e.record()
    torch.cuda.synchronize()
    out = B.infer_full_graph(rowptr, col, deg_out, None, layers, x, events=evs)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), ref.view(torch.int32))
    times = [evs[k].elapsed_time(evs[k + 1]) for k in range(len(evs) - 1)]
    assert all(t >= 0.0 for t in times)
    gather = [evs[4 * i + 1].elapsed_time(evs[4 * i + 2]) for i in range(len(layers))]
    assert all(g > 0.0 for g in gather)                      # every layer of this workload has a gather
    again = B.infer_full_graph(rowptr, col, deg_out, None, layers, x)    # recording off: same result, events untouched
    torch.cuda.synchronize()
    assert torch.equal(again.view(torch.int32), ref.view(torch.int32))
    assert [evs[k].elapsed_time(evs[k + 1]) for k in range(len(evs) - 1)] == times


@pytest.mark.parametrize("kind", [W.AGG_MEAN, W.AGG_GCN, W.AGG_MAX, W.AGG_GAT])
def test_infer_degenerate_graphs(B, kind):
    """No edges at all (every vertex keeps its self term; GAT returns the projected row), a single vertex with
    self-loops, and an empty vertex set."""
    import torch
    rng = np.random.default_rng(kind)
    for n, e in [(300, 0), (1, 0), (1, 7), (2, 1)]:
        src, dst, x = W.random_small_graph(n + e, n, e, 32, W.F32, 0.0)
        layers = (W.gat_layers(rng, (32, 32, 16), 2, W.F32, bias_random=True) if kind == W.AGG_GAT
                  else W.dense_layers(rng, kind, (32, 32, 16), W.F32, bias_random=True))
        rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
        r, c, d = oracle.build_csr(n, src, dst)
        out = B.infer_full_graph(rowptr, col, deg_out, B.split_hubs(rowptr, 2), B.device_layers(layers), B.to_device(x))
        check_features(B.to_numpy(out), W.as_f32(oracle.infer_full_graph(r, c, d, x, layers, W.F32)), W.F32, f"n={n} e={e}")
        if e == 0 and kind != W.AGG_GAT:
            # isolated vertices: the aggregate is zero, so only the self term is left (the paper-independent invariant)
            h = W.as_f32(x).astype(np.float64)
            for i, lay in enumerate(layers):
                h = h @ W.as_f32(lay.w_self).astype(np.float64) + lay.bias
                h = np.maximum(h, 0) if i == 0 else h
                h = h.astype(np.float32).astype(np.float64)
            assert np.abs(B.to_numpy(out) - h).max() <= 1e-4
    # empty vertex set: nothing to do, no error
    empty = B.infer_full_graph(torch.zeros(1, dtype=torch.int64, device="cuda"), torch.zeros(0, dtype=torch.int32, device="cuda"),
                               torch.zeros(0, dtype=torch.int32, device="cuda"), None, B.device_layers(layers),
                               torch.zeros((0, 32), dtype=torch.float32, device="cuda"))
    assert empty.shape == (0, 16)


def test_zero_sized_calls_are_accepted(B):
    """Every entry point with an empty vertex or edge set: no launch, no error, outputs of the right (empty) shape."""
    import torch
    z64 = torch.zeros(1, dtype=torch.int64, device="cuda")
    e32 = torch.zeros(0, dtype=torch.int32, device="cuda")
    x0 = torch.zeros((0, 64), dtype=torch.float32, device="cuda")
    rowptr, col, deg_out = B.build_csr_by_dst(0, e32, e32)
    assert rowptr.cpu().tolist() == [0] and col.numel() == 0 and deg_out.numel() == 0
    sp = B.split_hubs(rowptr, 4)
    assert sp.n_hubs == 0 and sp.n_shadows == 0
    for kind in (W.AGG_SUM, W.AGG_MEAN, W.AGG_MAX):
        assert B.gather_layer(kind, z64, e32, x0, sp).shape == (0, 64)
    ss, sd = B.gcn_norm_scales(z64, e32)
    assert ss.numel() == 0 and B.gcn_edge_coefficients(e32, ss).numel() == 0
    assert B.gather_layer(W.AGG_GCN, z64, e32, x0, None, ss, sd).shape == (0, 64)
    wt = torch.zeros((64, 16), dtype=torch.float32, device="cuda")
    assert B.apply_layer(x0, x0, wt, wt, None, W.ACT_RELU).shape == (0, 16)
    assert B.scale_rows(x0, ss).shape == (0, 64)
    # vertices without any edge
    rowptr, col, deg_out = B.build_csr_by_dst(5, e32, e32)
    assert rowptr.cpu().tolist() == [0] * 6 and deg_out.cpu().tolist() == [0] * 5
    x5 = torch.ones((5, 64), dtype=torch.float32, device="cuda")
    assert not B.gather_layer(W.AGG_MEAN, rowptr, col, x5, B.split_hubs(rowptr, 1)).any()
    assert not B.gather_layer(W.AGG_MIN, rowptr, col, x5).any()


def test_edge_feature_layer_chained_into_a_narrowing_layer(B):
    """A 64-wide bf16 layer with an edge matrix (its edge term enters in the gather's epilogue, through the projection
    buffer) whose update is chained into the next layer's projection (which is written to that same buffer afterwards):
    same bits as without the chaining, and every layer within its bar of Eq. (1)."""
    import torch
    from dataclasses import replace
    from paper_2307_00228_amd import compose
    dtype, n, e, d_e = W.BF16, 4000, 60000, 8
    src, dst, x, ef, rng = edge_case(77, n, e, 64, d_e, dtype)
    layers = W.dense_layers(rng, [W.AGG_MEAN, W.AGG_MEAN], (64, 64, 32), dtype, bias_random=True)
    layers[0] = replace(layers[0], w_edge=W.store(rng.uniform(-0.4, 0.4, (d_e, 64)).astype(np.float32), dtype))
    rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
    r, c, d = oracle.build_csr(n, src, dst)
    dl, xd, efd = B.device_layers(layers), B.to_device(x), B.to_device(ef)
    assert B.infer_layer_plan(dl, torch.bfloat16) == [B.PLAN_GATHER_UPDATE_CHAINED, B.PLAN_PROJECT_GATHER]
    split = B.split_hubs(rowptr, 50)
    out = B.infer_full_graph(rowptr, col, deg_out, split, dl, xd, edge_feat=efd, edge_chunk=e // 3)
    tr = compose.run_layers(rowptr, col, deg_out, split, dl, xd, edge_feat=efd)
    assert tr[0].out is None and torch.equal(out.view(torch.int16), tr[-1].out.view(torch.int16))
    B.set_tuning(9, 0)
    try:
        steps = compose.run_layers(rowptr, col, deg_out, split, dl, xd, edge_feat=efd)
        torch.cuda.synchronize()
    finally:
        B.set_tuning(9, 1)
    assert torch.equal(out.view(torch.int16), steps[-1].out.view(torch.int16))
    h = x
    for i, (lay, st) in enumerate(zip(layers, steps)):
        _, y64, a64 = oracle.dense_layer(r, c, d, h, lay, dtype, return_agg64=True, edge_feat=ef if lay.w_edge is not None else None)
        slack = 0.0 if st.projected else agg_rounding_slack(a64, lay.w_nbr, dtype)
        if lay.w_edge is not None:
            et = np.abs(W.as_f32(B.to_numpy(st.edge_term)).astype(np.float64))
            slack = slack + 2.0 ** -8 * (et @ np.abs(W.as_f32(lay.w_nbr).astype(np.float64)))
        check_features(B.to_numpy(st.out), y64, dtype, f"layer {i}", slack=slack)
        h = B.to_numpy(st.out)


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_layers_without_a_self_matrix(B, dtype):
    """h' = act(agg(h) W_nbr + b): dense layers whose self matrix is absent (the vertex's own state does not enter)."""
    import torch
    from dataclasses import replace
    n, e = 4000, 50000
    src, dst, x = W.random_small_graph(61, n, e, 64, dtype, 0.2)
    layers = [replace(l, w_self=None) for l in W.dense_layers(np.random.default_rng(62), [W.AGG_MEAN, W.AGG_MAX], (64, 64, 32), dtype,
                                                              bias_random=True)]
    rowptr, col, deg_out = B.build_csr_by_dst(n, dev_i32(src), dev_i32(dst))
    r, c, d = oracle.build_csr(n, src, dst)
    out = B.infer_full_graph(rowptr, col, deg_out, B.split_hubs(rowptr, 100), B.device_layers(layers), B.to_device(x))
    check_features(B.to_numpy(out), W.as_f32(oracle.infer_full_graph(r, c, d, x, layers, dtype)), dtype)
    iso = np.nonzero(np.diff(r) == 0)[0]
    if len(iso):                                  # no in-edges, no self term: bias only
        assert np.abs(W.as_f32(B.to_numpy(out))[iso] - layers[-1].bias).max() <= (1e-6 if dtype == W.F32 else 2e-3)


def test_very_wide_rows_with_hubs(B):
    """Rows wider than one pass of the combine kernels (more than 1024 16-byte columns of fp32 partials) and than one
    wavefront of lane groups: dense and attention gathers with hub partials."""
    import torch
    n, e, dim = 400, 6000, 4352
    src, dst, x = W.random_small_graph(71, n, e, dim, W.F32, 0.4)
    for kind in (W.AGG_MEAN, W.AGG_MAX):
        got, want, _ = run_gather(B, kind, n, src, dst, x, W.F32, T=16)
        if kind == W.AGG_MAX:
            assert_same_values(got, want)
        else:
            check_features(got, want, W.F32)
    heads = 4
    rng = np.random.default_rng(72)
    s_src = rng.standard_normal((n, heads)).astype(np.float32)
    s_dst = rng.standard_normal((n, heads)).astype(np.float32)
    r, c, _ = oracle.build_csr(n, src, dst)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    out = B.gather_layer(W.AGG_GAT, rp, cl, B.to_device(x), B.split_hubs(rp, 16), torch.from_numpy(s_src).cuda(),
                         torch.from_numpy(s_dst).cuda(), heads=heads, leaky_slope=0.2)
    check_features(B.to_numpy(out), oracle.gat_gather(r, c, x, s_src, s_dst, heads, 0.2), W.F32)


@pytest.mark.parametrize("kind", [W.AGG_MEAN, W.AGG_MAX, W.AGG_GAT])
def test_many_long_rows_wider_than_a_wavefront(B, kind):
    """Rows wider than 64 lanes are covered by several column blocks per row; most rows here lie above the (lowered)
    long-row limit and there is no split: every long row must enter the work list once, whatever the number of column
    blocks (the list holds one entry per vertex)."""
    import torch
    n, e, dim = 1000, 60000, 1040                        # 130 16-byte vectors of bf16: three column blocks
    src, dst, x = W.random_small_graph(91, n, e, dim, W.BF16, 0.0)
    r, c, _ = oracle.build_csr(n, src, dst)
    assert (np.diff(r) > 33).sum() > 0.9 * n
    B.set_tuning(3, 33)
    try:
        if kind == W.AGG_GAT:
            rng = np.random.default_rng(92)
            s_src = rng.standard_normal((n, 2)).astype(np.float32)
            s_dst = rng.standard_normal((n, 2)).astype(np.float32)
            out = B.gather_layer(kind, torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda(), B.to_device(x), None,
                                 torch.from_numpy(s_src).cuda(), torch.from_numpy(s_dst).cuda(), heads=2)
            torch.cuda.synchronize()
            check_features(B.to_numpy(out), oracle.gat_gather(r, c, x, s_src, s_dst, 2, 0.2), W.BF16)
        else:
            got, want, _ = run_gather(B, kind, n, src, dst, x, W.BF16)
            torch.cuda.synchronize()
            if kind == W.AGG_MAX:
                assert_same_values(got, want)
            else:
                check_features(got, want, W.BF16)
    finally:
        B.set_tuning(3, 512)


@pytest.mark.parametrize("kind", [W.AGG_SUM, W.AGG_MEAN, W.AGG_GCN, W.AGG_MAX, W.AGG_GAT])
@pytest.mark.parametrize("dtype,dim", [(W.F32, 64), (W.BF16, 64), (W.BF16, 256), (W.BF16, 520)])
def test_streamed_row_loads_give_the_same_bits(B, kind, dtype, dim):
    """Tables far beyond the caches are read with non-temporal loads and written with non-temporal stores (chosen by
    table size).  Forced on for a small graph with short rows, long rows and hubs, the result is the same bits as
    with plain loads, and within tolerance of the oracle."""
    import torch
    if kind == W.AGG_GAT and dim == 520:
        pytest.skip("520 is not a multiple of heads x 16 bytes")
    n, e = 3000, 70000
    src, dst, x = W.random_small_graph(dim + kind, n, e, dim, dtype, 0.3)
    dst[e // 2:e // 2 + 900] = 7            # a long row below the hub threshold
    r, c, d = oracle.build_csr(n, src, dst)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    split = B.split_hubs(rp, 2000)
    h = B.to_device(x)
    extra = {}
    if kind == W.AGG_GCN:
        ss, sd = B.gcn_norm_scales(rp, torch.from_numpy(d).cuda())
        args = (ss, sd)
    elif kind == W.AGG_GAT:
        rng = np.random.default_rng(dim)
        s_src = rng.standard_normal((n, 4)).astype(np.float32)
        s_dst = rng.standard_normal((n, 4)).astype(np.float32)
        args = (torch.from_numpy(s_src).cuda(), torch.from_numpy(s_dst).cuda())
        extra = dict(heads=4)
    else:
        args = (None, None)
    outs = []
    try:
        for policy in (0, 1):
            B.set_tuning(8, policy)
            outs.append(B.gather_layer(kind, rp, cl, h, split, *args, **extra))
            torch.cuda.synchronize()
    finally:
        B.set_tuning(8, -1)
    assert torch.equal(outs[0].view(torch.uint8), outs[1].view(torch.uint8))
    if kind == W.AGG_GAT:
        want = oracle.gat_gather(r, c, x, s_src, s_dst, 4, 0.2)
        check_features(B.to_numpy(outs[1]), want, dtype)
    elif kind == W.AGG_MAX:
        assert_same_values(B.to_numpy(outs[1]), oracle.gather(kind, r, c, x, deg_out=d))
    else:
        check_features(B.to_numpy(outs[1]), oracle.gather(kind, r, c, x, deg_out=d), dtype,
                       sum_terms=sum_scale((r, c, d), x) if kind == W.AGG_SUM else None)


def test_readme_example_runs(B):
    """The call sequence shown in README.md, executed as written there."""
    import os
    import re
    text = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "README.md")).read()
    code = re.search(r"```python\n(.*?)```", text, flags=re.S).group(1)
    scope = {}
    exec(compile(code, "README.md", "exec"), scope)
    w, out, agg = scope["w"], scope["out"], scope["agg"]
    assert tuple(out.shape) == (w.n_nodes, w.layers[-1].d_out) and tuple(agg.shape) == (w.n_nodes, w.layers[0].d_in)
    r, c, d = oracle.build_csr(w.n_nodes, w.src, w.dst)
    check_features(B.to_numpy(out), W.as_f32(oracle.infer_full_graph(r, c, d, w.x, w.layers, w.dtype)), w.dtype)


def test_shutdown_releases_the_helper_stream_and_later_calls_recreate_it(B):
    """itb_shutdown destroys the library-owned helper stream and its events; it is not terminal: the next call that wants
    the helper stream makes a new one, and the results are the same bits as before."""
    import torch
    n, e = 4000, 60000
    src, dst, x = W.random_small_graph(77, n, e, 64, W.F32, 0.3)
    r, c, d = oracle.build_csr(n, src, dst)
    rp, cl = torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()
    split = B.split_hubs(rp, 500)
    assert split.n_hubs >= 1
    h = B.to_device(x)
    first = B.gather_layer(W.AGG_MEAN, rp, cl, h, split, None, None)      # hubs: uses the helper stream
    torch.cuda.synchronize()
    B.shutdown()
    B.shutdown()                                                          # idempotent
    second = B.gather_layer(W.AGG_MEAN, rp, cl, h, split, None, None)
    src_d, dst_d = dev_i32(src), dev_i32(dst)
    rp2, cl2, deg2 = B.build_csr_by_dst(n, src_d, dst_d)                  # the out-degree branch forks as well
    torch.cuda.synchronize()
    assert torch.equal(first, second)
    assert torch.equal(rp2, rp) and torch.equal(cl2, cl) and np.array_equal(deg2.cpu().numpy(), d)
    check_features(B.to_numpy(second), oracle.gather(W.AGG_MEAN, r, c, x, deg_out=d), W.F32)

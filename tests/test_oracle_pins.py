"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- the definition by brute force on tiny graphs, library
routines for the special cases that reduce to one, closed forms, and the
invariants the paper states (Sec. IV-B: aggregate is commutative/associative;
Sec. IV-D: partial-gather and the even shadow split do not change the result;
Sec. II-A: the k-hop neighbourhood suffices for a k-layer model)."""
import math

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2307_00228_amd import workloads as W


def small_graph(seed, n, e, d, hub=0.0, dtype=W.F32):
    return W.random_small_graph(seed, n, e, d, dtype, hub)


# ---------------------------------------------------------------- brute force (definition, Eq. (1))
def dense_multiplicity(n, src, dst):
    """A[v][u] = number of edges u -> v, straight from the edge list."""
    A = np.zeros((n, n), dtype=np.float64)
    for s, t in zip(src.tolist(), dst.tolist()):
        A[t][s] += 1.0
    return A


def brute_gather(kind, n, src, dst, h):
    A = dense_multiplicity(n, src, dst)
    h = h.astype(np.float64)
    d = h.shape[1]
    out = np.zeros((n, d))
    din = A.sum(axis=1)
    dout = A.sum(axis=0)
    for v in range(n):
        for u in range(n):
            if A[v][u] == 0:
                continue
            c = A[v][u]
            if kind == oracle.GCN:
                c = c / math.sqrt(max(dout[u], 1.0) * max(din[v], 1.0))
            for k in range(d):
                out[v][k] += c * h[u][k]
        if kind == oracle.MEAN and din[v] > 0:
            out[v] /= din[v]
    return out


@pytest.mark.parametrize("seed,n,e", [(0, 1, 0), (1, 1, 5), (2, 7, 0), (3, 12, 40), (4, 33, 300), (5, 64, 1000)])
@pytest.mark.parametrize("kind", [oracle.SUM, oracle.MEAN, oracle.GCN])
def test_gather_matches_brute_force(seed, n, e, kind):
    src, dst, x = small_graph(seed, n, e, 5, hub=0.3)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    got = oracle.gather(kind, rowptr, col, x, deg_out=deg_out)
    want = brute_gather(kind, n, src, dst, x)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- library special cases
@pytest.mark.parametrize("seed,n,e", [(10, 50, 0), (11, 200, 3000), (12, 1000, 20000)])
def test_csr_is_stable_argsort_and_bincount(seed, n, e):
    src, dst, _ = small_graph(seed, n, e, 1, hub=0.2)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    order = np.argsort(dst, kind="stable")
    assert np.array_equal(col, src[order])
    assert np.array_equal(rowptr, np.concatenate([[0], np.cumsum(np.bincount(dst, minlength=n))]))
    assert np.array_equal(deg_out, np.bincount(src, minlength=n))
    assert rowptr[-1] == e and deg_out.sum() == e


def test_csr_rejects_out_of_range():
    with pytest.raises(ValueError):
        oracle.build_csr(3, np.array([0, 3], np.int32), np.array([1, 1], np.int32))
    with pytest.raises(ValueError):
        oracle.build_csr(3, np.array([0, 1], np.int32), np.array([1, -1], np.int32))


@pytest.mark.parametrize("seed", [20, 21])
def test_sum_gather_is_spmm(seed):
    n, e, d = 500, 9000, 16
    src, dst, x = small_graph(seed, n, e, d, hub=0.1)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    A = sp.csr_matrix((np.ones(e), (dst, src)), shape=(n, n))      # duplicates are summed
    want = A @ x.astype(np.float64)
    np.testing.assert_allclose(oracle.gather(oracle.SUM, rowptr, col, x), want, rtol=1e-12, atol=1e-12)
    din = np.asarray(A.sum(axis=1)).ravel()
    dout = np.asarray(A.sum(axis=0)).ravel()
    Dn = sp.diags(1.0 / np.sqrt(np.maximum(din, 1)))
    Do = sp.diags(1.0 / np.sqrt(np.maximum(dout, 1)))
    want_gcn = (Dn @ A @ Do) @ x.astype(np.float64)
    np.testing.assert_allclose(oracle.gather(oracle.GCN, rowptr, col, x, deg_out=deg_out), want_gcn,
                               rtol=1e-12, atol=1e-12)
    want_mean = sp.diags(1.0 / np.maximum(din, 1)) @ want
    np.testing.assert_allclose(oracle.gather(oracle.MEAN, rowptr, col, x), want_mean, rtol=1e-12, atol=1e-12)


def test_apply_is_matmul():
    rng = np.random.default_rng(30)
    n, di, do = 37, 24, 9
    h = rng.standard_normal((n, di)).astype(np.float32)
    a = rng.standard_normal((n, di)).astype(np.float32)
    ws = rng.standard_normal((di, do)).astype(np.float32)
    wn = rng.standard_normal((di, do)).astype(np.float32)
    b = rng.standard_normal(do).astype(np.float32)
    y = h.astype(np.float64) @ ws.astype(np.float64) + a.astype(np.float64) @ wn.astype(np.float64) + b
    np.testing.assert_allclose(oracle.apply(h, a, ws, wn, b, oracle.ACT_NONE), y, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.apply(h, a, ws, wn, b, oracle.ACT_RELU), np.maximum(y, 0), rtol=1e-12, atol=1e-12)
    # operands are not interchangeable: a transposed weight or swapped self/neighbour term must differ
    assert not np.allclose(oracle.apply(a, h, ws, wn, b, oracle.ACT_NONE), y)
    y_nb = a.astype(np.float64) @ wn.astype(np.float64)
    np.testing.assert_allclose(oracle.apply(None, a, None, wn, None, oracle.ACT_NONE), y_nb, rtol=1e-12, atol=1e-12)


def test_apply_non_square_index_order():
    """W is [d_in x d_out] row-major: a one-hot weight routes input k to output c."""
    di, do = 5, 3
    wn = np.zeros((di, do), np.float32)
    wn[4, 1] = 2.0
    a = np.arange(10, dtype=np.float32).reshape(2, di)
    out = oracle.apply(None, a, None, wn, None, oracle.ACT_NONE)
    assert np.array_equal(out, np.array([[0, 8, 0], [0, 18, 0]], dtype=np.float64))


# ---------------------------------------------------------------- closed forms
def test_closed_forms_ones_star_regular():
    # H = 1: sum-agg = in-degree, mean-agg = 1 where deg > 0
    n, e = 40, 300
    src, dst, _ = small_graph(40, n, e, 1)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    ones = np.ones((n, 3), np.float32)
    din = np.diff(rowptr)
    assert np.array_equal(oracle.gather(oracle.SUM, rowptr, col, ones), np.repeat(din[:, None], 3, 1).astype(float))
    m = oracle.gather(oracle.MEAN, rowptr, col, ones)
    assert np.array_equal(m, np.repeat((din > 0)[:, None], 3, 1).astype(float))
    # star: centre 0 receives every leaf; leaves are isolated (in-degree 0)
    L = 9
    src = np.arange(1, L + 1, dtype=np.int32)
    dst = np.zeros(L, np.int32)
    x = np.arange((L + 1) * 2, dtype=np.float32).reshape(L + 1, 2)
    rowptr, col, deg_out = oracle.build_csr(L + 1, src, dst)
    s = oracle.gather(oracle.SUM, rowptr, col, x)
    assert np.array_equal(s[0], x[1:].sum(0).astype(float)) and not s[1:].any()
    # ring (1-regular in and out): GCN == mean == sum == shifted features
    n = 11
    src = np.arange(n, dtype=np.int32)
    dst = ((src + 1) % n).astype(np.int32)
    x = np.random.default_rng(1).standard_normal((n, 4)).astype(np.float32)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    for kind in (oracle.SUM, oracle.MEAN, oracle.GCN):
        np.testing.assert_array_equal(oracle.gather(kind, rowptr, col, x, deg_out=deg_out), np.roll(x, 1, axis=0).astype(float))


def test_regular_graph_gcn_equals_mean():
    # d-regular multigraph: each vertex has in-degree = out-degree = 3 (three shifted rings)
    n, d = 13, 6
    base = np.arange(n, dtype=np.int32)
    src = np.concatenate([base, base, base])
    dst = np.concatenate([(base + 1) % n, (base + 2) % n, (base + 5) % n]).astype(np.int32)
    x = np.random.default_rng(2).standard_normal((n, d)).astype(np.float32)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    np.testing.assert_allclose(oracle.gather(oracle.GCN, rowptr, col, x, deg_out=deg_out),
                               oracle.gather(oracle.MEAN, rowptr, col, x), rtol=1e-14, atol=1e-14)


def test_mean_is_sum_over_degree_and_isolated_keep_self_term():
    n, e, d = 60, 200, 8
    src, dst, x = small_graph(50, n, e, d)
    dst[dst == 7] = 8                                   # vertex 7 has no in-edge
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    din = np.diff(rowptr)
    assert din[7] == 0
    s = oracle.gather(oracle.SUM, rowptr, col, x)
    m = oracle.gather(oracle.MEAN, rowptr, col, x)
    np.testing.assert_allclose(m[din > 0], s[din > 0] / din[din > 0][:, None], rtol=1e-15)
    assert not m[7].any() and not s[7].any()
    rng = np.random.default_rng(3)
    ws = rng.standard_normal((d, 4)).astype(np.float32)
    wn = rng.standard_normal((d, 4)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    y = oracle.apply(x, m.astype(np.float32), ws, wn, b, oracle.ACT_RELU)
    want7 = np.maximum(x[7].astype(np.float64) @ ws.astype(np.float64) + b, 0)
    np.testing.assert_allclose(y[7], want7, rtol=1e-13)
    # identity / zero weights
    eye = np.eye(d, dtype=np.float32)
    zero = np.zeros((d, d), np.float32)
    m32 = m.astype(np.float32)
    np.testing.assert_array_equal(oracle.apply(x, m32, zero, eye, None, oracle.ACT_NONE), m32.astype(float))
    np.testing.assert_array_equal(oracle.apply(x, m32, eye, zero, None, oracle.ACT_RELU), np.maximum(x, 0).astype(float))


# ---------------------------------------------------------------- hub split (Sec. IV-D)
def reference_split(rowptr, T):
    """Even n-way split written out independently with Python integers."""
    hubs, off, beg, end, own = [], [0], [], [], []
    for v in range(len(rowptr) - 1):
        d = int(rowptr[v + 1] - rowptr[v])
        if d > T:
            n = -(-d // T)
            hubs.append(v)
            for g in range(n):
                beg.append(int(rowptr[v]) + (g * d) // n)
                end.append(int(rowptr[v]) + ((g + 1) * d) // n)
                own.append(v)
            off.append(off[-1] + n)
    return hubs, off, beg, end, own


@pytest.mark.parametrize("T", [1, 2, 3, 7, 50, 99, 100, 101, 1000])
def test_split_structure(T):
    n, e = 30, 400
    src, dst, _ = small_graph(60, n, e, 1, hub=0.25)
    dst[:100][dst[:100] != 0] = 1                       # a second row with a known degree range
    rowptr, col, _ = oracle.build_csr(n, src, dst)
    sp_ = oracle.split_hubs(rowptr, T)
    hubs, off, beg, end, own = reference_split(rowptr, T)
    assert sp_["hub_ids"].tolist() == hubs and sp_["hub_shadow_off"].tolist() == off
    assert sp_["shadow_begin"].tolist() == beg and sp_["shadow_end"].tolist() == end
    assert sp_["shadow_owner"].tolist() == own
    din = np.diff(rowptr)
    assert set(hubs) == set(np.nonzero(din > T)[0].tolist())        # "exceeds": strictly greater
    for i, v in enumerate(hubs):
        sizes = (sp_["shadow_end"] - sp_["shadow_begin"])[off[i]:off[i + 1]]
        assert len(sizes) == -(-int(din[v]) // T)
        assert sizes.sum() == din[v] and sizes.max() - sizes.min() <= 1 and sizes.max() <= T
        assert sp_["shadow_begin"][off[i]] == rowptr[v] and sp_["shadow_end"][off[i + 1] - 1] == rowptr[v + 1]
        assert np.array_equal(sp_["shadow_begin"][off[i] + 1:off[i + 1]], sp_["shadow_end"][off[i]:off[i + 1] - 1])


def test_split_threshold_boundary_and_errors():
    # one vertex with in-degree exactly 8
    src = np.arange(1, 9, dtype=np.int32)
    dst = np.zeros(8, np.int32)
    rowptr, _, _ = oracle.build_csr(9, src, dst)
    assert oracle.split_hubs(rowptr, 8)["n_hubs"] == 0          # deg == T is not a hub
    s7 = oracle.split_hubs(rowptr, 7)
    assert s7["n_hubs"] == 1 and s7["n_shadows"] == 2
    assert (s7["shadow_end"] - s7["shadow_begin"]).tolist() == [4, 4]
    s3 = oracle.split_hubs(rowptr, 3)
    assert (s3["shadow_end"] - s3["shadow_begin"]).tolist() == [2, 3, 3]
    with pytest.raises(ValueError):
        oracle.split_hubs(rowptr, 0)


@pytest.mark.parametrize("kind", [oracle.SUM, oracle.MEAN, oracle.GCN])
@pytest.mark.parametrize("T", [1, 2, 3, 5, 64, 10_000])
def test_partial_gather_equals_unsplit(kind, T):
    n, e, d = 80, 2500, 6
    src, dst, x = small_graph(70, n, e, d, hub=0.4)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    whole = oracle.gather(kind, rowptr, col, x, deg_out=deg_out)
    parts, cnt = oracle.gather_split(kind, rowptr, col, x, oracle.split_hubs(rowptr, T), deg_out=deg_out)
    np.testing.assert_allclose(parts, whole, rtol=1e-12, atol=1e-13)
    assert np.array_equal(cnt, np.diff(rowptr))                  # message counts are exact


# ---------------------------------------------------------------- max / min aggregators (Sec. IV-B)
def brute_extremum(kind, n, src, dst, h):
    """Straight from the edge list: the element-wise extremum over the rows of the in-neighbours."""
    h = np.asarray(h, dtype=np.float64)
    out = np.zeros((n, h.shape[1]))
    for v in range(n):
        nb = src[dst == v]
        if len(nb):
            out[v] = h[nb].max(axis=0) if kind == oracle.MAX else h[nb].min(axis=0)
    return out


@pytest.mark.parametrize("seed,n,e", [(0, 1, 0), (1, 1, 5), (2, 7, 0), (3, 12, 40), (4, 33, 300), (5, 64, 1000)])
@pytest.mark.parametrize("kind", [oracle.MAX, oracle.MIN])
def test_extremum_matches_brute_force(seed, n, e, kind):
    src, dst, x = small_graph(seed, n, e, 5, hub=0.3)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    got = oracle.gather(kind, rowptr, col, x)
    assert np.array_equal(got, brute_extremum(kind, n, src, dst, x))     # exact: the result is one of the inputs
    assert not got[np.diff(rowptr) == 0].any()                           # isolated vertex -> 0


def test_extremum_invariants():
    n, e, d = 70, 900, 5
    src, dst, x = small_graph(83, n, e, d, hub=0.2)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    mx, mn = oracle.gather(oracle.MAX, rowptr, col, x), oracle.gather(oracle.MIN, rowptr, col, x)
    mean = oracle.gather(oracle.MEAN, rowptr, col, x)
    has = np.diff(rowptr) > 0
    assert (mx[has] >= mean[has] - 1e-12).all() and (mean[has] >= mn[has] - 1e-12).all()
    assert (mx[has] > mn[has]).any()
    assert np.array_equal(oracle.gather(oracle.MIN, rowptr, col, -x), -mx)   # min(x) = -max(-x)
    # a monotone map commutes with the extremum; doubling every edge changes nothing (idempotent)
    y = (np.float32(3.0) * x + np.float32(1.0)).astype(np.float32)
    assert np.array_equal(oracle.gather(oracle.MAX, rowptr, col, y),
                          np.where(has[:, None], (np.float32(3.0) * mx.astype(np.float32) + np.float32(1.0)).astype(np.float64), 0.0))
    r2, c2, _ = oracle.build_csr(n, np.concatenate([src, src]), np.concatenate([dst, dst]))
    assert np.array_equal(oracle.gather(oracle.MAX, r2, c2, x), mx)
    # a single in-edge returns the source row; the order of the edges does not matter
    one = np.nonzero(np.diff(rowptr) == 1)[0]
    if len(one):
        assert np.array_equal(mx[one], x[col[rowptr[one]]].astype(np.float64))
        assert np.array_equal(mn[one], mx[one])
    p = np.random.default_rng(84).permutation(e)
    r3, c3, _ = oracle.build_csr(n, src[p], dst[p])
    assert np.array_equal(oracle.gather(oracle.MIN, r3, c3, x), mn)
    verts = np.array([0, 5, 69, 17, 5], dtype=np.int64)
    assert np.array_equal(oracle.gather(oracle.MAX, rowptr, col, x, verts=verts), mx[verts])


@pytest.mark.parametrize("kind", [oracle.MAX, oracle.MIN])
@pytest.mark.parametrize("T", [1, 2, 3, 5, 64, 10_000])
def test_partial_extremum_equals_unsplit(kind, T):
    n, e, d = 80, 2500, 6
    src, dst, x = small_graph(71, n, e, d, hub=0.4)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    whole = oracle.gather(kind, rowptr, col, x)
    parts, cnt = oracle.gather_split(kind, rowptr, col, x, oracle.split_hubs(rowptr, T))
    assert np.array_equal(parts, whole)
    assert np.array_equal(cnt, np.diff(rowptr))
    assert np.array_equal(whole, brute_extremum(kind, n, src, dst, x))


def test_layer_without_gather_and_extremum_layers_against_numpy():
    """Encoder -> max-pool layer -> min-pool layer -> prediction head, recomputed with numpy from the stored states."""
    n, e = 60, 700
    src, dst, x = small_graph(150, n, e, 12)
    rng = np.random.default_rng(151)
    layers = W.dense_layers(rng, [W.AGG_NONE, W.AGG_MAX, W.AGG_MIN, W.AGG_NONE], (12, 8, 8, 8, 3), W.F32, bias_random=True)
    assert layers[0].w_self is None and layers[3].w_self is None and layers[1].w_self is not None
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    outs = oracle.infer_full_graph(rowptr, col, deg_out, x, layers, W.F32, return_all=True)
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    h = f64(x)
    for i, lay in enumerate(layers):
        if lay.agg == W.AGG_NONE:
            y = h @ f64(lay.w_nbr) + lay.bias
        else:
            agg = brute_extremum(oracle.MAX if lay.agg == W.AGG_MAX else oracle.MIN, n, src, dst, h)
            y = h @ f64(lay.w_self) + agg @ f64(lay.w_nbr) + lay.bias
        if i < len(layers) - 1:
            y = np.maximum(y, 0.0)
        np.testing.assert_allclose(f64(outs[i]), y, rtol=1e-6, atol=1e-6)
        h = f64(outs[i])                                         # next layer reads the stored (rounded) state
    assert outs[-1].shape == (n, 3)


# ---------------------------------------------------------------- algebraic invariants
def test_linearity_and_edge_permutation_and_relabelling():
    n, e, d = 70, 900, 5
    src, dst, x1 = small_graph(80, n, e, d, hub=0.2)
    x2 = np.random.default_rng(81).standard_normal((n, d)).astype(np.float32)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    rng = np.random.default_rng(82)
    for kind in (oracle.SUM, oracle.MEAN, oracle.GCN):
        g1 = oracle.gather(kind, rowptr, col, x1, deg_out=deg_out)
        g2 = oracle.gather(kind, rowptr, col, x2, deg_out=deg_out)
        mix = (np.float32(2.0) * x1 + np.float32(-0.5) * x2)
        np.testing.assert_allclose(oracle.gather(kind, rowptr, col, mix, deg_out=deg_out),
                                   2.0 * g1 - 0.5 * g2, rtol=1e-5, atol=1e-5)
        # shuffling the edge list only reorders sources inside a row
        p = rng.permutation(e)
        r2, c2, do2 = oracle.build_csr(n, src[p], dst[p])
        assert np.array_equal(r2, rowptr) and np.array_equal(do2, deg_out)
        np.testing.assert_allclose(oracle.gather(kind, r2, c2, x1, deg_out=do2), g1, rtol=1e-12, atol=1e-12)
        # relabelling vertices permutes the output rows
        pi = rng.permutation(n).astype(np.int32)
        r3, c3, do3 = oracle.build_csr(n, pi[src], pi[dst])
        xp = np.zeros_like(x1)
        xp[pi] = x1
        g3 = oracle.gather(kind, r3, c3, xp, deg_out=do3)
        np.testing.assert_allclose(g3[pi], g1, rtol=1e-12, atol=1e-12)


def test_vertex_subset_matches_full():
    n, e, d = 90, 1500, 4
    src, dst, x = small_graph(90, n, e, d, hub=0.3)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    verts = np.array([0, 5, 89, 17, 5], dtype=np.int64)
    for kind in (oracle.SUM, oracle.MEAN, oracle.GCN):
        full = oracle.gather(kind, rowptr, col, x, deg_out=deg_out)
        np.testing.assert_array_equal(oracle.gather(kind, rowptr, col, x, deg_out=deg_out, verts=verts), full[verts])


# ---------------------------------------------------------------- k-hop sufficiency (Sec. II-A)
def khop_value(v, k, in_nbrs, dout, x, layers):
    """Evaluate layer k at vertex v recursively from its k-hop in-neighbourhood only."""
    if k == 0:
        return x[v].astype(np.float64)
    lay = layers[k - 1]
    hv = khop_value(v, k - 1, in_nbrs, dout, x, layers)
    acc = np.zeros_like(hv)
    for u in in_nbrs[v]:
        hu = khop_value(u, k - 1, in_nbrs, dout, x, layers)
        c = 1.0
        if lay.agg == W.AGG_GCN:
            c = 1.0 / math.sqrt(max(dout[u], 1) * max(len(in_nbrs[v]), 1))
        acc += c * hu
    if lay.agg == W.AGG_MEAN and in_nbrs[v]:
        acc /= len(in_nbrs[v])
    y = hv @ lay.w_self.astype(np.float64) + acc @ lay.w_nbr.astype(np.float64) + lay.bias
    return np.maximum(y, 0) if lay.act == W.ACT_RELU else y


@pytest.mark.parametrize("agg", [W.AGG_MEAN, W.AGG_GCN, W.AGG_SUM])
def test_khop_recursion_equals_layerwise(agg):
    n, e, d = 25, 60, 6
    src, dst, x = small_graph(100, n, e, d)
    rng = np.random.default_rng(101)
    layers = W.dense_layers(rng, agg, (d, 7, 3), W.F32, bias_random=True)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    out = oracle.infer_full_graph(rowptr, col, deg_out, x, layers, W.F32)
    in_nbrs = [[] for _ in range(n)]
    for s, t in zip(src.tolist(), dst.tolist()):
        in_nbrs[t].append(s)
    dout = np.bincount(src, minlength=n)
    for v in (0, 3, 11, 24):
        want = khop_value(v, 2, in_nbrs, dout, x, layers)
        # layer-wise path rounds h^1 to fp32 storage once; the recursion does not
        np.testing.assert_allclose(out[v], want, rtol=2e-6, atol=2e-6)


# ---------------------------------------------------------------- storage rounding
def test_bf16_rounding_matches_torch_and_ties_to_even():
    import torch
    rng = np.random.default_rng(110)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000),
                        [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 257.0, 259.0, 3.0e38 * 0 + 65280.0]])
    x32 = x.astype(np.float32).astype(np.float64)               # fp32-representable => single rounding in torch
    got = oracle.round_store(x32, "bf16")
    want = torch.from_numpy(x32.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa wins (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert W.bf16_bits_to_f32(oracle.round_store(np.array([1.00390625, 1.01171875]), "bf16")).tolist() == [1.0, 1.015625]
    # generator-side rounding agrees too
    assert np.array_equal(W.f32_to_bf16_bits(x32.astype(np.float32)), want)


# ---------------------------------------------------------------- GAT (Sec. II-B, Sec. IV-B)
def brute_gat(n, src, dst, z, s_src, s_dst, heads, slope):
    z = z.astype(np.float64)
    dh = z.shape[1] // heads
    out = np.zeros_like(z)
    nb = [[v] for v in range(n)]                                  # implicit self edge
    for s, t in zip(src.tolist(), dst.tolist()):
        nb[t].append(s)
    for v in range(n):
        for k in range(heads):
            e = np.array([float(s_src[u, k]) + float(s_dst[v, k]) for u in nb[v]])
            e = np.where(e > 0, e, slope * e)
            a = np.exp(e - e.max())
            a /= a.sum()
            for w_, u in zip(a, nb[v]):
                out[v, k * dh:(k + 1) * dh] += w_ * z[u, k * dh:(k + 1) * dh]
    return out


def test_gat_gather_brute_force_and_invariants():
    n, e, heads, dh = 30, 200, 3, 4
    src, dst, z = small_graph(120, n, e, heads * dh, hub=0.3)
    dst[dst == 9] = 10                                            # vertex 9 isolated
    rng = np.random.default_rng(121)
    s_src = rng.standard_normal((n, heads)).astype(np.float32) * 3
    s_dst = rng.standard_normal((n, heads)).astype(np.float32) * 3
    rowptr, col, _ = oracle.build_csr(n, src, dst)
    got = oracle.gat_gather(rowptr, col, z, s_src, s_dst, heads, 0.2)
    np.testing.assert_allclose(got, brute_gat(n, src, dst, z, s_src, s_dst, heads, 0.2), rtol=1e-12, atol=1e-12)
    # isolated vertex attends only to itself
    np.testing.assert_allclose(got[9], z[9].astype(np.float64), rtol=1e-15)
    # zero attention vectors: uniform attention = mean over in(v) + {v}
    zero = np.zeros((n, heads), np.float32)
    uni = oracle.gat_gather(rowptr, col, z, zero, zero, heads, 0.2)
    s = oracle.gather(oracle.SUM, rowptr, col, z) + z.astype(np.float64)
    np.testing.assert_allclose(uni, s / (np.diff(rowptr) + 1)[:, None], rtol=1e-12, atol=1e-13)
    # all z rows equal: any convex combination returns that row
    zc = np.tile(z[:1], (n, 1))
    np.testing.assert_allclose(oracle.gat_gather(rowptr, col, zc, s_src, s_dst, heads, 0.2),
                               zc.astype(np.float64), rtol=1e-12, atol=1e-13)
    # slope 1 makes LeakyReLU the identity: a per-destination shift of scores cancels in the softmax
    a1 = oracle.gat_gather(rowptr, col, z, s_src, s_dst, heads, 1.0)
    a2 = oracle.gat_gather(rowptr, col, z, s_src, s_dst + np.float32(1.5), heads, 1.0)
    np.testing.assert_allclose(a1, a2, rtol=1e-6, atol=1e-6)
    # subset evaluation
    verts = np.array([9, 0, 29], np.int64)
    np.testing.assert_array_equal(oracle.gat_gather(rowptr, col, z, s_src, s_dst, heads, 0.2, verts=verts), got[verts])


def test_gat_scores_and_layer_against_numpy():
    n, e, heads, dh, di = 20, 90, 2, 3, 5
    src, dst, x = small_graph(130, n, e, di)
    rng = np.random.default_rng(131)
    lay = W.gat_layers(rng, (di, heads * dh), heads, W.F32, bias_random=True)[0]
    lay.act = W.ACT_RELU
    rowptr, col, _ = oracle.build_csr(n, src, dst)
    z_st, s_src, s_dst, y = oracle.gat_layer(rowptr, col, x, lay, W.F32)
    z64 = x.astype(np.float64) @ lay.w_nbr.astype(np.float64)
    np.testing.assert_allclose(z_st, z64, rtol=1e-6, atol=1e-6)
    want_src = np.einsum("nkd,kd->nk", z64.reshape(n, heads, dh), lay.att_src.astype(np.float64))
    want_dst = np.einsum("nkd,kd->nk", z64.reshape(n, heads, dh), lay.att_dst.astype(np.float64))
    np.testing.assert_allclose(s_src, want_src, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(s_dst, want_dst, rtol=1e-6, atol=1e-6)
    want = brute_gat(n, src, dst, z_st, s_src, s_dst, heads, 0.2) + lay.bias
    np.testing.assert_allclose(y, np.maximum(want, 0), rtol=1e-12, atol=1e-12)


def test_infer_rounds_between_layers_and_uses_relu_only_between():
    n, e, d = 40, 300, 8
    src, dst, x = small_graph(140, n, e, d, dtype=W.BF16)
    rng = np.random.default_rng(141)
    layers = W.dense_layers(rng, W.AGG_MEAN, (d, 8, 4), W.BF16, bias_random=True)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    outs = oracle.infer_full_graph(rowptr, col, deg_out, x, layers, W.BF16, return_all=True)
    assert outs[0].dtype == np.uint16 and outs[1].dtype == np.uint16
    h1 = W.bf16_bits_to_f32(outs[0])
    assert (h1 >= 0).all()                                        # ReLU after the first layer
    assert (W.bf16_bits_to_f32(outs[1]) < 0).any()                # identity after the last
    # second layer recomputed by numpy from the stored h1
    xf = h1.astype(np.float64)
    A = sp.csr_matrix((np.ones(e), (dst, src)), shape=(n, n))
    # (the aggregate itself is not rounded: a layer is Eq. (1), only its output is a stored tensor)
    agg = sp.diags(1.0 / np.maximum(np.diff(rowptr), 1)) @ (A @ xf)
    y = xf @ W.as_f32(layers[1].w_self).astype(np.float64) + agg @ W.as_f32(layers[1].w_nbr).astype(np.float64) + layers[1].bias
    got = W.bf16_bits_to_f32(outs[1]).astype(np.float64)
    # equal up to the summation order of the two fp64 evaluations: after rounding to bf16 at most a tie may flip
    assert np.abs(got - W.bf16_bits_to_f32(oracle.round_store(y, "bf16"))).max() <= 2.0 ** -8 * np.abs(y).max()
    assert (oracle.round_store(y, "bf16") == outs[1]).mean() > 0.99


def test_dense_layer_without_intermediate_rounding_is_plain_matmul():
    """The default: Eq. (1) in fp64, no stored aggregate; equals act(h W_self + (A h) W_nbr + b) by scipy/numpy, and
    differs from the rounded-aggregate form (round_agg=True) exactly by (agg - round(agg)) W_nbr."""
    n, e, d = 50, 600, 16
    src, dst, x = small_graph(160, n, e, d, hub=0.4, dtype=W.BF16)
    lay = W.dense_layers(np.random.default_rng(161), W.AGG_SUM, (d, 8, 8), W.BF16, bias_random=True)[0]
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    xf = W.as_f32(x).astype(np.float64)
    A = sp.csr_matrix((np.ones(e), (dst, src)), shape=(n, n))
    ws, wn = W.as_f32(lay.w_self).astype(np.float64), W.as_f32(lay.w_nbr).astype(np.float64)
    want = np.maximum(xf @ ws + (A @ xf) @ wn + lay.bias, 0.0)
    a_st, got, a64 = oracle.dense_layer(rowptr, col, deg_out, x, lay, W.BF16, return_agg64=True)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(a64, A @ xf, rtol=1e-12, atol=1e-12)
    _, rounded = oracle.dense_layer(rowptr, col, deg_out, x, lay, W.BF16, round_agg=True)
    want_r = np.maximum(xf @ ws + W.as_f32(a_st).astype(np.float64) @ wn + lay.bias, 0.0)
    np.testing.assert_allclose(rounded, want_r, rtol=1e-12, atol=1e-12)
    assert np.abs(rounded - got).max() > 0                       # the hub's aggregate does not fit bf16 exactly


# ---------------------------------------------------------------- threshold heuristic (Sec. IV-D / Sec. V)
def test_hub_threshold_golden_and_exact_rational():
    import os
    from fractions import Fraction
    path = os.path.join(os.path.dirname(__file__), "golden", "hub_threshold_heuristic.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert rows
    for e, w, num, den, want in rows:
        assert oracle.hub_threshold(int(e), int(w), (int(num), int(den))) == int(want)
    rng = np.random.default_rng(170)
    for _ in range(200):
        e, w = int(rng.integers(0, 1 << 40)), int(rng.integers(1, 5000))
        num, den = int(rng.integers(1, 50)), int(rng.integers(1, 1000))
        t = oracle.hub_threshold(e, w, (num, den))
        exact = Fraction(num * e, den * w)
        assert t == max(1, exact.numerator // exact.denominator)
        # "exceeds the real threshold" and "exceeds its floor" are the same statement about integer degrees
        if t > 1:
            assert (t + 1 > exact) and not (t > exact)
    with pytest.raises(ValueError):
        oracle.hub_threshold(10, 0)


# ---------------------------------------------------------------- edge-weighted messages (Sec. IV-B apply_edge)
def test_weighted_gather_is_weighted_spmm_and_reduces_to_the_plain_forms():
    n, e, d = 60, 900, 5
    src, dst, x = small_graph(180, n, e, d, hub=0.3)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    order = np.argsort(dst, kind="stable")                     # CSR position -> original edge
    w_edge = np.random.default_rng(181).standard_normal(e).astype(np.float32)   # per original edge
    w_csr = w_edge[order]
    A = sp.csr_matrix((w_edge.astype(np.float64), (dst, src)), shape=(n, n))      # duplicates are summed
    want = A @ x.astype(np.float64)
    got = oracle.gather_weighted(oracle.SUM, rowptr, col, x, w_csr)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    deg = np.diff(rowptr)
    mean = oracle.gather_weighted(oracle.MEAN, rowptr, col, x, w_csr)
    np.testing.assert_allclose(mean[deg > 0], want[deg > 0] / deg[deg > 0, None], rtol=1e-12, atol=1e-12)
    assert not mean[deg == 0].any()
    ones = np.ones(e, dtype=np.float32)
    assert np.array_equal(oracle.gather_weighted(oracle.SUM, rowptr, col, x, ones), oracle.gather(oracle.SUM, rowptr, col, x))
    assert np.array_equal(oracle.gather_weighted(oracle.MEAN, rowptr, col, x, ones), oracle.gather(oracle.MEAN, rowptr, col, x))
    # the GCN aggregate is the weighted sum with w_e = (deg_out(u) deg_in(v))^-1/2
    dv = np.repeat(np.maximum(deg, 1), deg)
    w_gcn = (1.0 / np.sqrt(np.maximum(deg_out[col], 1).astype(np.float64) * dv)).astype(np.float32)
    np.testing.assert_allclose(oracle.gather_weighted(oracle.SUM, rowptr, col, x, w_gcn),
                               oracle.gather(oracle.GCN, rowptr, col, x, deg_out=deg_out), rtol=1e-5, atol=1e-6)
    verts = np.array([3, 0, 59, 3], dtype=np.int64)
    assert np.array_equal(oracle.gather_weighted(oracle.SUM, rowptr, col, x, w_csr, verts=verts), got[verts])
    with pytest.raises(ValueError):
        oracle.gather_weighted(oracle.MAX, rowptr, col, x, w_csr)


# ---------------------------------------------------------------- messages with edge feature vectors (Sec. II-A E, Sec. II-B M)
def edge_feature_case(seed, n, e, d, d_e, hub=0.3):
    """Graph, states, per-edge features in ORIGINAL edge order and in CSR order, edge matrix."""
    src, dst, x = small_graph(seed, n, e, d, hub=hub)
    rng = np.random.default_rng(seed + 500)
    ef_orig = rng.standard_normal((e, d_e)).astype(np.float32)
    w_e = rng.uniform(-0.5, 0.5, (d_e, d)).astype(np.float32)
    rowptr, col, deg_out = oracle.build_csr(n, src, dst)
    order = np.argsort(dst, kind="stable")                # CSR slot -> original edge (the stable grouping, pinned above)
    return src, dst, x, ef_orig, ef_orig[order], w_e, rowptr, col, deg_out


@pytest.mark.parametrize("seed,n,e", [(0, 1, 0), (1, 1, 4), (2, 9, 0), (3, 12, 50), (4, 40, 400)])
@pytest.mark.parametrize("kind", [oracle.SUM, oracle.MEAN, oracle.GCN])
def test_edge_feature_gather_matches_brute_force(seed, n, e, kind):
    """Definition, edge by edge over the ORIGINAL edge list: m_e = h[src] + ef[e] W_e goes to dst (checks the CSR-slot
    indexing of the feature array as well as the arithmetic)."""
    d, d_e = 5, 3
    src, dst, x, ef_orig, ef_csr, w_e, rowptr, col, deg_out = edge_feature_case(seed, n, e, d, d_e)
    got = oracle.gather_edge_features(kind, rowptr, col, x, ef_csr, w_e, deg_out=deg_out)
    want = np.zeros((n, d))
    din = np.bincount(dst, minlength=n).astype(np.float64)
    dout = np.bincount(src, minlength=n).astype(np.float64)
    for k in range(e):
        u, v = int(src[k]), int(dst[k])
        m = x[u].astype(np.float64).copy()
        for t in range(d_e):
            for j in range(d):
                m[j] += float(ef_orig[k][t]) * float(w_e[t][j])
        c = 1.0 / math.sqrt(max(dout[u], 1.0) * max(din[v], 1.0)) if kind == oracle.GCN else 1.0
        want[v] += c * m
    if kind == oracle.MEAN:
        want /= np.maximum(din, 1.0)[:, None]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("kind", [oracle.SUM, oracle.MEAN, oracle.GCN])
def test_edge_feature_gather_special_cases_and_factorisation(kind):
    n, e, d, d_e = 60, 900, 7, 4
    src, dst, x, ef_orig, ef_csr, w_e, rowptr, col, deg_out = edge_feature_case(77, n, e, d, d_e, hub=0.4)
    plain = oracle.gather(kind, rowptr, col, x, deg_out=deg_out)
    full = oracle.gather_edge_features(kind, rowptr, col, x, ef_csr, w_e, deg_out=deg_out)
    # a zero edge matrix leaves the plain aggregate
    np.testing.assert_allclose(oracle.gather_edge_features(kind, rowptr, col, x, ef_csr, np.zeros_like(w_e), deg_out=deg_out),
                               plain, rtol=1e-13, atol=1e-13)
    # zero states leave the reduced edge features times W_e: a sparse matrix over (destination, edge) by scipy
    coef = np.ones(e)
    if kind == oracle.GCN:
        din, dout = np.bincount(dst, minlength=n), np.bincount(src, minlength=n)
        coef = 1.0 / np.sqrt(np.maximum(dout[src], 1) * np.maximum(din[dst], 1))
    if kind == oracle.MEAN:
        coef = 1.0 / np.maximum(np.bincount(dst, minlength=n), 1)[dst]
    S = sp.csr_matrix((coef, (dst, np.arange(e))), shape=(n, e)) @ ef_orig.astype(np.float64)
    only_edges = oracle.gather_edge_features(kind, rowptr, col, np.zeros_like(x), ef_csr, w_e, deg_out=deg_out)
    np.testing.assert_allclose(only_edges, S @ w_e.astype(np.float64), rtol=1e-12, atol=1e-12)
    # the reduce is linear in the message, so the whole is the sum of the two parts
    np.testing.assert_allclose(full, plain + S @ w_e.astype(np.float64), rtol=1e-12, atol=1e-12)
    # sampled vertices agree with the full evaluation; isolated vertices aggregate to zero
    verts = np.array([0, 3, 59, 17], dtype=np.int64)
    np.testing.assert_allclose(oracle.gather_edge_features(kind, rowptr, col, x, ef_csr, w_e, deg_out=deg_out, verts=verts),
                               full[verts], rtol=0, atol=0)
    iso = np.nonzero(np.diff(rowptr) == 0)[0]
    assert not full[iso].any()


def test_dense_layer_with_edge_features_is_eq1_with_those_messages():
    from dataclasses import replace
    n, e, d, d_e = 30, 300, 8, 4
    src, dst, x, ef_orig, ef_csr, w_e, rowptr, col, deg_out = edge_feature_case(91, n, e, d, d_e)
    lay = replace(W.dense_layers(np.random.default_rng(92), W.AGG_MEAN, (d, 6, 6), W.F32, bias_random=True)[0], w_edge=w_e)
    _, y = oracle.dense_layer(rowptr, col, deg_out, x, lay, W.F32, edge_feat=ef_csr)
    agg = oracle.gather_edge_features(oracle.MEAN, rowptr, col, x, ef_csr, w_e)
    want = np.maximum(x.astype(np.float64) @ lay.w_self.astype(np.float64) + agg @ lay.w_nbr.astype(np.float64) + lay.bias, 0.0)
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
    out = oracle.infer_full_graph(rowptr, col, deg_out, x, [lay], W.F32, edge_feat=ef_csr)
    np.testing.assert_array_equal(out, want.astype(np.float32))

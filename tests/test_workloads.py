"""The seeded input generators: reproducible, exact sizes, and the structure the workloads are named for (they stand in
for the paper's power-law graphs; no dataset is reconstructed)."""
import numpy as np
import pytest

from paper_2307_00228_amd import workloads as W


@pytest.mark.parametrize("name,scale", [("tiny_powerlaw", 1.0), ("medium_uniform", 0.01), ("hub_heavy", 0.005),
                                        ("hub_heavy_uniform_control", 0.005), ("attention", 0.01), ("huge_share", 0.0002)])
def test_generators_are_seeded_and_sized(name, scale):
    a, b, c = W.make(name, scale), W.make(name, scale), W.make(name, scale, seed=1)
    assert np.array_equal(a.src, b.src) and np.array_equal(a.dst, b.dst) and np.array_equal(a.x, b.x)
    assert all(np.array_equal(p.w_nbr, q.w_nbr) for p, q in zip(a.layers, b.layers))
    assert not np.array_equal(a.dst, c.dst)                      # another seed, another graph
    assert a.src.dtype == np.int32 and a.dst.dtype == np.int32 and len(a.src) == len(a.dst) == a.n_edges
    assert 0 <= a.src.min() and a.src.max() < a.n_nodes and 0 <= a.dst.min() and a.dst.max() < a.n_nodes
    assert a.x.shape == (a.n_nodes, a.layers[0].d_in)
    assert a.x.dtype == (np.uint16 if a.dtype == W.BF16 else np.float32)
    for l0, l1 in zip(a.layers, a.layers[1:]):
        assert l0.d_out == l1.d_in and l0.act == W.ACT_RELU
    assert a.layers[-1].act == W.ACT_NONE
    for l in a.layers:
        lim = np.sqrt(6.0 / (l.d_in + l.d_out))                  # Glorot-uniform bound
        assert np.abs(W.as_f32(l.w_nbr)).max() <= lim * 1.01 and not l.bias.any()


def test_full_size_parameters_follow_the_baseline_configs():
    """Sizes, widths, dtypes and thresholds at scale 1 (read off the factory without generating the big graphs)."""
    t = W.make("tiny_powerlaw")
    assert (t.n_nodes, t.n_edges, t.dtype, t.threshold) == (10_000, 100_000, W.F32, W.NO_SPLIT)
    assert [(l.d_in, l.d_out, l.agg) for l in t.layers] == [(64, 64, W.AGG_MEAN), (64, 16, W.AGG_MEAN)]
    m = W.make("medium_uniform", 0.001)
    assert [(l.d_in, l.d_out, l.agg) for l in m.layers] == [(128, 128, W.AGG_GCN), (128, 64, W.AGG_GCN)] and m.dtype == W.F32
    h = W.make("hub_heavy", 0.001)
    assert [(l.d_in, l.d_out, l.agg) for l in h.layers] == [(128, 128, W.AGG_MEAN)] * 2 and h.dtype == W.BF16
    a = W.make("attention", 0.001)
    assert [(l.d_in, l.d_out, l.agg, l.heads) for l in a.layers] == [(256, 256, W.AGG_GAT, 4)] * 3 and a.dtype == W.BF16
    g = W.make("huge_share", 0.0001)
    assert [(l.d_in, l.d_out) for l in g.layers] == [(64, 64), (64, 32)] and g.dtype == W.BF16


def test_structure_of_the_skewed_workloads():
    # tiny_powerlaw: rank-Zipf(1.2): the top destination holds about a fifth of the edges
    t = W.make("tiny_powerlaw")
    top = np.bincount(t.dst, minlength=t.n_nodes).max() / t.n_edges
    assert 0.15 < top < 0.30
    # hub_heavy: 16 planted hubs with in-degrees linspace(1e6, 4e6) * scale hold 5/8 of the edges; the rest is a tail
    s = 0.005
    h = W.make("hub_heavy", s)
    deg = np.sort(np.bincount(h.dst, minlength=h.n_nodes))[::-1]
    want = np.floor(np.linspace(1_000_000, 4_000_000, 16) * s)[::-1]
    assert np.array_equal(deg[:16], want)
    assert deg[16] < want.min() and abs(deg[:16].sum() / h.n_edges - 0.625) < 0.01
    assert (deg > h.threshold).sum() >= 16
    # its control has the same sizes and no hub
    u = W.make("hub_heavy_uniform_control", s)
    assert (u.n_nodes, u.n_edges, u.dtype) == (h.n_nodes, h.n_edges, h.dtype)
    assert np.bincount(u.dst, minlength=u.n_nodes).max() < 60
    # attention: rank-Zipf(1.5): the top destination holds well over a third of the edges, most vertices none
    a = W.make("attention", 0.01)
    da = np.bincount(a.dst, minlength=a.n_nodes)
    assert da.max() / a.n_edges > 0.3 and (da == 0).mean() > 0.6
    # the edge list is not sorted by destination
    assert (np.diff(h.dst.astype(np.int64)) < 0).mean() > 0.3


def test_bf16_storage_helpers_round_trip():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(1000).astype(np.float32)
    bits = W.f32_to_bf16_bits(x)
    assert bits.dtype == np.uint16
    back = W.bf16_bits_to_f32(bits)
    assert np.abs(back - x).max() <= np.abs(x).max() * 2.0 ** -8
    assert np.array_equal(W.f32_to_bf16_bits(back), bits)        # bf16 values are fixed points of the rounding
    assert np.array_equal(W.store(back, W.BF16), bits) and W.store(x, W.F32).dtype == np.float32

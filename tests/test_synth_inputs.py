"""The synthetic inputs have the structure the recipe promises (CPU only)."""
import numpy as np
import torch

from paper_2110_08450_amd import synth


def _check_simple_symmetric(g):
    indptr, indices = g.indptr.numpy(), g.indices.numpy()
    n = g.num_nodes
    assert indptr[0] == 0 and indptr[-1] == len(indices) and (np.diff(indptr) >= 0).all()
    assert indices.min() >= 0 and indices.max() < n
    src = np.repeat(np.arange(n), np.diff(indptr))
    assert (src != indices).all()                                   # no self loops
    key = src.astype(np.int64) * n + indices
    assert (np.diff(key) > 0).all()                                 # rows sorted, no duplicate edges
    rev = indices.astype(np.int64) * n + src
    assert np.array_equal(np.sort(rev), key)                        # symmetric


def test_tiny_and_mid_graphs_are_simple_symmetric_power_law():
    for name in ("tiny", "mid"):
        w = synth.WORKLOADS[name]
        g = synth.make_graph(w)
        _check_simple_symmetric(g)
        deg = np.diff(g.indptr.numpy())
        assert abs(g.num_edges - w.num_directed_edges) < 0.02 * w.num_directed_edges
        assert 0.5 * w.max_degree < deg.max() < 1.5 * w.max_degree
        # heavy tail: the top 1 % of the nodes hold far more than 1 % of the edge endpoints
        top = np.sort(deg)[-max(1, len(deg) // 100):].sum()
        assert top > 0.08 * deg.sum()
        # tail exponent of the degree distribution near 2.5: P(deg >= 4x) / P(deg >= x) ~ 4^-(gamma-1)
        x = 2 * deg.mean()
        ratio = (deg >= 4 * x).sum() / max(1, (deg >= x).sum())
        assert 4.0 ** -2.2 < ratio < 4.0 ** -0.9, ratio


def test_citation_style_recipe_is_symmetric_too():
    g = synth.powerlaw_graph(20_000, 400_000, 2_000.0, seed=5, gamma_src=3.5)
    _check_simple_symmetric(g)


def test_generation_does_not_depend_on_chunking_or_buckets():
    a = synth.powerlaw_graph(5000, 60_000, 200.0, seed=9)
    b = synth.powerlaw_graph(5000, 60_000, 200.0, seed=9, chunk_pairs=777, bucket_keys=5000)
    assert torch.equal(a.indptr, b.indptr) and torch.equal(a.indices, b.indices)
    c = synth.powerlaw_graph(5000, 60_000, 200.0, seed=10)
    assert not torch.equal(a.indices[:1000], c.indices[:1000])


def test_features_are_standard_normal_and_row_major():
    for dtype in (torch.float32, torch.float16):
        f = synth.normal_features(20_000, 33, dtype, seed=3)
        assert f.shape == (20_000, 33) and f.is_contiguous() and f.dtype == dtype
        x = f.double()
        assert abs(x.mean().item()) < 0.01 and abs(x.std().item() - 1.0) < 0.01
        assert abs((x ** 4).mean().item() - 3.0) < 0.15                 # kurtosis of a normal
    a = synth.normal_features(1000, 8, torch.float32, seed=3, chunk_rows=17)
    b = synth.normal_features(1000, 8, torch.float32, seed=3)
    assert torch.equal(a, b)


def test_seed_splits():
    w = synth.WORKLOADS["mid"]
    batches = synth.make_seed_batches(w)
    allseeds = torch.cat(batches).numpy()
    assert len(allseeds) == int(0.55 * w.num_nodes) and len(np.unique(allseeds)) == len(allseeds)
    assert all(b.numel() == w.batch_size for b in batches[:-1]) and 0 < batches[-1].numel() <= w.batch_size
    assert batches[0].dtype == torch.int32
    # the inference split of the large graph does not overlap its training split
    tr, te = synth.WORKLOADS["large"], synth.WORKLOADS["large_wide"]
    perm = synth.node_permutation(tr.num_nodes, tr.graph_seed)
    a = perm[: int(tr.split_frac * tr.num_nodes)]
    b0 = int(te.split_offset_frac * te.num_nodes)
    b = perm[b0: b0 + int(te.split_frac * te.num_nodes)]
    assert len(np.intersect1d(a.numpy(), b.numpy())) == 0
    assert synth.batch_rng_key(w, 7) == (w.graph_seed << 32) | 7

"""Shared test utilities: small hand-made graphs and a brute-force MFG checker.

The checker verifies a result against the graph alone (it never recomputes the sample), so it
applies to the oracle's output and to the HIP library's output alike.
"""
from __future__ import annotations

import numpy as np


def csr_from_adj(adj):
    """adj: list of neighbour lists -> (indptr int64, indices int32)."""
    indptr = np.zeros(len(adj) + 1, dtype=np.int64)
    for i, row in enumerate(adj):
        indptr[i + 1] = indptr[i] + len(row)
    indices = np.array([u for row in adj for u in row], dtype=np.int32)
    return indptr, indices


def random_simple_graph(n, avg_deg, rng, hub=None):
    """Symmetric simple graph as adjacency lists with sorted rows; optional hub of given degree."""
    nbrs = [set() for _ in range(n)]
    m = n * avg_deg // 2
    for _ in range(m):
        u, v = int(rng.integers(n)), int(rng.integers(n))
        if u != v:
            nbrs[u].add(v)
            nbrs[v].add(u)
    if hub is not None:
        for v in rng.choice(np.arange(1, n), size=hub, replace=False):
            nbrs[0].add(int(v))
            nbrs[int(v)].add(0)
    return [sorted(s) for s in nbrs]


def check_mfg(indptr, indices, seeds, fanouts, node_ids, blk_indptr, blk_indices, n, e):
    """Structural checks that hold for ANY valid sample (sections 2.2, 4.1; OneHopMFG):

    * node_ids is a list of distinct nodes beginning with the seeds (relabel is a bijection);
    * every block row i holds min(deg, d) distinct true neighbours of node_ids[i];
      the whole row in CSR order when deg <= d;
    * new local ids appear in increasing order along the (dst, slot) scan, and each node list
      N_h is a prefix of N_{h+1};
    * E_h equals the closed form sum_i min(deg_i, d_h).
    """
    L = len(fanouts)
    node_ids = np.asarray(node_ids)
    assert len(n) == L + 1 and len(e) == L
    assert n[0] == len(seeds)
    assert np.array_equal(node_ids[:n[0]], np.asarray(seeds))
    assert len(node_ids) == n[L]
    assert len(np.unique(node_ids)) == len(node_ids)
    deg_all = np.diff(indptr)
    for h in range(L):
        d = fanouts[h]
        bp, bi = np.asarray(blk_indptr[h]), np.asarray(blk_indices[h])
        assert len(bp) == n[h] + 1 and bp[0] == 0 and bp[-1] == e[h] == len(bi)
        dst = node_ids[:n[h]]
        want = np.minimum(deg_all[dst], d)
        assert np.array_equal(np.diff(bp), want)
        assert e[h] == int(want.sum())
        assert n[h] <= n[h + 1] <= n[h] + e[h]
        next_new = n[h]
        for i in range(n[h]):
            v = int(dst[i])
            row_true = indices[indptr[v]:indptr[v + 1]]
            loc = bi[bp[i]:bp[i + 1]]
            assert loc.min(initial=0) >= 0 and loc.max(initial=0) < n[h + 1]
            glob = node_ids[loc]
            assert len(set(glob.tolist())) == len(glob)
            assert set(glob.tolist()) <= set(row_true.tolist())
            if len(row_true) <= d:
                assert np.array_equal(glob, row_true)
            for x in loc.tolist():
                if x >= next_new:          # first appearance of a new node
                    assert x == next_new
                    next_new += 1
        assert next_new == n[h + 1]

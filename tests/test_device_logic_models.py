"""CPU models of the two reformulations the kernels rely on, each checked against the oracle.

The HIP path does not walk a destination's slots one by one (Floyd's rule), nor a hop's samples
one by one (the first-encounter numbering of procedure OneHopMFG).  It settles both in parallel:

* Floyd's rule by a duplicate test plus pointer jumping (`floyd_positions` of the wide sampler);
* the numbering by grouping records by node hash, keeping the smallest value per node, and an
  exclusive scan of the first appearances in (destination, slot) order (the partition strategy).

The models below restate those steps in plain Python / numpy, in the kernels' order, and are
compared with the oracle: they show that the reformulations are exact, so that a GPU mismatch can
only be a coding error.  (The GPU parity tests compare the kernels themselves with the oracle.)
"""
import itertools

import numpy as np
import pytest

import oracle
from helpers import csr_from_adj, random_simple_graph

KNOWN, REFUSED, REF_MASK = 0x80000000, 0x40000000, 0x3FFFFFFF


def floyd_by_pointer_jumping(deg, k, draws):
    """draws[s] in [0, deg - k + s].  Slot s is refused (takes j_s = deg - k + s) exactly if an
    earlier slot drew the same value, or if its draw is the j of the earlier slot
    q = draws[s] - (deg - k) and slot q was refused itself."""
    j0 = deg - k
    state = [0] * k
    for s in range(k):
        t = draws[s]
        dup = any(draws[q] == t for q in range(s))
        refers = (not dup) and t >= j0 and t - j0 < s
        state[s] = (KNOWN | REFUSED) if dup else ((t - j0) if refers else KNOWN)
    passes = 0
    while True:
        open_ = False
        nxt = list(state)
        for s in range(k):                      # all slots at once: reads see the previous pass
            if not state[s] & KNOWN:
                sq = state[state[s] & REF_MASK]
                nxt[s] = sq if sq & KNOWN else sq & REF_MASK
                open_ = open_ or not sq & KNOWN
        state = nxt
        passes += 1
        if not open_:
            break
    return [j0 + s if state[s] & REFUSED else draws[s] for s in range(k)], passes


def words_for(draws, deg, k):
    """32-bit words that the oracle's floor scaling turns into the given draws."""
    out = []
    for s, t in enumerate(draws):
        m = deg - k + s + 1
        out.append(-(-(t << 32) // m))          # smallest w with floor(w m / 2^32) = t
    return out


def test_floyd_by_pointer_jumping_equals_the_serial_rule_exhaustively():
    """Every possible sequence of draws for small (deg, k): the parallel settlement gives the serial
    positions, slot by slot."""
    for deg, k in [(3, 2), (4, 3), (5, 3), (5, 4), (6, 4), (7, 3), (6, 5)]:
        ranges = [range(deg - k + s + 1) for s in range(k)]
        for draws in itertools.product(*ranges):
            got, _ = floyd_by_pointer_jumping(deg, k, list(draws))
            ref = oracle.floyd_positions(deg, k, words_for(draws, deg, k))
            assert got == list(ref), (deg, k, draws)


def test_floyd_by_pointer_jumping_on_dense_and_sparse_rows():
    """Random draws for fanouts up to 1024, degrees from just above the fanout (almost every slot
    refused, long chains of references) to far above it; the passes stay within log2 k + 1."""
    rng = np.random.default_rng(17)
    for k, deg in [(33, 34), (64, 65), (100, 101), (100, 110), (100, 150), (100, 1000), (100, 17000), (257, 300),
                   (1024, 1025), (1024, 1100), (1024, 100000)]:
        for _ in range(6):
            draws = [int(rng.integers(0, deg - k + s + 1)) for s in range(k)]
            got, passes = floyd_by_pointer_jumping(deg, k, draws)
            ref = oracle.floyd_positions(deg, k, words_for(draws, deg, k))
            assert got == list(ref), (deg, k)
            assert len(set(got)) == k and max(got) < deg
            assert passes <= int(np.ceil(np.log2(k))) + 1


def test_floyd_chain_of_references_is_shortcut():
    """A worst case for the references: slot s draws j_{s-1}, and slot 1 is refused as a repeat of
    slot 0, so every later slot is refused 'as the slot before it' - a chain through all k slots."""
    k, deg = 64, 200
    j0 = deg - k
    draws = [5, 5] + [j0 + s - 1 for s in range(2, k)]
    got, passes = floyd_by_pointer_jumping(deg, k, draws)
    assert got == list(oracle.floyd_positions(deg, k, words_for(draws, deg, k)))
    assert got[1:] == [j0 + s for s in range(1, k)]
    assert passes <= 7


HASH = 0x9E3779B1
PEND, RESOLVED, POINTER = 0x80000000, 0x80000000, 0xC0000000


def number_hop_by_partition(known_ids, rows, d, lg_buckets):
    """One hop the way the partition strategy settles it.  known_ids: global ids of the n known
    nodes (destination i = known node i); rows[i]: the sampled global ids of destination i (at most
    d).  Returns (block indptr, block indices, new node ids in local-id order)."""
    n = len(known_ids)
    gsrc = np.full(n * d, -1, dtype=np.int64)            # padded positions pos = i d + s
    rowk = np.array([len(r) for r in rows], dtype=np.int64)
    for i, r in enumerate(rows):
        gsrc[i * d:i * d + len(r)] = r
    # records (node, value): known nodes carry their local id, samples tag | position
    recs = [(int(v), i) for i, v in enumerate(known_ids)]
    recs += [(int(gsrc[p]), PEND | p) for p in range(n * d) if p % d < rowk[p // d]]
    buckets = {}
    for node, val in recs:
        b = ((node * HASH) & 0xFFFFFFFF) >> (32 - lg_buckets) if lg_buckets else 0
        buckets.setdefault(b, []).append((node, val))
    state = gsrc.copy()                                   # a first appearance keeps its node id
    for recs_b in buckets.values():
        least = {}
        for node, val in recs_b:                          # any order: only minima are kept
            least[node] = min(least.get(node, val), val)
        for node, val in recs_b:
            if val >= PEND and least[node] != val:
                m = least[node]
                state[val & 0x3FFFFFFF] = (RESOLVED | m) if m < PEND else (POINTER | (m & 0x3FFFFFFF))
    # first appearances numbered by an exclusive scan in position order
    valid = np.array([p % d < rowk[p // d] for p in range(n * d)])
    first = valid & (state >= 0) & (state < RESOLVED)
    rank = np.cumsum(first) - first
    indptr = np.concatenate([[0], np.cumsum(rowk)])
    indices, new_ids = [], []
    for p in range(n * d):
        if not valid[p]:
            continue
        e = int(state[p])
        if first[p]:
            indices.append(n + int(rank[p]))
            new_ids.append(e)
        elif e & POINTER == POINTER:
            q = e & 0x3FFFFFFF
            assert first[q]                               # a pointer names a first appearance
            indices.append(n + int(rank[q]))
        else:
            indices.append(e & 0x3FFFFFFF)
    return indptr, np.array(indices, dtype=np.int64), np.array(new_ids, dtype=np.int64)


@pytest.mark.parametrize("lg_buckets", [0, 3, 7])
def test_partition_numbering_equals_the_serial_first_encounter_numbering(lg_buckets):
    """Random small dense graphs (many repeats, many known nodes among the samples): per hop, the
    sampled ids of the oracle's own output go through the partition model; block arrays and the new
    nodes' order must come out as the oracle's serial walk numbered them."""
    rng = np.random.default_rng(100 + lg_buckets)
    for trial in range(12):
        n_nodes = int(rng.integers(30, 300))
        adj = random_simple_graph(n_nodes, int(rng.integers(4, 25)), rng, hub=1 if trial % 2 else None)
        indptr, indices = csr_from_adj(adj)
        orc = oracle.Oracle(indptr, indices)
        fan = [(4, 4), (15, 10, 5), (8,), (3, 3, 3, 3)][trial % 4]
        seeds = rng.choice(n_nodes, size=int(rng.integers(1, min(n_nodes, 40))), replace=False).astype(np.int32)
        ref = orc.sample_mfg(seeds, fan, int(rng.integers(0, 2**62)), with_features=False)
        n = ref.num_nodes
        for h, d in enumerate(fan):
            known = ref.node_ids[:n[h]]
            rows = [ref.node_ids[ref.indices[h][ref.indptr[h][i]:ref.indptr[h][i + 1]]] for i in range(n[h])]
            blk_indptr, blk_indices, new_ids = number_hop_by_partition(known, rows, d, lg_buckets)
            assert np.array_equal(blk_indptr, ref.indptr[h])
            assert np.array_equal(blk_indices, ref.indices[h])
            assert np.array_equal(new_ids, ref.node_ids[n[h]:n[h + 1]])

"""Parity at the full benchmark sizes, in the launch configuration bench.py times
(several batches per launch set), against the oracle element by element (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2110_08450_amd import binding as smfg
from paper_2110_08450_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check_batches(w, graph, feat, g, orc, batches, batch_ids, per_call, sample_capacity=0):
    """Runs the chosen batches `per_call` at a time and compares every output array.  The feature
    rows are checked against torch indexing of the same table with the oracle's node list."""
    L = len(w.fanouts)
    wss = [smfg.workspace_create(g, w.batch_size, w.fanouts, 0, sample_capacity) for _ in range(per_call)]
    assert all(ws.strategy == "partition" for ws in wss)      # every benchmark workload but `tiny` takes it
    outs = [smfg.alloc_output(g, w.batch_size, w.fanouts) for _ in range(per_call)]
    for c0 in range(0, len(batch_ids), per_call):
        ids = batch_ids[c0:c0 + per_call]
        keys = [synth.batch_rng_key(w, b) for b in ids]
        k = len(ids)
        smfg.sample_mfg_many(g, wss[:k], [batches[b] for b in ids], w.fanouts, keys, outs[:k])
        for q, b in enumerate(ids):
            c = smfg.read_counts(outs[q])
            ref = orc.sample_mfg(batches[b].cpu().numpy(), w.fanouts, keys[q], with_features=False)
            assert ref.status == 0
            assert c == [int(x) for x in ref.counts], f"batch {b}"
            n, e = c[:L + 1], c[L + 1:2 * L + 1]
            assert np.array_equal(outs[q].node_ids[:n[L]].cpu().numpy(), ref.node_ids), f"batch {b}"
            for h in range(L):
                assert np.array_equal(outs[q].indptr[h][:n[h] + 1].cpu().numpy(), ref.indptr[h]), (b, h)
                assert np.array_equal(outs[q].indices[h][:e[h]].cpu().numpy(), ref.indices[h]), (b, h)
            ids_ref = torch.from_numpy(ref.node_ids).to(DEV).long()
            assert torch.equal(outs[q].features[:n[L]], feat[ids_ref]), f"features of batch {b}"
            print(f"{w.name} batch {b}: nodes {n} edges {e} ok", flush=True)


@pytest.fixture(scope="module")
def large():
    w = synth.WORKLOADS["large"]
    graph = synth.make_graph(w, device=DEV)
    feat = synth.make_features(w, device=DEV)
    g = smfg.graph_create(graph.indptr, graph.indices, feat)
    orc = oracle.Oracle(graph.indptr.cpu().numpy(), graph.indices.cpu().numpy())
    return graph, feat, g, orc


def test_large_workload_first_pass_batches(large):
    """products-shaped workload (fp16 x 100: 200-byte rows), 8 batches per launch set."""
    graph, feat, g, orc = large
    w = synth.WORKLOADS["large"]
    batches = synth.make_seed_batches(w, device=DEV)
    ids = list(range(8)) + [len(batches) // 2, len(batches) - 1]
    _check_batches(w, graph, feat, g, orc, batches, ids, 8)


@pytest.mark.parametrize("name", ["large_wide", "large_all"])
def test_large_fanouts_and_full_neighbourhoods_at_full_size(large, name):
    """The inference fanouts of section 5 / Table 6 on the products-shaped graph, in the launch
    configuration the benchmark times (2 batches per launch set): fanouts (100,100) with 1024 seeds
    (about 2.4 M sampled edges per batch) and full neighbourhoods (-1,-1) with 256 seeds (about
    5.5 M edges per batch, more than the 4096 x 1024 samples one grid pass of the flat kernels
    covers).  First four batches and the last one."""
    graph, feat, g, orc = large
    w = synth.WORKLOADS[name]
    batches = synth.make_seed_batches(w, device=DEV)
    ids = [0, 1, 2, 3, len(batches) - 1]
    _check_batches(w, graph, feat, g, orc, batches, ids, 2, sample_capacity=min(graph.num_edges, (1 << 30) - 1))


def test_wide_path_beyond_one_grid_pass(large):
    """Full neighbourhoods for two hops, then a fanout of 2 over everything found: the last hop has
    more than 4096 x 256 destinations and the second more than 4096 x 1024 samples, so the
    destination-tile and sample-tile kernels of the exact-offset path each wrap around their grid."""
    graph, feat, g, orc = large
    w = synth.WORKLOADS["large_all"]
    seeds = synth.make_seed_batches(w, device=DEV)[0]
    fan = (-1, -1, 2)
    key = 4242
    ref = orc.sample_mfg(seeds.cpu().numpy(), fan, key, with_features=False)
    assert ref.status == 0
    assert ref.num_nodes[2] > 4096 * 256 and ref.num_edges[1] > 4096 * 1024
    m = min(graph.num_edges, (1 << 30) - 1)
    ws = smfg.workspace_create(g, seeds.numel(), fan, 0, m)
    out = smfg.alloc_output(g, seeds.numel(), fan, with_features=False)
    smfg.sample_mfg(g, ws, seeds, fan, key, out)
    c = smfg.read_counts(out)
    assert c == [int(x) for x in ref.counts]
    n, e = c[:4], c[4:7]
    assert np.array_equal(out.node_ids[:n[3]].cpu().numpy(), ref.node_ids)
    for h in range(3):
        assert np.array_equal(out.indptr[h][:n[h] + 1].cpu().numpy(), ref.indptr[h]), h
        assert np.array_equal(out.indices[h][:e[h]].cpu().numpy(), ref.indices[h]), h
    print(f"wide path beyond one grid pass: nodes {n} edges {e} ok", flush=True)


def test_half_a_million_seeds_split_buckets(large):
    """One batch of 500 000 seeds with fanouts (32, 2) on the products-shaped graph: 16 M and 7 M
    records per hop, so the hash buckets of both hops are split into sub-buckets before the dedup
    (the same path the inference-shaped workload takes on the larger graph)."""
    graph, feat, g, orc = large
    w = synth.WORKLOADS["large"]
    seeds = synth.node_permutation(w.num_nodes, w.graph_seed, device=DEV)[:500_000].to(torch.int32).contiguous()
    fan = (32, 2)
    key = 99
    ref = orc.sample_mfg(seeds.cpu().numpy(), fan, key, with_features=False)
    assert ref.status == 0
    ws = smfg.workspace_create(g, seeds.numel(), fan)
    out = smfg.alloc_output(g, seeds.numel(), fan, with_features=False)
    for rep in range(2):
        smfg.sample_mfg(g, ws, seeds, fan, key, out)
        c = smfg.read_counts(out)
        assert c == [int(x) for x in ref.counts]
        n, e = c[:3], c[3:5]
        assert np.array_equal(out.node_ids[:n[2]].cpu().numpy(), ref.node_ids)
        for h in range(2):
            assert np.array_equal(out.indptr[h][:n[h] + 1].cpu().numpy(), ref.indptr[h]), h
            assert np.array_equal(out.indices[h][:e[h]].cpu().numpy(), ref.indices[h]), h
    print(f"500 000 seeds: nodes {n} edges {e} ok", flush=True)


@pytest.fixture(scope="module")
def papers():
    w = synth.WORKLOADS["papers"]
    graph = synth.make_graph(w, device=DEV)
    feat = synth.make_features(w, device=DEV)
    torch.cuda.empty_cache()
    g = smfg.graph_create(graph.indptr, graph.indices, feat)
    orc = oracle.Oracle(graph.indptr.cpu().numpy(), graph.indices.cpu().numpy())
    print(f"papers graph: {graph.num_edges} directed edges", flush=True)
    return graph, feat, g, orc


def test_papers_workload_batches(papers):
    """papers100M-shaped workload (111 M nodes, 3.2 B edges, int64 offsets beyond 2^31), training
    fanouts, 8 batches per launch set; first eight batches and the partial last one."""
    graph, feat, g, orc = papers
    w = synth.WORKLOADS["papers"]
    assert graph.num_edges > 2**31
    batches = synth.make_seed_batches(w, device=DEV)
    assert batches[-1].numel() < w.batch_size
    _check_batches(w, graph, feat, g, orc, batches, list(range(8)) + [len(batches) - 1], 8)


def test_papers_inference_shaped_batches(papers):
    """Same graph, fanouts (20,20,20), 4096 seeds from the held-out split: about 20 M nodes and
    26 M edges per batch (the dedup table's largest load)."""
    graph, feat, g, orc = papers
    w = synth.WORKLOADS["papers_infer"]
    batches = synth.make_seed_batches(w, device=DEV)
    _check_batches(w, graph, feat, g, orc, batches, [0, len(batches) - 1], 2)


def _full_pass(w, graph, feat, g, base_oracle, threads=12, per_call=8):
    """Every batch of one pass over the seed split: GPU in launch sets of `per_call`, the oracle on
    host threads (one scratch map each); counts, node ids and blocks compared bit for bit, feature
    rows against torch indexing."""
    from concurrent.futures import ThreadPoolExecutor
    import queue
    L = len(w.fanouts)
    batches = synth.make_seed_batches(w, device=DEV)
    h_batches = [b.cpu().numpy() for b in batches]
    keys = [synth.batch_rng_key(w, b) for b in range(len(batches))]
    pool_oracles = queue.Queue()
    pool_oracles.put(base_oracle)
    for _ in range(threads - 1):
        pool_oracles.put(base_oracle.clone_scratch())

    def ref_of(b):
        o = pool_oracles.get()
        try:
            return o.sample_mfg(h_batches[b], w.fanouts, keys[b], with_features=False)
        finally:
            pool_oracles.put(o)

    wss = [smfg.workspace_create(g, w.batch_size, w.fanouts) for _ in range(per_call)]
    assert all(ws.strategy == "partition" for ws in wss)
    outs = [smfg.alloc_output(g, w.batch_size, w.fanouts) for _ in range(per_call)]
    total_nodes = total_edges = 0
    with ThreadPoolExecutor(threads) as ex:
        for c0 in range(0, len(batches), per_call):
            ids = list(range(c0, min(len(batches), c0 + per_call)))
            refs = [ex.submit(ref_of, b) for b in ids]
            k = len(ids)
            smfg.sample_mfg_many(g, wss[:k], [batches[b] for b in ids], w.fanouts, [keys[b] for b in ids], outs[:k])
            for q, b in enumerate(ids):
                ref = refs[q].result()
                c = smfg.read_counts(outs[q])
                assert ref.status == 0 and c == [int(x) for x in ref.counts], f"batch {b}"
                n, e = c[:L + 1], c[L + 1:2 * L + 1]
                assert np.array_equal(outs[q].node_ids[:n[L]].cpu().numpy(), ref.node_ids), f"batch {b}"
                for h in range(L):
                    assert np.array_equal(outs[q].indptr[h][:n[h] + 1].cpu().numpy(), ref.indptr[h]), (b, h)
                    assert np.array_equal(outs[q].indices[h][:e[h]].cpu().numpy(), ref.indices[h]), (b, h)
                assert torch.equal(outs[q].features[:n[L]], feat[outs[q].node_ids[:n[L]].long()]), f"batch {b}"
                total_nodes += n[L]
                total_edges += sum(e)
            if c0 % (per_call * 16) == 0:
                print(f"{w.name}: {c0 + k} of {len(batches)} batches identical", flush=True)
    print(f"{w.name}: full pass of {len(batches)} batches identical, {total_nodes} nodes, {total_edges} edges",
          flush=True)


def test_mid_workload_full_pass():
    w = synth.WORKLOADS["mid"]
    graph = synth.make_graph(w, device=DEV)
    feat = synth.make_features(w, device=DEV)
    g = smfg.graph_create(graph.indptr, graph.indices, feat)
    _full_pass(w, graph, feat, g, oracle.Oracle(graph.indptr.cpu().numpy(), graph.indices.cpu().numpy()))


def test_large_workload_full_pass(large):
    graph, feat, g, orc = large
    _full_pass(synth.WORKLOADS["large"], graph, feat, g, orc)


def test_papers_workload_full_pass(papers):
    """All 1193 batches of the pass over the 1.1 % train split of the papers100M-shaped graph."""
    graph, feat, g, orc = papers
    _full_pass(synth.WORKLOADS["papers"], graph, feat, g, orc)


def test_papers_inference_full_pass(papers):
    """All 55 batches of the held-out split with fanouts (20,20,20): about 1.07 G nodes and 1.4 G
    edges in total."""
    graph, feat, g, orc = papers
    _full_pass(synth.WORKLOADS["papers_infer"], graph, feat, g, orc, threads=8, per_call=2)

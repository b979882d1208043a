"""smfg_sample_mfg_static (the entry point that allocates nothing; its scratch is a fixed array
inside the library) against smfg_sample_mfg on the same inputs, bit for bit (needs an MI355X)."""
import numpy as np
import pytest
import torch

from paper_2110_08450_amd import binding as smfg
from paper_2110_08450_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _fetch(out, L):
    c = smfg.read_counts(out)
    n, e = c[:L + 1], c[L + 1:2 * L + 1]
    return dict(counts=c, node_ids=out.node_ids[:n[L]].cpu().numpy(),
                indptr=[out.indptr[h][:n[h] + 1].cpu().numpy() for h in range(L)],
                indices=[out.indices[h][:e[h]].cpu().numpy() for h in range(L)],
                features=out.features[:n[L]].cpu().numpy().view(np.uint8))


def _same(a, b, L):
    assert a["counts"] == b["counts"]
    assert np.array_equal(a["node_ids"], b["node_ids"])
    for h in range(L):
        assert np.array_equal(a["indptr"][h], b["indptr"][h]), h
        assert np.array_equal(a["indices"][h], b["indices"][h]), h
    assert np.array_equal(a["features"], b["features"])


def test_static_scratch_entry_point_matches_the_workspace_one():
    """Two calls in a row on the shared scratch array, the second with a smaller input and other
    fanouts (what the first call left in the array must not show), then the first input again."""
    w = synth.WORKLOADS["mid"]
    graph = synth.make_graph(w, device=DEV)
    feat = synth.make_features(w, device=DEV)
    batches = synth.make_seed_batches(w, device=DEV)
    g = smfg.graph_create(graph.indptr, graph.indices, feat)
    cases = [(batches[0], w.fanouts, synth.batch_rng_key(w, 0)),
             (batches[1][:100].contiguous(), (7, 3), synth.batch_rng_key(w, 1)),
             (batches[0], w.fanouts, synth.batch_rng_key(w, 0)),
             (batches[2][:300].contiguous(), (40, 2), synth.batch_rng_key(w, 2))]    # a wide fanout
    for seeds, fanouts, key in cases:
        L = len(fanouts)
        ws = smfg.workspace_create(g, seeds.numel(), fanouts)
        assert ws.nbytes <= smfg.STATIC_SCRATCH_BYTES
        ref_out = smfg.alloc_output(g, seeds.numel(), fanouts)
        out = smfg.alloc_output(g, seeds.numel(), fanouts)
        smfg.sample_mfg(g, ws, seeds, fanouts, key, ref_out)
        ref = _fetch(ref_out, L)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]      # the driver's view: sees any hipMalloc, torch's or not
        smfg.sample_mfg_static(g, seeds, fanouts, key, out)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] >= free_before
        got = _fetch(out, L)
        _same(got, ref, L)
        print(f"static scratch: {seeds.numel()} seeds, fanouts {fanouts}: nodes {got['counts'][:L + 1]} identical",
              flush=True)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    """Sizes beyond the array are refused on the host, before any launch."""
    w = synth.WORKLOADS["tiny"]
    graph = synth.make_graph(w, device=DEV)
    feat = synth.make_features(w, device=DEV)
    g = smfg.graph_create(graph.indptr, graph.indices, feat)
    seeds = synth.make_seed_batches(w, device=DEV)[0]
    out = smfg.alloc_output(g, seeds.numel(), w.fanouts)
    out.c.node_capacity = 1 << 28            # claims room for 2^28 nodes: a table far beyond the array
    # the graph caps the reachable nodes at 10 000, so this still fits; a fanout of "all" has no bound
    smfg.sample_mfg_static(g, seeds, w.fanouts, 1, out)
    assert smfg.read_counts(out)[-1] == 0
    with pytest.raises(smfg.SmfgError) as ei:
        smfg.sample_mfg_static(g, seeds, (smfg.FANOUT_ALL,), 1, out)
    assert ei.value.code == smfg.ERR_INVALID_ARG
    big = synth.WORKLOADS["papers"]           # 1024 x (15,10,5,32) on a graph of 111 M nodes needs > 64 MiB
    indptr = torch.zeros(big.num_nodes + 1, dtype=torch.int64, device=DEV)
    g2 = smfg.graph_create(indptr, torch.zeros(1, dtype=torch.int32, device=DEV)[:0], None)
    seeds2 = torch.arange(1024, dtype=torch.int32, device=DEV)
    fan = (15, 10, 5, 32)
    out2 = smfg.alloc_output(g2, 1024, fan, node_capacity=4_000_000, edge_capacity=[16] * 4)
    with pytest.raises(smfg.SmfgError) as ei:
        smfg.sample_mfg_static(g2, seeds2, fan, 1, out2)
    assert ei.value.code == smfg.ERR_CAPACITY

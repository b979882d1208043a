"""HIP library vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from helpers import check_mfg, csr_from_adj, random_simple_graph
from paper_2110_08450_amd import binding as smfg
from paper_2110_08450_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True, params=["partition", "table"])
def dedup_strategy(request, monkeypatch):
    """Every test of this file runs with both dedup strategies of the fast path: the hash partition
    (no global table; the default unless every hop of a call is small) and the global table (what
    small calls and wide fanouts use).  The environment variable SMFG_DEDUP selects one for the
    workspaces created while it is set."""
    monkeypatch.setenv("SMFG_DEDUP", request.param)   # also for calls whose size alone would pick the other
    return request.param


class GpuGraph:
    def __init__(self, indptr, indices, feat):
        self.h_indptr, self.h_indices, self.h_feat = indptr, indices, feat
        self.indptr = torch.from_numpy(np.ascontiguousarray(indptr)).to(DEV)
        self.indices = torch.from_numpy(np.ascontiguousarray(indices)).to(DEV)
        self.feat = torch.from_numpy(feat).to(DEV) if feat is not None else None
        self.g = smfg.graph_create(self.indptr, self.indices, self.feat)
        self.oracle = oracle.Oracle(indptr, indices,
                                    feat.view(np.uint8).reshape(feat.shape[0], -1) if feat is not None else None)


def fetch(out, L):
    """Device outputs -> host arrays trimmed to the reported counts."""
    c = smfg.read_counts(out, check=False)
    n, e, st = c[:L + 1], c[L + 1:2 * L + 1], c[2 * L + 1]
    if st != 0:
        return dict(status=st, counts=c)
    res = dict(status=0, counts=c, n=n, e=e,
               node_ids=out.node_ids[:n[L]].cpu().numpy(),
               indptr=[out.indptr[h][:n[h] + 1].cpu().numpy() for h in range(L)],
               indices=[out.indices[h][:e[h]].cpu().numpy() for h in range(L)])
    if out.features is not None:
        rb = out.features.shape[1] * out.features.element_size()
        res["features"] = out.features[:n[L]].cpu().numpy().view(np.uint8).reshape(n[L], rb)
    return res


def assert_same(res, ref, L):
    """Bit-exact: counts, node ids, block indptr / indices, feature bytes."""
    assert res["status"] == 0 and ref.status == 0
    assert res["counts"] == [int(x) for x in ref.counts]
    assert np.array_equal(res["node_ids"], ref.node_ids)
    for h in range(L):
        assert np.array_equal(res["indptr"][h], ref.indptr[h]), f"indptr hop {h}"
        assert np.array_equal(res["indices"][h], ref.indices[h]), f"indices hop {h}"
    if ref.features is not None:
        assert np.array_equal(res["features"], ref.features)


def run_one(gg, seeds_np, fanouts, key, **cap):
    import os
    seeds = torch.from_numpy(np.ascontiguousarray(seeds_np, dtype=np.int32)).to(DEV)
    ws = smfg.workspace_create(gg.g, len(seeds_np), fanouts)
    assert ws.strategy == os.environ["SMFG_DEDUP"]      # the strategy under test is the one that runs
    out = smfg.alloc_output(gg.g, len(seeds_np), fanouts, **cap)
    smfg.sample_mfg(gg.g, ws, seeds, fanouts, key, out)
    return fetch(out, len(fanouts))


@pytest.fixture(scope="module")
def tiny():
    w = synth.WORKLOADS["tiny"]
    g = synth.make_graph(w)
    f = synth.make_features(w)
    return w, GpuGraph(g.indptr.numpy(), g.indices.numpy(), f.numpy()), synth.make_seed_batches(w)


def test_tiny_workload_all_batches(tiny):
    w, gg, batches = tiny
    for b, seeds in enumerate(batches):
        key = synth.batch_rng_key(w, b)
        res = run_one(gg, seeds.numpy(), w.fanouts, key)
        ref = gg.oracle.sample_mfg(seeds.numpy(), w.fanouts, key)
        assert_same(res, ref, len(w.fanouts))
        check_mfg(gg.h_indptr, gg.h_indices, seeds.numpy(), w.fanouts, res["node_ids"], res["indptr"],
                  res["indices"], res["n"], res["e"])


def test_many_equals_single_and_is_repeatable(tiny):
    w, gg, batches = tiny
    L = len(w.fanouts)
    G = len(batches)
    wss = [smfg.workspace_create(gg.g, w.batch_size, w.fanouts) for _ in range(G)]
    outs = [smfg.alloc_output(gg.g, w.batch_size, w.fanouts) for _ in range(G)]
    seeds = [b.to(DEV) for b in batches]
    keys = [synth.batch_rng_key(w, b) for b in range(G)]
    for rep in range(2):                     # second round reuses the dirty workspaces
        smfg.sample_mfg_many(gg.g, wss, seeds, w.fanouts, keys, outs)
        for b in range(G):
            ref = gg.oracle.sample_mfg(batches[b].numpy(), w.fanouts, keys[b])
            assert_same(fetch(outs[b], L), ref, L)


@pytest.mark.parametrize("fanouts", [(1,), (3, 1), (4, 4), (5, 8), (9,), (16, 2), (17,), (32, 3), (2, 2, 2, 2),
                                     (7, 6), (21, 13), (32, 32), (2,) * 8])
def test_fanout_group_sizes(fanouts):
    """Every lane-group width (4, 8, 16, 32) and both branches (whole row / Floyd)."""
    rng = np.random.default_rng(sum(fanouts))
    adj = random_simple_graph(3000, 12, rng, hub=900)
    adj[7] = []                                              # isolated node as a destination
    adj = [[u for u in row if u != 7] for row in adj]
    indptr, indices = csr_from_adj(adj)
    feat = rng.standard_normal((3000, 8)).astype(np.float32)
    gg = GpuGraph(indptr, indices, feat)
    seeds = np.concatenate([[7, 0], rng.choice(np.arange(8, 3000), size=1201, replace=False)]).astype(np.int32)
    res = run_one(gg, seeds, fanouts, 0xC0FFEE)
    ref = gg.oracle.sample_mfg(seeds, fanouts, 0xC0FFEE)
    assert_same(res, ref, len(fanouts))


@pytest.mark.parametrize("dim,dtype", [(100, np.float16), (3, np.float16), (5, np.uint8), (1, np.float32),
                                       (128, np.float16), (33, np.float32)])
def test_gather_row_widths(dim, dtype):
    """Row sizes that take the 16-, 8-, 4-, 2- and 1-byte vector paths."""
    rng = np.random.default_rng(dim)
    adj = random_simple_graph(2000, 10, rng)
    indptr, indices = csr_from_adj(adj)
    feat = (rng.standard_normal((2000, dim)) * 50).astype(dtype)
    gg = GpuGraph(indptr, indices, feat)
    seeds = rng.choice(2000, size=300, replace=False).astype(np.int32)
    res = run_one(gg, seeds, (6, 4), 99)
    ref = gg.oracle.sample_mfg(seeds, (6, 4), 99)
    assert_same(res, ref, 2)
    # stand-alone gather entry point against torch indexing
    ids = torch.from_numpy(res["node_ids"]).to(DEV)
    n = torch.tensor([ids.numel()], dtype=torch.int64, device=DEV)
    out = torch.zeros((ids.numel() + 3, dim), dtype=gg.feat.dtype, device=DEV)
    smfg.gather_rows(gg.g, ids, n, ids.numel() + 3, out)
    torch.cuda.synchronize()
    assert torch.equal(out[:ids.numel()], gg.feat[ids.long()])
    assert (out[ids.numel():] == 0).all()


def test_gather_very_long_rows():
    """Rows of more than 8192 sixteen-byte vectors (and of an odd number of 4-byte ones): the row /
    column split of the gather's flat index takes its division path."""
    rng = np.random.default_rng(31)
    adj = random_simple_graph(60, 6, rng)
    indptr, indices = csr_from_adj(adj)
    for dim in (4 * 8200, 8200 + 1):
        feat = rng.integers(-2**31, 2**31 - 1, size=(60, dim), dtype=np.int64).astype(np.int32).view(np.float32)
        gg = GpuGraph(indptr, indices, feat)
        ids = torch.from_numpy(rng.permutation(60).astype(np.int32)).to(DEV)
        n = torch.tensor([45], dtype=torch.int64, device=DEV)
        out = torch.zeros((60, dim), dtype=torch.float32, device=DEV)
        smfg.gather_rows(gg.g, ids, n, 60, out)
        torch.cuda.synchronize()
        assert torch.equal(out[:45].view(torch.int32), gg.feat[ids[:45].long()].view(torch.int32))
        assert (out[45:].view(torch.int32) == 0).all()


def test_ragged_batches_in_one_call(tiny):
    """16 batches of different sizes (including an empty one) in one launch set."""
    w, gg, batches = tiny
    rng = np.random.default_rng(8)
    sizes = [0, 1, 2, 63, 64, 65, 255, 256, 100, 17, 200, 31, 128, 5, 250, 77]
    seeds = [rng.choice(gg.g.num_nodes, size=k, replace=False).astype(np.int32) for k in sizes]
    fan = (6, 11, 3)
    wss = [smfg.workspace_create(gg.g, 256, fan) for _ in sizes]
    outs = [smfg.alloc_output(gg.g, 256, fan) for _ in sizes]
    keys = [1000 + i for i in range(len(sizes))]
    smfg.sample_mfg_many(gg.g, wss, [torch.from_numpy(s).to(DEV) for s in seeds], fan, keys, outs)
    for i in range(len(sizes)):
        assert_same(fetch(outs[i], 3), gg.oracle.sample_mfg(seeds[i], fan, keys[i]), 3)


@pytest.mark.parametrize("dtype", [np.int64, np.int32, np.int16, np.uint8])
def test_label_slice(tiny, dtype):
    """ys = y[ids[:batch_size]] (Listing 1) written by the same call."""
    w, gg, batches = tiny
    rng = np.random.default_rng(5)
    y = rng.integers(0, 100, size=gg.g.num_nodes).astype(dtype)
    g2 = smfg.graph_create(gg.indptr, gg.indices, gg.feat)
    smfg.graph_set_labels(g2, torch.from_numpy(y).to(DEV))
    ws = smfg.workspace_create(g2, 256, w.fanouts)
    out = smfg.alloc_output(g2, 256, w.fanouts)
    assert out.labels is not None and out.labels.dtype == torch.from_numpy(y).dtype
    for b in (0, 3):
        smfg.sample_mfg(g2, ws, batches[b].to(DEV), w.fanouts, 21, out)
        res = fetch(out, 2)
        assert_same(res, gg.oracle.sample_mfg(batches[b].numpy(), w.fanouts, 21), 2)
        assert np.array_equal(out.labels[:256].cpu().numpy(), oracle.slice_labels(y, batches[b].numpy()))
    # an output that asks for labels on a graph without labels is refused
    with pytest.raises(smfg.SmfgError):
        smfg.sample_mfg(gg.g, smfg.workspace_create(gg.g, 256, w.fanouts), batches[0].to(DEV), w.fanouts, 1, out)


def test_empty_and_single_seed(tiny):
    w, gg, _ = tiny
    res = run_one(gg, np.zeros(0, dtype=np.int32), (3, 2), 5)
    assert res["status"] == 0 and res["counts"] == [0, 0, 0, 0, 0, 0]
    for v in (0, 9999):
        res = run_one(gg, np.array([v], dtype=np.int32), (3, 2), 5)
        assert_same(res, gg.oracle.sample_mfg(np.array([v], dtype=np.int32), (3, 2), 5), 2)


def test_full_neighbourhood_no_rng():
    rng = np.random.default_rng(4)
    adj = random_simple_graph(500, 6, rng)
    maxdeg = max(len(r) for r in adj)
    assert maxdeg <= 32
    indptr, indices = csr_from_adj(adj)
    gg = GpuGraph(indptr, indices, None)
    seeds = rng.choice(500, size=20, replace=False).astype(np.int32)
    a = run_one(gg, seeds, (maxdeg, maxdeg), 1)
    b = run_one(gg, seeds, (maxdeg, maxdeg), 2)
    assert_same(a, gg.oracle.sample_mfg(seeds, (maxdeg, maxdeg), 1), 2)
    assert np.array_equal(a["node_ids"], b["node_ids"])


def test_device_status_codes(tiny):
    w, gg, batches = tiny
    s = batches[0].numpy().copy()
    dup = s.copy(); dup[5] = dup[200]
    assert run_one(gg, dup, (4,), 1)["status"] == smfg.ST_DUPLICATE_SEED
    oob = s.copy(); oob[17] = gg.g.num_nodes
    assert run_one(gg, oob, (4,), 1)["status"] == smfg.ST_SEED_OUT_OF_RANGE
    neg = s.copy(); neg[0] = -1
    assert run_one(gg, neg, (4,), 1)["status"] == smfg.ST_SEED_OUT_OF_RANGE
    ref = gg.oracle.sample_mfg(s, (10, 5), 3)
    n, e = ref.num_nodes, ref.num_edges
    assert run_one(gg, s, (10, 5), 3, node_capacity=n[2] - 1)["status"] == smfg.ST_NODE_CAPACITY
    assert run_one(gg, s, (10, 5), 3, node_capacity=n[1] - 1)["status"] == smfg.ST_NODE_CAPACITY
    assert run_one(gg, s, (10, 5), 3, edge_capacity=[e[0], e[1] - 1])["status"] == smfg.ST_EDGE_CAPACITY
    # exact capacities succeed
    assert_same(run_one(gg, s, (10, 5), 3, node_capacity=n[2], edge_capacity=e), ref, 2)


def test_overloaded_workspace_reports_and_recovers(tiny):
    """Far more distinct nodes than the workspace was sized for: the call ends with a status
    (table full or node capacity), and the same workspace then serves a small batch correctly."""
    w, gg, batches = tiny
    fan = (10, 5)
    ws = smfg.workspace_create(gg.g, 256, fan, node_capacity=300)
    out = smfg.alloc_output(gg.g, 256, fan, node_capacity=300)
    for rep in range(2):
        smfg.sample_mfg(gg.g, ws, batches[rep].to(DEV), fan, 7 + rep, out)
        st = fetch(out, 2)["status"]
        assert st in (smfg.ST_TABLE_FULL, smfg.ST_NODE_CAPACITY)
        small = batches[2][:12].contiguous()
        smfg.sample_mfg(gg.g, ws, small.to(DEV), (3, 2), 11, out)
        ref = gg.oracle.sample_mfg(small.numpy(), (3, 2), 11)
        assert ref.num_nodes[-1] <= 300
        assert_same(fetch(out, 2), ref, 2)


def test_host_argument_errors(tiny):
    w, gg, batches = tiny
    seeds = batches[0].to(DEV)
    ws = smfg.workspace_create(gg.g, 256, (10, 5))
    out = smfg.alloc_output(gg.g, 256, (10, 5))

    def code(fn):
        with pytest.raises(smfg.SmfgError) as ei:
            fn()
        return ei.value.code
    assert code(lambda: smfg.sample_mfg(gg.g, ws, seeds, (0, 5), 1, out)) == smfg.ERR_BAD_FANOUT
    assert code(lambda: smfg.sample_mfg(gg.g, ws, seeds, (1025,), 1, out)) == smfg.ERR_BAD_FANOUT
    assert code(lambda: smfg.sample_mfg(gg.g, ws, seeds, (-2,), 1, out)) == smfg.ERR_BAD_FANOUT
    assert code(lambda: smfg.sample_mfg(gg.g, ws, seeds, (), 1, out)) == smfg.ERR_TOO_MANY_LAYERS
    assert code(lambda: smfg.sample_mfg(gg.g, ws, seeds, (2,) * 9, 1, out)) == smfg.ERR_TOO_MANY_LAYERS
    big = torch.arange(257, dtype=torch.int32, device=DEV)
    assert code(lambda: smfg.sample_mfg(gg.g, ws, big, (10, 5), 1, out)) == smfg.ERR_TOO_MANY_SEEDS
    assert code(lambda: smfg.sample_mfg(gg.g, ws, seeds, (10, 5, 5), 1,
                                        smfg.alloc_output(gg.g, 256, (10, 5, 5)))) == smfg.ERR_CAPACITY
    assert code(lambda: smfg.sample_mfg_many(gg.g, [ws, ws], [seeds, seeds], (10, 5), [1, 2], [out, out])) \
        == smfg.ERR_INVALID_ARG
    # a smaller request on the same workspace is fine, and the workspace is still usable
    smfg.sample_mfg(gg.g, ws, seeds, (10,), 1, out)
    assert fetch(out, 1)["status"] == 0


def test_host_argument_errors_of_a_launch_set(tiny):
    """Mixed feature buffers, a label buffer without graph labels and misaligned pointers are
    refused on the host before anything is launched (so these cases cannot touch the GPU)."""
    import copy
    import ctypes
    w, gg, batches = tiny
    fan = (10, 5)
    seeds = [batches[b].to(DEV) for b in range(2)]
    wss = [smfg.workspace_create(gg.g, 256, fan) for _ in range(2)]
    outs = [smfg.alloc_output(gg.g, 256, fan) for _ in range(2)]

    def variant(o, **fields):
        v = copy.copy(o)
        v.c = smfg._Output()
        ctypes.memmove(ctypes.byref(v.c), ctypes.byref(o.c), ctypes.sizeof(smfg._Output))
        for k, val in fields.items():
            setattr(v.c, k, val)
        return v

    def code(fn):
        with pytest.raises(smfg.SmfgError) as ei:
            fn()
        return ei.value.code

    def many(os_, sd=seeds):
        smfg.sample_mfg_many(gg.g, wss, sd, fan, [1, 2], os_)
    # either every batch of a set gathers or none: both orders of the mix
    assert code(lambda: many([variant(outs[0], features=None), outs[1]])) == smfg.ERR_INVALID_ARG
    assert code(lambda: many([outs[0], variant(outs[1], features=None)])) == smfg.ERR_INVALID_ARG
    # a label buffer needs the graph's label vector
    lab = torch.zeros(256, dtype=torch.int64, device=DEV)
    assert gg.g.labels is None
    assert code(lambda: many([outs[0], variant(outs[1], labels=lab.data_ptr())])) == smfg.ERR_INVALID_ARG
    # typed pointers must be multiples of their element size
    room = torch.zeros(260, dtype=torch.int32, device=DEV)

    class FakeSeeds:            # "256 int32" starting one byte off an int32 boundary
        dtype = torch.int32

        def numel(self):
            return 256

        def is_contiguous(self):
            return True

        def data_ptr(self):
            return room.data_ptr() + 1
    assert code(lambda: many(outs, [seeds[0], FakeSeeds()])) == smfg.ERR_INVALID_ARG
    assert code(lambda: many([outs[0], variant(outs[1], counts=outs[1].counts.data_ptr() + 4)])) \
        == smfg.ERR_INVALID_ARG
    assert code(lambda: many([outs[0], variant(outs[1], node_ids=outs[1].node_ids.data_ptr() + 2)])) \
        == smfg.ERR_INVALID_ARG
    bad_blk = variant(outs[1])
    bad_blk.c.indices[1] = outs[1].indices[1].data_ptr() + 1
    assert code(lambda: many([outs[0], bad_blk])) == smfg.ERR_INVALID_ARG
    # nothing above disturbed the handles: the plain call still matches the oracle
    many(outs)
    for b in range(2):
        assert_same(fetch(outs[b], 2), gg.oracle.sample_mfg(batches[b].numpy(), fan, b + 1), 2)


def test_mid_workload_sampled_batches():
    """arxiv-shaped workload: first, middle and the partial last batch, element by element."""
    w = synth.WORKLOADS["mid"]
    g = synth.make_graph(w)
    f = synth.make_features(w)
    gg = GpuGraph(g.indptr.numpy(), g.indices.numpy(), f.numpy())
    batches = synth.make_seed_batches(w)
    L = len(w.fanouts)
    ws = smfg.workspace_create(gg.g, w.batch_size, w.fanouts)
    out = smfg.alloc_output(gg.g, w.batch_size, w.fanouts)
    for b in (0, 1, len(batches) // 2, len(batches) - 1):
        key = synth.batch_rng_key(w, b)
        smfg.sample_mfg(gg.g, ws, batches[b].to(DEV), w.fanouts, key, out)
        assert_same(fetch(out, L), gg.oracle.sample_mfg(batches[b].numpy(), w.fanouts, key), L)


def test_pipelined_hand_off_matches_oracle():
    """Two buffer sets, sampling and gather on side streams, the consumer on its own stream: every
    yielded batch equals the oracle's, also when the consumer is slow or reads late."""
    from paper_2110_08450_amd.pipeline import BatchPipeline
    w = synth.WORKLOADS["mid"]
    g = synth.make_graph(w)
    f = synth.make_features(w)
    gg = GpuGraph(g.indptr.numpy(), g.indices.numpy(), f.numpy())
    batches = synth.make_seed_batches(w)[:11]
    keys = [synth.batch_rng_key(w, b) for b in range(len(batches))]
    L = len(w.fanouts)
    pipe = BatchPipeline(gg.g, w.fanouts, w.batch_size, batches_per_set=3)
    dev_batches = [b.to(DEV) for b in batches]
    seen = 0
    held = []
    for outs in pipe.run(dev_batches, keys):
        # consumer work on the current stream: copies that must see complete data
        held = [(o.node_ids.clone(), o.features.clone(), o.counts.clone()) for o in outs]
        burn = torch.randn(2048, 2048, device=DEV) @ torch.randn(2048, 2048, device=DEV)   # a slow consumer
        for o, (ids, feats, cnt) in zip(outs, held):
            ref = gg.oracle.sample_mfg(batches[seen].numpy(), w.fanouts, keys[seen])
            assert_same(fetch(o, L), ref, L)
            n = int(cnt[L].item())
            assert np.array_equal(ids[:n].cpu().numpy(), ref.node_ids)
            assert np.array_equal(feats[:n].cpu().numpy().view(np.uint8).reshape(n, -1), ref.features)
            seen += 1
        del burn
    assert seen == len(batches)


@pytest.mark.parametrize("dim,dtype", [(128, np.float16), (100, np.float16), (33, np.float16),
                                       (128, np.float32), (5, np.float32), (34, np.float16), (300, np.float16),
                                       (272, np.float16), (200, np.float32)])
def test_mean_aggregate_consumer(dim, dtype):
    """GraphSAGE mean aggregation over the blocks of a sampled batch, outermost hop first, feeding
    each layer's output (cast back to the input type) to the next block, as the model listing of
    Appendix C consumes an MFG.  Float sums in slot order, k - 1 rounded additions and one rounded
    division: error <= k * 2^-24 * mean magnitude of the terms."""
    rng = np.random.default_rng(dim)
    adj = random_simple_graph(4000, 14, rng, hub=700)
    adj[3] = []
    adj = [[u for u in row if u != 3] for row in adj]
    indptr, indices = csr_from_adj(adj)
    feat = (rng.standard_normal((4000, dim)) * 4).astype(dtype)
    gg = GpuGraph(indptr, indices, feat)
    seeds = np.concatenate([[3], rng.choice(np.arange(4, 4000), size=700, replace=False)]).astype(np.int32)
    fan = (7, 5, 3)
    seeds_d = torch.from_numpy(seeds).to(DEV)
    ws = smfg.workspace_create(gg.g, len(seeds), fan)
    out = smfg.alloc_output(gg.g, len(seeds), fan)
    smfg.sample_mfg(gg.g, ws, seeds_d, fan, 31, out)
    res = fetch(out, 3)
    ref = gg.oracle.sample_mfg(seeds, fan, 31)
    assert_same(res, ref, 3)
    x_gpu = out.features                       # [cap x dim], first n_3 rows valid
    x_ref = ref.features.view(dtype).reshape(-1, dim)
    for h in (2, 1, 0):
        n_dst = res["n"][h]
        y = torch.full((out.node_capacity, dim), float("nan"), dtype=torch.float32, device=DEV)
        smfg.mean_aggregate(out.indptr[h], out.indices[h], out.counts[h:h + 1], out.indptr[h].numel() - 1, x_gpu, y)
        torch.cuda.synchronize()
        mean, mag = oracle.mean_aggregate(ref.indptr[h], ref.indices[h], np.ascontiguousarray(x_ref))
        got = y[:n_dst].cpu().numpy().astype(np.float64)
        assert np.isnan(y[n_dst:].cpu().numpy()).all()          # nothing written past n_dst
        k = np.diff(ref.indptr[h])
        assert (np.abs(got - mean) <= k[:, None] * 2.0 ** -24 * mag).all(), f"hop {h}"
        assert (got[k == 0] == 0).all()
        # next layer: both sides continue from the GPU's float output cast to the input type
        x_gpu = y[:n_dst].to(x_gpu.dtype).contiguous()
        x_ref = x_gpu.cpu().numpy()


@pytest.mark.parametrize("fanouts", [(33,), (64, 3), (5, 100), (100, 100), (-1,), (3, -1), (-1, -1, -1), (40, -1, 7),
                                     (1024,)])
def test_wide_fanouts_and_full_neighbourhood(fanouts):
    """Fanouts above 32 and SMFG_FANOUT_ALL (every neighbour) take the exact-offset path: rows
    longer than a wave (hub of degree 900, several Floyd rounds), rows shorter than the fanout,
    an isolated destination."""
    rng = np.random.default_rng(len(fanouts) * 100 + abs(fanouts[0]))
    adj = random_simple_graph(3000, 12, rng, hub=900)
    for extra in (1, 2):                                         # two more long rows
        for v in rng.choice(np.arange(10, 3000), size=150 * extra, replace=False):
            if int(v) not in adj[extra]:
                adj[extra].append(int(v)); adj[int(v)].append(extra)
    adj[7] = []
    adj = [sorted(set(u for u in row if u != 7)) for row in adj]
    indptr, indices = csr_from_adj(adj)
    feat = rng.standard_normal((3000, 8)).astype(np.float32)
    gg = GpuGraph(indptr, indices, feat)
    seeds = np.concatenate([[7, 0, 1, 2], rng.choice(np.arange(8, 3000), size=300, replace=False)]).astype(np.int32)
    ref = gg.oracle.sample_mfg(seeds, fanouts, 0xABCDEF)
    assert ref.status == 0
    m = len(indices)
    ws = smfg.workspace_create(gg.g, len(seeds), fanouts, node_capacity=3000, sample_capacity=m)
    out = smfg.alloc_output(gg.g, len(seeds), fanouts, node_capacity=3000, edge_capacity=[m] * len(fanouts))
    smfg.sample_mfg(gg.g, ws, torch.from_numpy(seeds).to(DEV), fanouts, 0xABCDEF, out)
    res = fetch(out, len(fanouts))
    assert_same(res, ref, len(fanouts))
    if all(d > 0 for d in fanouts):
        check_mfg(indptr, indices, seeds, fanouts, res["node_ids"], res["indptr"], res["indices"], res["n"], res["e"])
    # a fast-path call on the same workspace afterwards still works
    out2 = smfg.alloc_output(gg.g, len(seeds), (4, 3), node_capacity=3000)
    smfg.sample_mfg(gg.g, ws, torch.from_numpy(seeds).to(DEV), (4, 3), 5, out2)
    assert_same(fetch(out2, 2), gg.oracle.sample_mfg(seeds, (4, 3), 5), 2)


def test_wide_path_capacity_status():
    rng = np.random.default_rng(3)
    adj = random_simple_graph(1000, 20, rng)
    indptr, indices = csr_from_adj(adj)
    gg = GpuGraph(indptr, indices, None)
    seeds = rng.choice(1000, size=50, replace=False).astype(np.int32)
    ref = gg.oracle.sample_mfg(seeds, (-1, -1), 1)
    e = ref.num_edges
    ws = smfg.workspace_create(gg.g, 50, (-1, -1), node_capacity=1000, sample_capacity=e[1] - 1)
    out = smfg.alloc_output(gg.g, 50, (-1, -1), node_capacity=1000, edge_capacity=[len(indices)] * 2)
    smfg.sample_mfg(gg.g, ws, torch.from_numpy(seeds).to(DEV), (-1, -1), 1, out)
    assert fetch(out, 2)["status"] == smfg.ST_EDGE_CAPACITY
    with pytest.raises(smfg.SmfgError):                 # no bound without an explicit sample capacity
        smfg.workspace_create(gg.g, 50, (-1, -1), node_capacity=1000)
    ws2 = smfg.workspace_create(gg.g, 50, (-1, -1), node_capacity=1000, sample_capacity=e[1])
    smfg.sample_mfg(gg.g, ws2, torch.from_numpy(seeds).to(DEV), (-1, -1), 1, out)
    assert_same(fetch(out, 2), ref, 2)


def test_launch_set_replays_from_a_hip_graph(tiny):
    """A launch set allocates nothing and never synchronises, so it can be captured into a HIP
    graph; every replay (with eager work and synchronisation in between) must give the oracle's
    result again, the workspace resetting itself each time."""
    w, gg, batches = tiny
    L = len(w.fanouts)
    G = 3
    wss = [smfg.workspace_create(gg.g, w.batch_size, w.fanouts) for _ in range(G)]
    outs = [smfg.alloc_output(gg.g, w.batch_size, w.fanouts) for _ in range(G)]
    seeds = [torch.empty(w.batch_size, dtype=torch.int32, device=DEV) for _ in range(G)]
    keys = [synth.batch_rng_key(w, b) for b in range(G)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up outside the capture
        for b in range(G):
            seeds[b].copy_(batches[b].to(DEV))
        smfg.sample_mfg_many(gg.g, wss, seeds, w.fanouts, keys, outs, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        smfg.sample_mfg_many(gg.g, wss, seeds, w.fanouts, keys, outs, stream=torch.cuda.current_stream())
    refs = {}
    for rep in range(4):
        # new seeds in the same buffers for replays 2 and 3: the captured pointers stay valid
        shift = rep % 2
        for b in range(G):
            seeds[b].copy_(batches[(b + shift) % len(batches)].to(DEV))
        for o in outs:                                  # eager work between the replays
            o.node_ids.fill_(-7)
            o.features.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for b in range(G):
            src = (b + shift) % len(batches)
            ref = refs.setdefault((src, b), gg.oracle.sample_mfg(batches[src].numpy(), w.fanouts, keys[b]))
            assert_same(fetch(outs[b], L), ref, L)


def test_one_bad_batch_does_not_disturb_the_others(tiny):
    """In a launch set, a batch with a duplicate seed, one with an out-of-range seed and one whose
    node capacity is too small end with their own status; the remaining batches match the oracle."""
    w, gg, batches = tiny
    fan = w.fanouts
    good = [batches[0].numpy(), batches[1].numpy()]
    dup = batches[2].numpy().copy(); dup[3] = dup[77]
    oob = batches[3].numpy().copy(); oob[100] = -5
    seeds = [good[0], dup, good[1], oob, batches[2].numpy()]
    caps = [None, None, None, None, 1000]           # the last one overflows its node capacity
    wss = [smfg.workspace_create(gg.g, 256, fan) for _ in seeds]
    outs = [smfg.alloc_output(gg.g, 256, fan, node_capacity=c) for c in caps]
    keys = [50 + i for i in range(len(seeds))]
    for rep in range(2):
        smfg.sample_mfg_many(gg.g, wss, [torch.from_numpy(x).to(DEV) for x in seeds], fan, keys, outs)
        st = [fetch(o, 2) for o in outs]
        assert st[1]["status"] == smfg.ST_DUPLICATE_SEED and st[3]["status"] == smfg.ST_SEED_OUT_OF_RANGE
        assert st[4]["status"] == smfg.ST_NODE_CAPACITY
        assert_same(st[0], gg.oracle.sample_mfg(seeds[0], fan, keys[0]), 2)
        assert_same(st[2], gg.oracle.sample_mfg(seeds[2], fan, keys[2]), 2)


def test_wide_path_overload_and_recovery():
    """Wide path with a node capacity far too small: table full or node capacity status, then the
    same workspace serves a call that fits."""
    rng = np.random.default_rng(12)
    adj = random_simple_graph(2000, 16, rng, hub=500)
    indptr, indices = csr_from_adj(adj)
    gg = GpuGraph(indptr, indices, None)
    seeds = np.concatenate([[0], rng.choice(np.arange(1, 2000), size=99, replace=False)]).astype(np.int32)
    m = len(indices)
    ws = smfg.workspace_create(gg.g, 100, (-1, 40), node_capacity=150, sample_capacity=m)
    out = smfg.alloc_output(gg.g, 100, (-1, 40), node_capacity=150, edge_capacity=[m, m])
    for rep in range(2):
        smfg.sample_mfg(gg.g, ws, torch.from_numpy(seeds).to(DEV), (-1, 40), 3, out)
        assert fetch(out, 2)["status"] in (smfg.ST_TABLE_FULL, smfg.ST_NODE_CAPACITY)
        few = seeds[1:4].copy()
        smfg.sample_mfg(gg.g, ws, torch.from_numpy(few).to(DEV), (-1, 40), 4, out)
        ref = gg.oracle.sample_mfg(few, (-1, 40), 4)
        if ref.num_nodes[-1] <= 150:
            assert_same(fetch(out, 2), ref, 2)
        else:
            assert fetch(out, 2)["status"] != 0
        one = smfg.alloc_output(gg.g, 100, (40,), node_capacity=150, edge_capacity=[m])
        smfg.sample_mfg(gg.g, ws, torch.from_numpy(few).to(DEV), (40,), 4, one)
        assert_same(fetch(one, 1), gg.oracle.sample_mfg(few, (40,), 4), 1)


def test_multigraph_rows_and_self_loops():
    """Rows with repeated neighbours and self loops: sampling is over row positions, so a block row
    may name the same source twice and a node may be its own neighbour; the oracle defines it."""
    rng = np.random.default_rng(77)
    n = 500
    adj = []
    for v in range(n):
        k = int(rng.integers(0, 30))
        row = rng.integers(0, n, size=k).tolist()          # with repeats
        if v % 7 == 0:
            row += [v, v]                                   # self loops, twice
        adj.append(row)
    indptr, indices = csr_from_adj(adj)
    gg = GpuGraph(indptr, indices, rng.standard_normal((n, 4)).astype(np.float32))
    seeds = rng.choice(n, size=64, replace=False).astype(np.int32)
    for fan in [(5, 5), (32,), (3, 3, 3), (-1, 4), (40, -1)]:
        ref = gg.oracle.sample_mfg(seeds, fan, 9)
        m = len(indices)
        ws = smfg.workspace_create(gg.g, 64, fan, node_capacity=n, sample_capacity=m)
        out = smfg.alloc_output(gg.g, 64, fan, node_capacity=n, edge_capacity=[m] * len(fan))
        smfg.sample_mfg(gg.g, ws, torch.from_numpy(seeds).to(DEV), fan, 9, out)
        assert_same(fetch(out, len(fan)), ref, len(fan))


def test_giant_hub_and_isolated_seeds():
    """A hub of degree 120 000 (more than 2^16 positions to draw from, many Floyd rounds on the wide
    path, a row of 1875 rounds when every neighbour is taken) and a batch of isolated seeds."""
    rng = np.random.default_rng(5)
    n = 150_000
    hub_nbrs = np.sort(rng.choice(np.arange(1, n), size=120_000, replace=False))
    indptr = np.zeros(n + 1, dtype=np.int64)
    deg = np.zeros(n, dtype=np.int64)
    deg[0] = len(hub_nbrs)
    deg[hub_nbrs] = 1
    indptr[1:] = np.cumsum(deg)
    indices = np.zeros(int(indptr[-1]), dtype=np.int32)
    indices[:len(hub_nbrs)] = hub_nbrs                      # row 0; every neighbour's row is [0]
    gg = GpuGraph(indptr, indices, None)
    lonely = np.setdiff1d(np.arange(1, n), hub_nbrs)[:50].astype(np.int32)
    seeds = np.concatenate([[0], hub_nbrs[:20]]).astype(np.int32)
    m = len(indices)
    for fan in [(32, 2), (10,), (1024,), (-1,), (-1, 3), (500, -1)]:
        for s in (seeds, lonely):
            ref = gg.oracle.sample_mfg(s, fan, 1234)
            ws = smfg.workspace_create(gg.g, len(s), fan, node_capacity=n, sample_capacity=m)
            out = smfg.alloc_output(gg.g, len(s), fan, node_capacity=n, edge_capacity=[m] * len(fan))
            smfg.sample_mfg(gg.g, ws, torch.from_numpy(s).to(DEV), fan, 1234, out)
            assert_same(fetch(out, len(fan)), ref, len(fan))
    assert gg.oracle.sample_mfg(lonely, (5, 5), 1).num_edges == [0, 0]


def test_partition_bucket_overflow_and_rounds(dedup_strategy):
    """The partition strategy's per-bucket LDS table: 5000 distinct nodes whose hashes share their
    12 leading bits all land in one bucket and, on the first attempt, in one round of that
    bucket, which overflows the 4096-slot table; the bucket must start over with more rounds and
    still number every node exactly as the serial walk does.  Each of those nodes is sampled 12
    times (60 000 single-neighbour destinations), so the rounds also see repeats."""
    hash_mult = 0x9E3779B1            # the library's bucket hash is node * this mod 2^32, leading bits
    n = 1 << 25
    h = (np.arange(n, dtype=np.uint64) * np.uint64(hash_mult)) & np.uint64(0xFFFFFFFF)
    special = np.nonzero((h >> np.uint64(20)) == np.uint64(0x5A3))[0][:5000]
    assert len(special) == 5000
    seeds = np.setdiff1d(np.arange(70_000), special)[:60_000].astype(np.int32)     # sorted
    deg = np.zeros(n, dtype=np.int64)
    deg[seeds] = 1
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=indptr[1:])
    indices = special[np.arange(len(seeds)) % len(special)].astype(np.int32)       # row of the j-th seed
    gg = GpuGraph(indptr, indices, None)
    rng = np.random.default_rng(5)
    order = rng.permutation(len(seeds))
    # the table strategy probes linearly from the same hash, so for it these ids are one long
    # cluster: slow, still exact; a second hop makes the call too large for the partition strategy
    for fan in [(32,), (32, 1)] if dedup_strategy == "partition" else [(32,)]:
        s = seeds[order]
        ref = gg.oracle.sample_mfg(s, fan, 77)
        assert ref.num_nodes[1] == 65_000
        res = run_one(gg, s, fan, 77)
        assert_same(res, ref, len(fan))


def test_single_node_graph():
    indptr = np.array([0, 0], dtype=np.int64)
    indices = np.zeros(0, dtype=np.int32)
    gg = GpuGraph(indptr, indices, np.ones((1, 2), dtype=np.float32))
    res = run_one(gg, np.array([0], dtype=np.int32), (4, 4), 3)
    assert_same(res, gg.oracle.sample_mfg(np.array([0], dtype=np.int32), (4, 4), 3), 2)
    assert res["counts"] == [1, 1, 1, 0, 0, 0]


def test_randomised_small_dense_graphs():
    """Many small dense graphs (few nodes, long rows, fanouts near the node count): almost every
    sample is a duplicate of another, so ownership changes hands repeatedly and pointer chains
    form; both paths, up to 16 batches per launch set, compared with the oracle."""
    rng = np.random.default_rng(2024)
    fan_choices = [(3,), (8, 8), (15, 10, 5), (32, 32), (5, 5, 5, 5), (31, 2), (40, 3), (7, 64), (-1, 6), (100, 100),
                   (12, -1, 4)]
    cases = 0
    for trial in range(36):
        n = int(rng.integers(20, 260))
        avg = int(rng.integers(8, 70))
        adj = random_simple_graph(n, min(avg, n - 1), rng, hub=int(rng.integers(1, n - 1)) if trial % 3 == 0 else None)
        indptr, indices = csr_from_adj(adj)
        m = max(1, len(indices))
        gg = GpuGraph(indptr, indices, rng.standard_normal((n, 3)).astype(np.float32))
        fan = fan_choices[trial % len(fan_choices)]
        G = int(rng.integers(1, 17))
        seeds = [rng.choice(n, size=int(rng.integers(1, min(n, 60))), replace=False).astype(np.int32) for _ in range(G)]
        keys = [int(rng.integers(0, 2**62)) for _ in range(G)]
        wide = any(d < 0 or d > 32 for d in fan)     # the padded fast path sizes its own scratch
        wss = [smfg.workspace_create(gg.g, 64, fan, node_capacity=n, sample_capacity=m if wide else 0)
               for _ in range(G)]
        outs = [smfg.alloc_output(gg.g, 64, fan, node_capacity=n, edge_capacity=[m] * len(fan)) for _ in range(G)]
        for rep in range(2):
            smfg.sample_mfg_many(gg.g, wss, [torch.from_numpy(s).to(DEV) for s in seeds], fan, keys, outs)
            for b in range(G):
                assert_same(fetch(outs[b], len(fan)), gg.oracle.sample_mfg(seeds[b], fan, keys[b]), len(fan))
                cases += 1
    assert cases > 300


def test_graph_validate_names_what_is_broken(tiny):
    """The optional CSR check: a sound graph passes; each planted defect sets its own bit.  The
    check only reads the two arrays inside their stated lengths, so broken contents are safe."""
    assert smfg.graph_validate(tiny[1].g) == 0
    rng = np.random.default_rng(5)
    indptr, indices = csr_from_adj(random_simple_graph(3000, 9, rng, hub=7))
    n, m = len(indptr) - 1, len(indices)

    def flags_of(ip, ix):
        a = torch.from_numpy(np.ascontiguousarray(ip)).to(DEV)
        b = torch.from_numpy(np.ascontiguousarray(ix)).to(DEV)
        return smfg.graph_validate(smfg.graph_create(a, b, None))

    assert flags_of(indptr, indices) == 0
    ip = indptr.copy(); ip[0] = 1
    assert flags_of(ip, indices) & smfg.BAD_INDPTR_START
    ip = indptr.copy(); ip[n] = m - 1                      # last row shrinks: the end no longer matches
    assert flags_of(ip, indices) == smfg.BAD_INDPTR_END
    ip = indptr.copy(); ip[1500] = ip[1499] - 1            # one step backwards in the middle
    assert flags_of(ip, indices) == smfg.BAD_INDPTR_ORDER
    ip = indptr.copy(); ip[2000:] += 1 << 31               # a degree of 2^31 or more
    assert flags_of(ip, indices) == smfg.BAD_INDPTR_ORDER | smfg.BAD_INDPTR_END
    for bad in (-1, n, 2**31 - 1):
        for where in (0, m // 2, m - 1):
            ix = indices.copy(); ix[where] = bad
            assert flags_of(indptr, ix) == smfg.BAD_INDEX_RANGE
    ix = indices.copy(); ix[m - 1] = n - 1                 # the largest valid id
    assert flags_of(indptr, ix) == 0
    # no nodes, no edges
    assert flags_of(np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32)) == 0
    assert flags_of(np.ones(1, dtype=np.int64), np.zeros(0, dtype=np.int32)) == (smfg.BAD_INDPTR_START
                                                                                    | smfg.BAD_INDPTR_END)


def test_gather_rows_never_reads_outside_the_feature_matrix():
    """Row ids outside [0, num_nodes) are served from row 0; the valid rows around them are exact."""
    rng = np.random.default_rng(11)
    n, dim = 500, 24
    indptr = np.zeros(n + 1, dtype=np.int64)
    feat = rng.standard_normal((n, dim)).astype(np.float16)
    gg = GpuGraph(indptr, np.zeros(0, dtype=np.int32), feat)
    ids_np = rng.integers(0, n, size=777).astype(np.int32)
    bad_at = np.array([0, 5, 31, 32, 400, 776])
    ids_np[bad_at] = np.array([-1, n, n + 12345, 2**31 - 1, -2**31, n], dtype=np.int32)
    ids = torch.from_numpy(ids_np).to(DEV)
    cnt = torch.tensor([ids.numel()], dtype=torch.int64, device=DEV)
    out = torch.zeros((ids.numel(), dim), dtype=gg.feat.dtype, device=DEV)
    smfg.gather_rows(gg.g, ids, cnt, ids.numel(), out)
    torch.cuda.synchronize()
    want_ids = ids_np.astype(np.int64)
    want_ids[bad_at] = 0
    assert np.array_equal(out.cpu().numpy().view(np.uint16), feat[want_ids].view(np.uint16))


def test_mean_aggregate_clamps_stray_offsets_and_ids():
    """A block left behind by a failed batch may hold anything: offsets are clamped to the indices
    array and ids outside x read row 0.  The rows that are sound keep their exact means."""
    rng = np.random.default_rng(3)
    n_src, n_dst, dim, m = 40, 6, 8, 20
    x = rng.standard_normal((n_src, dim)).astype(np.float32)
    indptr = np.array([0, 3, 7, 7, 12, 18, 31], dtype=np.int32)        # last row runs past the 20 edges
    indices = rng.integers(0, n_src, size=m).astype(np.int32)
    indices[[1, 8, 13]] = [-5, n_src, 2**31 - 1]                        # stray ids -> row 0
    y = torch.full((n_dst, dim), float("nan"), dtype=torch.float32, device=DEV)
    smfg.mean_aggregate(torch.from_numpy(indptr).to(DEV), torch.from_numpy(indices).to(DEV),
                        torch.tensor([n_dst], dtype=torch.int64, device=DEV), n_dst,
                        torch.from_numpy(x).to(DEV), y)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    ids = indices.astype(np.int64)
    ids[(ids < 0) | (ids >= n_src)] = 0
    for i in range(n_dst):
        a, b = int(indptr[i]), min(int(indptr[i + 1]), m)
        want = x[ids[a:b]].astype(np.float64).mean(axis=0) if b > a else np.zeros(dim)
        assert np.allclose(got[i], want, rtol=0, atol=1e-5), i


def test_blocks_in_consumer_order(tiny):
    """mfg_blocks hands out trimmed views, outermost hop first, whose shapes chain."""
    w, gg, batches = tiny
    seeds = batches[1].to(DEV)
    L = len(w.fanouts)
    ws = smfg.workspace_create(gg.g, seeds.numel(), w.fanouts)
    out = smfg.alloc_output(gg.g, seeds.numel(), w.fanouts)
    smfg.sample_mfg(gg.g, ws, seeds, w.fanouts, 77, out)
    counts = smfg.read_counts(out)
    ref = gg.oracle.sample_mfg(batches[1].numpy(), w.fanouts, 77)
    blocks = smfg.mfg_blocks(out, counts)
    assert len(blocks) == L
    n_src_prev = None
    for j, (indptr, indices, (n_src, n_dst)) in enumerate(blocks):
        h = L - 1 - j
        assert np.array_equal(indptr.cpu().numpy(), ref.indptr[h]) and np.array_equal(indices.cpu().numpy(), ref.indices[h])
        assert indptr.data_ptr() == out.indptr[h].data_ptr()          # a view, not a copy
        assert (n_src, n_dst) == (int(ref.counts[h + 1]), int(ref.counts[h]))
        assert n_src_prev is None or n_src == n_src_prev[1]          # dst of the outer block = src of the next
        n_src_prev = (n_src, n_dst)
    assert blocks[0][2][0] == counts[L] and blocks[-1][2][1] == seeds.numel()


@pytest.mark.parametrize("fanouts", [(-1,), (40, 2)])
def test_mean_aggregate_long_and_empty_rows(fanouts):
    """Blocks of the wide path: a destination with 700 samples next to destinations with none,
    one or a few, so the sums cross many load rounds and the groups of neighbouring destinations
    end at different places."""
    rng = np.random.default_rng(17)
    adj = random_simple_graph(2500, 6, rng, hub=700)
    for v in (10, 11, 500):
        adj[v] = []
    adj = [[u for u in row if u not in (10, 11, 500)] for row in adj]
    indptr, indices = csr_from_adj(adj)
    dim = 64
    feat = (rng.standard_normal((2500, dim)) * 3).astype(np.float16)
    gg = GpuGraph(indptr, indices, feat)
    hub = int(np.argmax(np.diff(indptr)))
    seeds = np.unique(np.concatenate([[10, hub, 11, 500], rng.choice(2500, size=333, replace=False)])).astype(np.int32)
    rng.shuffle(seeds)
    L = len(fanouts)
    m = len(indices)
    ws = smfg.workspace_create(gg.g, len(seeds), fanouts, sample_capacity=m)
    out = smfg.alloc_output(gg.g, len(seeds), fanouts, edge_capacity=[m] * L)
    smfg.sample_mfg(gg.g, ws, torch.from_numpy(seeds).to(DEV), fanouts, 5, out)
    res = fetch(out, L)
    ref = gg.oracle.sample_mfg(seeds, fanouts, 5)
    assert_same(res, ref, L)
    x_ref = ref.features.view(np.float16).reshape(-1, dim)
    h = 0                      # the block of the seeds: its sources are a prefix of the node list
    n_dst = res["n"][h]
    y = torch.full((out.node_capacity, dim), float("nan"), dtype=torch.float32, device=DEV)
    smfg.mean_aggregate(out.indptr[h], out.indices[h], out.counts[h:h + 1], out.indptr[h].numel() - 1, out.features, y)
    torch.cuda.synchronize()
    mean, mag = oracle.mean_aggregate(ref.indptr[h], ref.indices[h], np.ascontiguousarray(x_ref))
    got = y[:n_dst].cpu().numpy().astype(np.float64)
    k = np.diff(ref.indptr[h])
    assert k.max() >= 40 and (k == 0).sum() >= 1
    assert np.isnan(y[n_dst:].cpu().numpy()).all()
    assert (np.abs(got - mean) <= np.maximum(k, 1)[:, None] * 2.0 ** -24 * mag).all()
    assert (got[k == 0] == 0).all()


@pytest.mark.parametrize("dim,out_dims,out_dtype,with_bias", [
    (128, (256, 256, 64), torch.float16, True),      # the shape of the papers workload, 64-row tiles
    (64, (48, 40, 1), torch.float32, False),         # output widths that are no multiple of 32
    (256, (128, 8, 100), torch.float16, True),       # 32-row tiles
    (8, (16, 24, 5), torch.float32, True),           # smallest input width
])
def test_sage_layer_consumer(dim, out_dims, out_dtype, with_bias):
    """Three GraphSAGE layers over the blocks of a sampled batch, outermost hop first, ReLU after all
    but the last (model listing of Appendix C), each compared with the fp64 oracle fed the same
    half inputs.  Bound per output: S (2^-11 + (2 dim + k + 2) 2^-24) for the half rounding of the
    mean and the float sums, plus the rounding of a half result; S = sum of |w| |input| + |bias|."""
    rng = np.random.default_rng(dim + out_dims[0])
    adj = random_simple_graph(4000, 14, rng, hub=700)
    adj[3] = []
    adj = [[u for u in row if u != 3] for row in adj]
    indptr, indices = csr_from_adj(adj)
    feat = (rng.standard_normal((4000, dim)) * 2).astype(np.float16)
    gg = GpuGraph(indptr, indices, feat)
    seeds = np.concatenate([[3], rng.choice(np.arange(4, 4000), size=700, replace=False)]).astype(np.int32)
    fan = (7, 5, 3)
    ws = smfg.workspace_create(gg.g, len(seeds), fan)
    out = smfg.alloc_output(gg.g, len(seeds), fan)
    smfg.sample_mfg(gg.g, ws, torch.from_numpy(seeds).to(DEV), fan, 31, out)
    res = fetch(out, 3)
    ref = gg.oracle.sample_mfg(seeds, fan, 31)
    assert_same(res, ref, 3)
    x_gpu = out.features
    x_ref = ref.features.view(np.float16).reshape(-1, dim)
    d_in = dim
    for layer, h in enumerate((2, 1, 0)):
        d_out = out_dims[layer]
        relu = layer < 2
        w = (rng.standard_normal((d_out, 2 * d_in)) / np.sqrt(d_in)).astype(np.float16)
        b = (rng.standard_normal(d_out) * 0.5).astype(np.float32) if with_bias else None
        n_dst = res["n"][h]
        y = torch.full((out.node_capacity, d_out), float("nan"), dtype=out_dtype, device=DEV)
        smfg.sage_layer(out.indptr[h], out.indices[h], out.counts[h:h + 1], out.indptr[h].numel() - 1, x_gpu,
                        smfg.sage_pack_weights(torch.from_numpy(w).to(DEV)),
                        torch.from_numpy(b).to(DEV) if b is not None else None, relu, y)
        torch.cuda.synchronize()
        want, mag = oracle.sage_layer(ref.indptr[h], ref.indices[h], np.ascontiguousarray(x_ref),
                                      w.astype(np.float64), None if b is None else b.astype(np.float64), relu)
        got = y[:n_dst].float().cpu().numpy().astype(np.float64)
        assert np.isnan(y[n_dst:].float().cpu().numpy()).all()         # nothing written past n_dst
        k = np.diff(ref.indptr[h]).astype(np.float64)
        tol = mag * (2.0 ** -11 + (2 * d_in + k[:, None] + 2) * 2.0 ** -24)
        if out_dtype == torch.float16:
            tol = tol + np.abs(want) * 2.0 ** -11 + 2.0 ** -24
        assert (np.abs(got - want) <= tol).all(), f"layer {layer}: worst {np.max(np.abs(got - want) / tol)}"
        if relu:
            assert (got >= 0).all() and (got == 0).any() and (got > 0).any()
        if layer == 0 and d_out > 1:
            # the bound is tight enough to tell a wrong layer: an oracle with the two halves of W
            # exchanged (a mistake planted on the CPU side) is far outside it
            w_bad = np.concatenate([w[:, d_in:], w[:, :d_in]], axis=1).astype(np.float64)
            bad, _ = oracle.sage_layer(ref.indptr[h], ref.indices[h], np.ascontiguousarray(x_ref), w_bad,
                                       None if b is None else b.astype(np.float64), relu)
            assert (np.abs(got - bad) > 10 * tol).mean() > 0.25
        # the next layer continues from the GPU's output as halfs on both sides
        x_gpu = y[:n_dst].to(torch.float16).contiguous()
        x_ref = x_gpu.cpu().numpy()
        d_in = d_out if d_out % 8 == 0 and d_out >= 8 else None
        if d_in is None:
            break


def test_sage_layer_argument_errors_and_empty_block():
    x = torch.zeros((16, 16), dtype=torch.float16, device=DEV)
    indptr = torch.zeros(17, dtype=torch.int32, device=DEV)
    indices = torch.zeros(4, dtype=torch.int32, device=DEV)
    one = torch.tensor([16], dtype=torch.int64, device=DEV)
    wp = smfg.sage_pack_weights(torch.ones((8, 32), dtype=torch.float16, device=DEV))
    out = torch.full((16, 8), float("nan"), dtype=torch.float32, device=DEV)
    with pytest.raises(smfg.SmfgError) as ei:                      # a width that is no multiple of 8
        smfg.sage_pack_weights(torch.ones((8, 24), dtype=torch.float16, device=DEV))
    assert ei.value.code == smfg.ERR_INVALID_ARG
    L = smfg.lib()
    import ctypes
    vp = ctypes.c_void_p
    args = lambda dim, out_eb: (vp(indptr.data_ptr()), vp(indices.data_ptr()), 4, vp(one.data_ptr()), 16, vp(x.data_ptr()),
                                16, dim, vp(wp.data.data_ptr()), None, 8, 0, vp(out.data_ptr()), out_eb, None)
    assert L.smfg_sage_layer(*args(12, 4)) == smfg.ERR_INVALID_ARG
    assert L.smfg_sage_layer(*args(16, 3)) == smfg.ERR_INVALID_ARG
    assert L.smfg_sage_layer(*((None,) + args(16, 4)[1:])) == smfg.ERR_NULL_PTR
    # all destinations empty: the output is the own-row half of the product, the mean half is zero
    x.copy_(torch.arange(16, device=DEV).view(16, 1).expand(16, 16).to(torch.float16))
    smfg.sage_layer(indptr, indices, one, 16, x, wp, None, False, out)
    torch.cuda.synchronize()
    assert torch.equal(out, (torch.arange(16, device=DEV).float() * 16).view(16, 1).expand(16, 8))
    # zero destinations: nothing is written
    out.fill_(float("nan"))
    smfg.sage_layer(indptr, indices, torch.zeros(1, dtype=torch.int64, device=DEV), 16, x, wp, None, False, out)
    torch.cuda.synchronize()
    assert torch.isnan(out).all()

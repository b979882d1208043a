#!/usr/bin/env python3
"""Benchmark of the mini-batch preparation path on one MI355X.

A "step" is one prepared mini-batch: neighbour sampling over all hops, MFG block construction and
the feature gather for one batch of seeds, everything resident in HBM.  Several batches share each
set of launches (`--batches-per-call`), which is how independent batches are kept in flight.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload papers]

Prints one JSON line (metric: sampled mini-batches/s) with a `roofline` object for the dominant
kernel (the feature gather, HBM bound) and a `cpu_baseline` object (the CPU oracle timed on the
host cores on a bounded sample of the same batches).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak

# HBM bytes per k_gather launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# command (profiles/*_kernel_trace_and_hbm_traffic.txt), scaled by what the same counters read
# for the identity copy of known size; keyed by (workload, batches per launch).
MEASURED_GATHER_TRAFFIC_BYTES = {("papers", 8): 3.610e9, ("large", 8): 2.414e9}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(n, e, row_bytes):
    """Compulsory reads + writes of one batch: seeds, two int64 indptr words per destination, the
    chosen neighbour ids, feature rows in; block indptr / indices, node ids, feature rows out."""
    L = len(e)
    reads = 4 * n[0] + sum(16 * n[h] + 4 * e[h] for h in range(L)) + row_bytes * n[L]
    writes = sum(4 * (n[h] + 1) + 4 * e[h] for h in range(L)) + 4 * n[L] + row_bytes * n[L]
    return reads + writes


def cpu_baseline(w, graph, feat, batches, keys, budget_s, threads, gpu_check):
    """Times the oracle as it stands on `threads` host threads, each with its own scratch map,
    over a bounded number of the same batches; also checks the first batches against the GPU."""
    import numpy as np
    import oracle
    t0 = time.time()
    h_indptr = graph.indptr.cpu().numpy()
    h_indices = graph.indices.cpu().numpy()
    h_feat = feat.cpu().numpy()
    h_feat = h_feat.view(np.uint8).reshape(h_feat.shape[0], -1)
    log(f"[cpu] host copies of graph and features: {time.time() - t0:.1f}s")
    base = oracle.Oracle(h_indptr, h_indices, h_feat)
    h_batches = [b.cpu().numpy() for b in batches]

    t0 = time.time()
    ref0 = base.sample_mfg(h_batches[0], w.fanouts, keys[0])
    t_one = time.time() - t0
    # bit-for-bit comparison of the first batches with the GPU (bounded to a few seconds of oracle time)
    n_check = max(1, min(8, len(h_batches), int(4.0 / max(t_one, 1e-3))))
    parity = gpu_check(ref0, 0)
    for i in range(1, n_check):
        parity = parity and gpu_check(base.sample_mfg(h_batches[i], w.fanouts, keys[i]), i)
    per_thread = max(1, min(int(budget_s / max(t_one, 1e-4)), 4096))
    n_total = per_thread * threads
    workers = [base] + [base.clone_scratch() for _ in range(threads - 1)]
    edges = [0] * threads

    def run(t):
        for q in range(per_thread):
            i = (t * per_thread + q) % len(h_batches)
            r = workers[t].sample_mfg(h_batches[i], w.fanouts, keys[i])
            edges[t] += sum(r.num_edges)

    ths = [threading.Thread(target=run, args=(t,)) for t in range(threads)]
    t0 = time.time()
    for t in ths:
        t.start()
    for t in ths:
        t.join()
    dt = time.time() - t0
    return {
        "value": n_total / dt, "unit": "batches/s", "cores": threads, "kind": "oracle",
        "sample": f"{n_total} batches of workload '{w.name}' ({per_thread} per thread, {threads} threads, "
                  f"one batch on one thread: {t_one * 1e3:.1f} ms)",
        "sampled_edges_per_s": sum(edges) / dt, "parity_vs_gpu": parity, "parity_batches": n_check,
        "one_thread_batches_per_s": 1.0 / t_one,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="papers")
    ap.add_argument("--batches-per-call", type=int, default=8)
    ap.add_argument("--streams", type=int, default=1,
                    help="launch sets alternate over this many HIP streams, each with its own workspaces")
    ap.add_argument("--pipeline", type=int, default=1,
                    help="1: gather of launch set i runs on a second stream while set i+1 is sampled (two "
                         "buffer sets); 0: every launch set runs start to end on one stream (see --streams)")
    ap.add_argument("--feat-dim", type=int, default=0, help="experiment: override the feature width")
    ap.add_argument("--depth", type=int, default=2, help="buffer sets of the pipelined run")
    ap.add_argument("--sample-streams", type=int, default=1,
                    help="pipelined run: launch sets alternate over this many sampling streams (needs depth > streams)")
    ap.add_argument("--row-stride", type=int, default=0,
                    help="experiment: feature row stride in bytes (>= row bytes; 0 = dense rows)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="oracle time budget per host thread")
    ap.add_argument("--cpu-threads", type=int, default=0, help="0 = min(16, cores available)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--stages", action="store_true", help="extra untimed pass with every launch timed")
    ap.add_argument("--consume", action="store_true",
                    help="extra untimed-for-value pass: a consumer stream runs the mean aggregation of all hops "
                         "on every prepared batch while the next launch set is being prepared")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run plain copies of known size (1 GiB in, 1 GiB out) for counter calibration")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (batches are independent, so more GPUs would each "
            "take their own batches of a replicated graph); run with --gpus 1")
        sys.exit(2)

    import torch
    from paper_2110_08450_amd import binding as smfg, synth

    w = synth.WORKLOADS[args.workload]
    if args.feat_dim:
        import dataclasses
        w = dataclasses.replace(w, feat_dim=args.feat_dim)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    t0 = time.time()
    graph = synth.make_graph(w, device=dev)
    torch.cuda.synchronize()
    log(f"[gen] graph '{w.name}': {graph.num_nodes} nodes, {graph.num_edges} directed edges, {time.time() - t0:.1f}s")
    t0 = time.time()
    feat = synth.make_features(w, device=dev)
    if args.row_stride:
        eb = feat.element_size()
        assert args.row_stride % eb == 0 and args.row_stride >= feat.shape[1] * eb
        padded = torch.zeros((feat.shape[0], args.row_stride // eb), dtype=feat.dtype, device=dev)
        padded[:, :feat.shape[1]] = feat
        feat = padded[:, :feat.shape[1]]      # same values, rows args.row_stride bytes apart
        del padded
    batches = synth.make_seed_batches(w, device=dev)
    torch.cuda.synchronize()
    log(f"[gen] features {tuple(feat.shape)} {feat.dtype}, {len(batches)} seed batches, {time.time() - t0:.1f}s")
    torch.cuda.empty_cache()

    G = max(1, min(args.batches_per_call, smfg.MAX_BATCHES))
    L = len(w.fanouts)
    g = smfg.graph_create(graph.indptr, graph.indices, feat)
    pipe = None
    wide = any(d < 0 or d > smfg.MAX_FANOUT for d in w.fanouts)
    scap = min(graph.num_edges, (1 << 30) - 1) if wide else 0   # a hop never has more samples than the graph has edges
    if args.pipeline:
        from paper_2110_08450_amd.pipeline import BatchPipeline
        pipe = BatchPipeline(g, w.fanouts, w.batch_size, batches_per_set=G, sample_capacity=scap,
                             depth=max(2, args.depth, args.sample_streams + 1), sample_streams=args.sample_streams)
        S, streams, wss, outs = 2, [pipe.s_sample, pipe.s_gather], pipe.wss, pipe.outs
    else:
        S = max(1, args.streams)
        streams = [torch.cuda.Stream() for _ in range(S)]
        wss = [[smfg.workspace_create(g, w.batch_size, w.fanouts, 0, scap) for _ in range(G)] for _ in range(S)]
        outs = [[smfg.alloc_output(g, w.batch_size, w.fanouts) for _ in range(G)] for _ in range(S)]
    row_bytes = g.row_bytes

    K = max(1, args.steps)      # exactly K timed batches; the last launch set may be partial
    W = max(0, args.warmup)
    keys = [synth.batch_rng_key(w, i) for i in range(len(batches))]
    counts_all = torch.zeros((K + W, 2 * L + 2), dtype=torch.int64, device=dev)
    stride = counts_all.stride(0) * 8

    last_call = {}   # buffer set -> (first batch index, batches) of the last launch set that used it
    sets_issued = [0]

    def run_pipelined(first, n):
        for c in range(first, first + n, G):
            k = min(G, first + n - c)
            q = sets_issued[0] % pipe.depth
            sets_issued[0] += 1
            last_call[q] = (c, k)
            idx = [(c + b) % len(batches) for b in range(k)]

            def point_counts(os_, c=c):
                for b, o in enumerate(os_):
                    o.c.counts = counts_all.data_ptr() + (c + b) * stride
            pipe.issue(q, [batches[i] for i in idx], [keys[i] for i in idx], before_launch=point_counts)

    def run_calls(first, n):
        if args.pipeline:
            return run_pipelined(first, n)
        for c in range(first, first + n, G):
            k = min(G, first + n - c)
            q = sets_issued[0] % S
            sets_issued[0] += 1
            last_call[q] = (c, k)
            idx = [(c + b) % len(batches) for b in range(k)]
            for b in range(k):
                outs[q][b].c.counts = counts_all.data_ptr() + (c + b) * stride
            smfg.sample_mfg_many(g, wss[q][:k], [batches[i] for i in idx], w.fanouts, [keys[i] for i in idx],
                                 outs[q][:k], stream=streams[q])

    run_calls(0, W)
    torch.cuda.synchronize()
    smfg.profile_begin(1, K // G + 2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_calls(W, K)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stages = smfg.profile_end()

    cnt = counts_all[W:].cpu().tolist()
    assert all(c[2 * L + 1] == 0 for c in cnt), "a timed batch reported a device status"
    n_final = sum(c[L] for c in cnt)
    edges = sum(sum(c[L + 1:2 * L + 1]) for c in cnt)
    alg = sum(algorithmic_bytes(c[:L + 1], c[L + 1:2 * L + 1], row_bytes) for c in cnt)
    gather_ms, gather_launches = stages["gather"]
    gather_bytes = 2 * row_bytes * n_final
    gather_gbs = gather_bytes / (gather_ms * 1e-3) / 1e9 if gather_ms > 0 else 0.0

    # The same gather launches once more with nothing else on the chip (the buffers of the last
    # launch sets are still in place): the kernel's own rate, next to the overlapped one above.
    smfg.profile_begin(1, 16)
    rows_alone = 0
    timed_sets = [q for q, (c, k) in last_call.items() if c >= W]
    for rep in range(6):
        q = timed_sets[rep % len(timed_sets)]
        c0, k = last_call[q][0] - W, last_call[q][1]
        smfg.gather_many(g, outs[q][:k], stream=streams[0])
        rows_alone += sum(c[L] for c in cnt[c0:c0 + k])
    torch.cuda.synchronize()
    alone_ms, alone_launches = smfg.profile_end()["gather"]
    alone_gbs = 2 * row_bytes * rows_alone / (alone_ms * 1e-3) / 1e9 if alone_ms > 0 else 0.0

    # What a plain device-to-device copy reaches on this machine (1 GiB in, 1 GiB out, nothing else
    # running): the achievable ceiling next to the published peak.
    copy_gbs = 0.0
    try:
        a = torch.empty(1 << 28, dtype=torch.int32, device=dev).fill_(1)
        b = torch.empty_like(a)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        b.copy_(a)
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(8):
            b.copy_(a)
        ev[1].record()
        torch.cuda.synchronize()
        copy_gbs = 8 * 2 * (1 << 30) / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
        del a, b
    except torch.OutOfMemoryError:
        pass

    # A consumer of the prepared batches (not part of the timed path): GraphSAGE mean aggregation
    # over the outermost block of the batches of the last launch set.
    consumer = None
    if feat.dtype in (torch.float16, torch.float32):
        q = max(timed_sets, key=lambda t: last_call[t][1])
        c0, k_set = last_call[q][0] - W, last_call[q][1]
        agg_out = torch.empty((outs[q][0].node_capacity, w.feat_dim), dtype=torch.float32, device=dev)
        smfg.profile_begin(2, 4 * G)
        agg_bytes = 0
        for rep in range(2):
            for b in range(k_set):
                o, c = outs[q][b], cnt[c0 + b]
                o.c.counts = counts_all.data_ptr() + (W + c0 + b) * stride
                n_dst, e_last = c[L - 1], c[2 * L]
                cview = counts_all[W + c0 + b]
                smfg.mean_aggregate(o.indptr[L - 1], o.indices[L - 1], cview[L - 1:L], o.indptr[L - 1].numel() - 1, o.features,
                                    agg_out, stream=streams[0])
                agg_bytes += e_last * row_bytes + 4 * e_last + 4 * (n_dst + 1) + 4 * w.feat_dim * n_dst
        torch.cuda.synchronize()
        agg_ms, agg_n = smfg.profile_end()["mean_aggregate"]
        consumer = {"kernel": "k_mean_aggregate", "block": f"hop {L - 1}", "launches": agg_n,
                    "avg_launch_ms": agg_ms / max(1, agg_n),
                    "achieved": agg_bytes / (agg_ms * 1e-3) / 1e9 if agg_ms > 0 else 0.0, "unit": "GB/s",
                    "frac": agg_bytes / (agg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if agg_ms > 0 else 0.0}
        del agg_out
        # the same block through one whole GraphSAGE layer on the matrix cores (half in, 256 half out)
        if feat.dtype == torch.float16 and w.feat_dim % 8 == 0 and w.feat_dim <= 256:
            hid = 256
            lw = smfg.sage_pack_weights((torch.randn((hid, 2 * w.feat_dim), device=dev) / w.feat_dim ** 0.5)
                                        .to(torch.float16))
            lb = torch.zeros(hid, dtype=torch.float32, device=dev)
            lay_out = torch.empty((outs[q][0].indptr[L - 1].numel() - 1, hid), dtype=torch.float16, device=dev)
            smfg.profile_begin(2, 4 * G)
            lay_bytes = lay_flops = 0
            for rep in range(2):
                for b in range(k_set):
                    o, c = outs[q][b], cnt[c0 + b]
                    n_dst, e_last = c[L - 1], c[2 * L]
                    cview = counts_all[W + c0 + b]
                    smfg.sage_layer(o.indptr[L - 1], o.indices[L - 1], cview[L - 1:L], o.indptr[L - 1].numel() - 1,
                                    o.features, lw, lb, True, lay_out, stream=streams[0])
                    lay_bytes += (e_last + n_dst) * row_bytes + 4 * e_last + 4 * (n_dst + 1) + 2 * hid * n_dst
                    lay_flops += 2 * n_dst * 2 * w.feat_dim * hid
            torch.cuda.synchronize()
            lay_ms, lay_n = smfg.profile_end()["sage_layer"]
            consumer["layer"] = {"kernel": "k_sage_layer", "block": f"hop {L - 1}", "out_dim": hid, "launches": lay_n,
                                 "avg_launch_ms": lay_ms / max(1, lay_n),
                                 "achieved": lay_bytes / (lay_ms * 1e-3) / 1e9 if lay_ms > 0 else 0.0, "unit": "GB/s",
                                 "frac": lay_bytes / (lay_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if lay_ms > 0 else 0.0,
                                 "TFLOPs": lay_flops / (lay_ms * 1e-3) / 1e12 if lay_ms > 0 else 0.0}
            del lay_out, lw, lb

    result = {
        "metric": "sampled mini-batches/sec (MFG build + feature gather)",
        "value": K / dt, "unit": "batches/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": dt / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.num_nodes} nodes, {graph.num_edges} directed edges, "
                               f"features {w.feat_dim}x{str(w.feat_dtype).split('.')[-1]}, fanouts {list(w.fanouts)}, "
                               f"batch {w.batch_size}", "batches_per_call": G, "streams": S, "pipeline": bool(args.pipeline),
                   "row_stride_bytes": int(feat.stride(0) * feat.element_size()),
                   "mean_nodes_per_batch": n_final / K, "mean_edges_per_batch": edges / K},
        "sampled_edges_per_s": edges / dt,
        "gather_GBps": gather_gbs,
        "path_algorithmic_GBps": alg / dt / 1e9,
        "path_frac_of_hbm_peak": alg / dt / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "k_gather", "achieved": gather_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": gather_gbs / HBM_PEAK_GBS,
                     "traffic": None if (args.feat_dim or args.row_stride) else MEASURED_GATHER_TRAFFIC_BYTES.get((w.name, G)), "traffic_unit": "bytes per launch",
                     "avg_launch_ms": gather_ms / max(1, gather_launches),
                     "note": "achieved is measured inside the timed region, where (with --pipeline 1) the gather "
                             "shares the chip with the sampling kernels of the next launch set; alone_* is the same "
                             "launch repeated right after with nothing else running",
                     "alone_achieved": alone_gbs, "alone_frac": alone_gbs / HBM_PEAK_GBS,
                     "alone_avg_launch_ms": alone_ms / max(1, alone_launches),
                     "algorithmic_bytes_per_launch": gather_bytes / max(1, gather_launches),
                     "device_copy_GBps": copy_gbs,
                     "alone_frac_of_device_copy": alone_gbs / copy_gbs if copy_gbs > 0 else None,
                     "read_only_half_GBps": gather_gbs / 2},
    }

    if consumer is not None:
        result["consumer"] = consumer

    if args.consume and pipe is not None and feat.dtype in (torch.float16, torch.float32):
        # Preparation hidden behind a consumer (the paper's pipelining, section 4.3, with everything on
        # one GPU): the consumer aggregates hop L-1 .. 0 of each batch on the current stream.
        n_b = min(K, 1024)
        idx = [i % len(batches) for i in range(n_b)]
        cap = pipe.outs[0][0].node_capacity
        use_layers = feat.dtype == torch.float16 and w.feat_dim % 8 == 0 and w.feat_dim <= 256
        if use_layers:
            # a GraphSAGE model forward (Appendix C): hidden width 256, 172 classes, ReLU between layers
            widths = [w.feat_dim] + [256] * (L - 1) + [172]
            lws = [smfg.sage_pack_weights((torch.randn((widths[i + 1], 2 * widths[i]), device=dev)
                                           / widths[i] ** 0.5).to(torch.float16)) for i in range(L)]
            lbs = [torch.zeros(widths[i + 1], dtype=torch.float32, device=dev) for i in range(L)]
            bufs = [torch.empty((cap, widths[i + 1]), dtype=torch.float16, device=dev) for i in range(L)]
            what = f"GraphSAGE forward, widths {widths}, half activations"

            def consume(o):
                x = o.features
                for i, h in enumerate(range(L - 1, -1, -1)):
                    smfg.sage_layer(o.indptr[h], o.indices[h], o.counts[h:h + 1], o.indptr[h].numel() - 1, x,
                                    lws[i], lbs[i], i < L - 1, bufs[i])
                    x = bufs[i]
        else:
            bufs = [torch.empty((cap, w.feat_dim), dtype=torch.float32, device=dev) for _ in range(2)]
            what = "mean aggregation of hops L-1..0 (fp32 out)"

            def consume(o):
                x = o.features
                for h in range(L - 1, -1, -1):
                    y = bufs[h % 2]
                    smfg.mean_aggregate(o.indptr[h], o.indices[h], o.counts[h:h + 1], o.indptr[h].numel() - 1, x, y)
                    x = y

        def one_pass(with_consumer):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for outs_ in pipe.run([batches[i] for i in idx], [keys[i] for i in idx]):
                if with_consumer:
                    for o in outs_:
                        consume(o)
            torch.cuda.synchronize()
            return time.perf_counter() - t0
        for o_set in pipe.outs:           # each output needs its own counts buffer again
            for o in o_set:
                o.c.counts = o.counts.data_ptr()
        one_pass(True)
        t_prep = one_pass(False)
        t_both = one_pass(True)
        # the consumer alone, on the batches of the last set left in the buffers
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 8
        for _ in range(reps):
            for o in pipe.outs[0]:
                consume(o)
        torch.cuda.synchronize()
        t_cons = (time.perf_counter() - t0) / (reps * len(pipe.outs[0]))
        result["with_consumer"] = {"batches": n_b, "prepare_only_ms_per_batch": t_prep / n_b * 1e3,
                                   "consumer_only_ms_per_batch": t_cons * 1e3,
                                   "prepare_and_consume_ms_per_batch": t_both / n_b * 1e3,
                                   "consumer": what}

    if args.stages:
        smfg.profile_begin(2, 64 * (K // G + 2))
        run_calls(W, K)
        st = smfg.profile_end()
        result["stage_ms_per_batch"] = {s: ms / K for s, (ms, _) in st.items()}

    if args.calibrate:
        a = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                       # plain device copy: 1 GiB read, 1 GiB written
        rows = min((1 << 30) // row_bytes, graph.num_nodes)   # identity ids must stay inside the feature table
        ids = torch.arange(rows, dtype=torch.int32, device=dev)
        nrows = torch.tensor([rows], dtype=torch.int64, device=dev)
        dst = b.view(torch.uint8)[:rows * row_bytes].view(feat.dtype).view(rows, -1)
        smfg.gather_rows(g, ids, nrows, rows, dst)   # identity gather: rows * row_bytes in and out
        torch.cuda.synchronize()
        log(f"[calibrate] torch copy 1 GiB; identity gather of {rows} rows x {row_bytes} B")
        del a, b

    if not args.no_cpu:
        import numpy as np

        def gpu_check(ref, i):
            o = outs[0][0]
            o.c.counts = counts_all.data_ptr()
            smfg.sample_mfg(g, wss[0][0], batches[i], w.fanouts, keys[i], o)
            c = smfg.read_counts(o)
            n, e = c[:L + 1], c[L + 1:2 * L + 1]
            ok = c == [int(x) for x in ref.counts]
            ok = ok and np.array_equal(o.node_ids[:n[L]].cpu().numpy(), ref.node_ids)
            for h in range(L):
                ok = ok and np.array_equal(o.indptr[h][:n[h] + 1].cpu().numpy(), ref.indptr[h])
                ok = ok and np.array_equal(o.indices[h][:e[h]].cpu().numpy(), ref.indices[h])
            got = o.features[:n[L]].cpu().numpy().view(np.uint8).reshape(n[L], row_bytes)
            return bool(ok and np.array_equal(got, ref.features))

        threads = args.cpu_threads or min(16, len(os.sched_getaffinity(0)))
        result["cpu_baseline"] = cpu_baseline(w, graph, feat, batches, keys, args.cpu_seconds, threads, gpu_check)

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()

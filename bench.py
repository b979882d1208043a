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

# Launch configuration per workload: (batches per launch set, sampling streams, buffer sets).
# Small batches are bound by the latency of the chain of short kernels, so they take more batches
# per set and two sampling streams; the largest batches fill the chip one at a time.
LAUNCH_CONFIG = {"tiny": (4, 1, 2), "mid": (16, 2, 3), "large": (8, 2, 3), "papers": (8, 1, 2),
                 "papers_infer": (1, 2, 3), "large_wide": (4, 2, 3), "large_all": (4, 2, 3)}
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")


def source_hash():
    """sha256 over the library's sources (kernels, host side, header) without their comments and
    blank space: names the code a stored counter figure was measured on."""
    import hashlib
    import re
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2110_08450_amd", "csrc")
    files = sorted(os.path.join(csrc, f) for f in os.listdir(csrc)) + [os.path.join(ROOT, "include", "smfg.h")]
    for f in files:
        text = open(f, "r", encoding="utf-8").read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)   # no string literal of these files holds a comment mark
        text = re.sub(r"//[^\n]*", " ", text)
        h.update(os.path.basename(f).encode())
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:16]


def stored_traffic(workload, batches_per_call):
    """HBM bytes per k_gather launch from the two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of
    this command, as `bench.py --traffic-from` stored them in profiles/traffic.json; None with a
    note if there is no entry, or if it was measured on other sources than the ones present."""
    try:
        table = json.load(open(TRAFFIC_JSON))
    except (OSError, ValueError):
        return None, "no profiles/traffic.json"
    e = table.get(f"{workload}/{batches_per_call}")
    if e is None:
        return None, f"profiles/traffic.json has no entry for {workload}/{batches_per_call}"
    if e.get("source_hash") != source_hash():
        return None, (f"profiles/traffic.json entry for {workload}/{batches_per_call} was measured on sources "
                      f"{e.get('source_hash')}, present sources are {source_hash()}: not reported")
    return e["gather_bytes_per_row"], (f"stored figure from rocprofv3 --pmc runs of this command on these sources "
                                          f"(FETCH_SIZE x {e['fetch_scale']:.3f} + WRITE_SIZE x {e['write_scale']:.3f}, "
                                          f"scales from the identity copy of known size)")


def traffic_from(fetch_csv, write_csv, bench_json):
    """Reads the counter_collection csv files of `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE`
    runs of `bench.py --calibrate ...` and the JSON line one of those runs printed, scales both
    counters by what they read for the identity gather of known size (k_gather_plain, launched by
    --calibrate) and stores the k_gather figure per gathered row."""
    line = [ln for ln in open(bench_json) if ln.startswith('{"metric"')][-1]
    res = json.loads(line)
    workload = res["config"]["workload"].split(":")[0]
    batches_per_call = res["config"]["batches_per_call"]
    rows_per_launch = res["config"]["mean_nodes_per_batch"] * batches_per_call
    import csv
    import re

    def per_kernel(path, counter):
        acc = {}
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != counter:
                continue
            m = re.search(r"(k_gather_plain|k_gather)\b", r["Kernel_Name"])
            if m:
                acc.setdefault(m.group(1), []).append((float(r["Counter_Value"]), int(r["Grid_Size"])))
        return acc
    fe, wr = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    # the identity gather: grid = ceil(rows / rows per block) blocks of 256 threads (the library copies 64 rows
    # per block when a row has fewer than 256 bytes, else 32), rows x row_bytes in and out (+ 4 B ids in)
    import torch  # noqa: F401  (only for the workload table's dtypes)
    from paper_2110_08450_amd import synth
    w = synth.WORKLOADS[workload]
    row_bytes = w.feat_dim * (2 if "16" in str(w.feat_dtype) else 4)
    (f_plain, grid), (w_plain, _) = fe["k_gather_plain"][0], wr["k_gather_plain"][0]
    rows = min((1 << 30) // row_bytes, w.num_nodes)
    per_block = 64 if row_bytes < 256 else 32
    assert (rows + per_block - 1) // per_block * 256 == grid, "the calibration launch is not the identity gather this expects"
    fetch_scale = (rows * (row_bytes + 4) / 1024.0) / f_plain
    write_scale = (rows * row_bytes / 1024.0) / w_plain
    # timed-region launches only: the largest grids are the full launch sets
    full = max(g for _, g in fe["k_gather"])
    f_mean = sum(v for v, g in fe["k_gather"] if g == full) / sum(1 for _, g in fe["k_gather"] if g == full)
    w_mean = sum(v for v, g in wr["k_gather"] if g == full) / sum(1 for _, g in wr["k_gather"] if g == full)
    try:
        table = json.load(open(TRAFFIC_JSON))
    except (OSError, ValueError):
        table = {}
    table[f"{workload}/{batches_per_call}"] = {
        "gather_bytes_per_row": (f_mean * fetch_scale + w_mean * write_scale) * 1024.0 / rows_per_launch,
        "rows_per_full_launch": rows_per_launch,
        "fetch_KiB": f_mean, "write_KiB": w_mean, "fetch_scale": fetch_scale, "write_scale": write_scale,
        "source_hash": source_hash()}
    json.dump(table, open(TRAFFIC_JSON, "w"), indent=1, sort_keys=True)
    print(json.dumps(table[f"{workload}/{batches_per_call}"]))


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
    ap.add_argument("--batches-per-call", type=int, default=0,
                    help="batches per launch set (0 = the workload's entry in LAUNCH_CONFIG, else 8)")
    ap.add_argument("--streams", type=int, default=1,
                    help="launch sets alternate over this many HIP streams, each with its own workspaces")
    ap.add_argument("--pipeline", type=int, default=1,
                    help="1: gather of launch set i runs on a second stream while set i+1 is sampled (two "
                         "buffer sets); 0: every launch set runs start to end on one stream (see --streams)")
    ap.add_argument("--feat-dim", type=int, default=0, help="experiment: override the feature width")
    ap.add_argument("--depth", type=int, default=0, help="buffer sets of the pipelined run (0 = LAUNCH_CONFIG, else 2)")
    ap.add_argument("--sample-streams", type=int, default=0,
                    help="pipelined run: launch sets alternate over this many sampling streams (needs depth > streams; 0 = LAUNCH_CONFIG, else 1)")
    ap.add_argument("--row-stride", type=int, default=0,
                    help="experiment: feature row stride in bytes (>= row bytes; 0 = dense rows)")
    ap.add_argument("--passes", type=int, default=0,
                    help="timed passes of --steps batches each (0 = at least 5, more until about 0.6 s are timed)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="oracle time budget per host thread")
    ap.add_argument("--cpu-threads", type=int, default=0,
                    help="0 = the CPU share the harness reports (OMP_NUM_THREADS if set, else the affinity mask)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--stages", action="store_true", help="extra untimed pass with every launch timed")
    ap.add_argument("--consume", action="store_true",
                    help="extra untimed-for-value pass: a consumer stream runs the mean aggregation of all hops "
                         "on every prepared batch while the next launch set is being prepared")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run plain copies of known size (1 GiB in, 1 GiB out) for counter calibration")
    ap.add_argument("--traffic-from", nargs=3, metavar=("FETCH_CSV", "WRITE_CSV", "BENCH_LOG"),
                    help="no benchmark: store the k_gather HBM traffic of two rocprofv3 --pmc runs (FETCH_SIZE, "
                         "WRITE_SIZE counter_collection csv files) of `bench.py --calibrate` and the log holding "
                         "that run's JSON line into profiles/traffic.json")
    args = ap.parse_args()
    if args.traffic_from:
        traffic_from(*args.traffic_from)
        return
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

    cfg = LAUNCH_CONFIG.get(w.name, (8, 1, 2))
    args.batches_per_call = args.batches_per_call or cfg[0]
    args.sample_streams = args.sample_streams or cfg[1]
    args.depth = args.depth or max(cfg[2], args.sample_streams + 1)
    G = max(1, min(args.batches_per_call, smfg.MAX_BATCHES))
    L = len(w.fanouts)
    K = max(1, args.steps)      # a pass = exactly K batches
    W = max(0, args.warmup)

    def set_bounds(first, n):
        """Cuts batches first .. first+n-1 into launch sets of equal size (give or take one batch):
        G batches each, or more - up to the library's limit of 16 - when n is not a multiple of G,
        because a short last set would run against a full one in the other stream and lose the overlap."""
        if n <= 0:
            return [first]
        n_sets = max(1, (n + smfg.MAX_BATCHES - 1) // smfg.MAX_BATCHES, n // G)
        return [first + (n * i) // n_sets for i in range(n_sets + 1)]

    def largest_set(n):
        b = set_bounds(0, n)
        return max([y - x for x, y in zip(b[:-1], b[1:])] + [0])
    g = smfg.graph_create(graph.indptr, graph.indices, feat)
    pipe = None
    wide = any(d < 0 or d > smfg.MAX_FANOUT for d in w.fanouts)
    scap = min(graph.num_edges, (1 << 30) - 1) if wide else 0   # a hop never has more samples than the graph has edges
    if args.pipeline:
        from paper_2110_08450_amd.pipeline import BatchPipeline
        depth_ = max(2, args.depth, args.sample_streams + 1)
        Gbuf = max(G, largest_set(K), largest_set(max(W, depth_ * G)))     # batches a buffer set must hold
        pipe = BatchPipeline(g, w.fanouts, w.batch_size, batches_per_set=Gbuf, sample_capacity=scap,
                             depth=depth_, sample_streams=args.sample_streams)
        streams, wss, outs = pipe.s_samples + [pipe.s_gather], pipe.wss, pipe.outs
        S = len(streams)
    else:
        S = max(1, args.streams)
        Gbuf = max(G, largest_set(K), largest_set(max(W, S * G)))
        streams = [torch.cuda.Stream() for _ in range(S)]
        wss = [[smfg.workspace_create(g, w.batch_size, w.fanouts, 0, scap) for _ in range(Gbuf)] for _ in range(S)]
        outs = [[smfg.alloc_output(g, w.batch_size, w.fanouts) for _ in range(Gbuf)] for _ in range(S)]
    row_bytes = g.row_bytes

    keys = [synth.batch_rng_key(w, i) for i in range(len(batches))]
    depth = pipe.depth if pipe is not None else S
    # Per-batch counts live in a ring of rows: a buffer set is reused `depth` launch sets later (the
    # pipeline's events order that), a ring slot one launch set after that.
    ring = depth + 1
    counts_ring = torch.zeros((ring * Gbuf, 2 * L + 2), dtype=torch.int64, device=dev)
    stride = counts_ring.stride(0) * 8

    last_call = {}   # buffer set -> (first batch index, batches, ring slot) of the last launch set that used it
    sets_issued = [0]

    def run_calls(first, n):
        """Issues batches first .. first+n-1 (indices modulo the number of seed batches)."""
        bounds = set_bounds(first, n)
        for c, c_next in zip(bounds[:-1], bounds[1:]):
            k = c_next - c
            s_no = sets_issued[0]
            sets_issued[0] += 1
            q = s_no % depth
            slot = s_no % ring
            last_call[q] = (c, k, slot)
            idx = [(c + b) % len(batches) for b in range(k)]
            base = counts_ring.data_ptr() + slot * Gbuf * stride
            if pipe is not None:
                def point_counts(os_, base=base):
                    for b, o in enumerate(os_):
                        o.c.counts = base + b * stride
                pipe.issue(q, [batches[i] for i in idx], [keys[i] for i in idx], before_launch=point_counts)
            else:
                for b in range(k):
                    outs[q][b].c.counts = base + b * stride
                smfg.sample_mfg_many(g, wss[q][:k], [batches[i] for i in idx], w.fanouts, [keys[i] for i in idx],
                                     outs[q][:k], stream=streams[q])

    # Accounting pass (untimed, also the first warm-up): the K batches of a pass, launch set by
    # launch set with a synchronisation after each, to read their sizes.
    cnt = []
    for c in range(0, K, G):
        k = min(G, K - c)
        run_calls(c, k)
        torch.cuda.synchronize()
        slot = (sets_issued[0] - 1) % ring
        cnt += counts_ring[slot * Gbuf:slot * Gbuf + k].cpu().tolist()
    assert all(c[2 * L + 1] == 0 for c in cnt), "a batch reported a device status"
    n_final = sum(c[L] for c in cnt)
    edges = sum(sum(c[L + 1:2 * L + 1]) for c in cnt)
    alg = sum(algorithmic_bytes(c[:L + 1], c[L + 1:2 * L + 1], row_bytes) for c in cnt)

    # Warm-up as asked, but never less than `depth` full launch sets, then one probe pass to size
    # the number of timed passes.
    warm = max(W, depth * G)
    run_calls(K, warm)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_calls(0, K)
    torch.cuda.synchronize()
    probe = time.perf_counter() - t0
    passes = args.passes if args.passes > 0 else int(min(max(5, 0.6 / max(probe, 1e-6)), 400, max(5, 30.0 / max(probe, 1e-6))))
    sets_per_pass = len(set_bounds(0, K)) - 1

    # Timed region: `passes` passes of K batches each, issued back to back (no host synchronisation
    # between them), bracketed by device synchronisations.  A pass ends when the last stream has
    # finished its work of that pass: events on every stream after each pass, all measured from one
    # start event.
    ev_start = torch.cuda.Event(enable_timing=True)
    ev_end = [[torch.cuda.Event(enable_timing=True) for _ in streams] for _ in range(passes)]
    smfg.profile_begin(1, passes * sets_per_pass + 2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    ev_start.record(streams[0])
    for st in streams[1:]:
        st.wait_event(ev_start)
    for p_ in range(passes):
        run_calls(0, K)
        for e, st in zip(ev_end[p_], streams):
            e.record(st)
    torch.cuda.synchronize()
    region_s = time.perf_counter() - t0
    stages = smfg.profile_end()
    ends = [max(ev_start.elapsed_time(e) for e in evs) * 1e-3 for evs in ev_end]
    pass_s = sorted(b_ - a_ for a_, b_ in zip([0.0] + ends[:-1], ends))
    dt = pass_s[len(pass_s) // 2] if len(pass_s) % 2 else 0.5 * (pass_s[len(pass_s) // 2 - 1] + pass_s[len(pass_s) // 2])
    gather_ms, gather_launches = stages["gather"]
    gather_bytes = 2 * row_bytes * n_final * passes
    gather_gbs = gather_bytes / (gather_ms * 1e-3) / 1e9 if gather_ms > 0 else 0.0
    cnt_of_slot = {}
    for q, (c, k, slot) in last_call.items():
        cnt_of_slot[q] = [cnt[(c + b) % K] for b in range(k)]

    # The same gather launches once more with nothing else on the chip (the buffers of the last
    # launch sets are still in place): the kernel's own rate, next to the overlapped one above.
    smfg.profile_begin(1, 16)
    rows_alone = 0
    full_sets = [q for q, (c, k, slot) in last_call.items() if k == max(v[1] for v in last_call.values())]
    for rep in range(6):
        q = full_sets[rep % len(full_sets)]
        k = last_call[q][1]
        smfg.gather_many(g, outs[q][:k], stream=streams[0])
        rows_alone += sum(c[L] for c in cnt_of_slot[q])
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
        q = full_sets[0]
        k_set, slot_q = last_call[q][1], last_call[q][2]
        cnt_q = cnt_of_slot[q]
        agg_out = torch.empty((outs[q][0].node_capacity, w.feat_dim), dtype=torch.float32, device=dev)
        smfg.profile_begin(2, 4 * G)
        agg_bytes = 0
        for rep in range(2):
            for b in range(k_set):
                o, c = outs[q][b], cnt_q[b]
                n_dst, e_last = c[L - 1], c[2 * L]
                cview = counts_ring[slot_q * Gbuf + b]
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
                    o, c = outs[q][b], cnt_q[b]
                    n_dst, e_last = c[L - 1], c[2 * L]
                    cview = counts_ring[slot_q * Gbuf + b]
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

    traffic_row, traffic_note = (None, "not stored for an overridden feature width or row stride") \
        if (args.feat_dim or args.row_stride) else stored_traffic(w.name, G)
    result = {
        "metric": "sampled mini-batches/sec (MFG build + feature gather)",
        "value": K / dt, "unit": "batches/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": dt / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "timing": {"what": "median over `passes` passes of `steps` batches each, issued back to back and bracketed by "
                           "device synchronisations; a pass ends when every stream has finished its work of the pass "
                           "(HIP events on the issuing streams)",
                   "passes": passes, "pass_ms_median": dt * 1e3, "pass_ms_min": pass_s[0] * 1e3,
                   "pass_ms_max": pass_s[-1] * 1e3, "warmup_batches_run": warm + K,
                   "region_s_host_clock": region_s, "region_batches_per_s": passes * K / region_s},
        "config": {"workload": f"{w.name}: {w.num_nodes} nodes, {graph.num_edges} directed edges, "
                               f"features {w.feat_dim}x{str(w.feat_dtype).split('.')[-1]}, fanouts {list(w.fanouts)}, "
                               f"batch {w.batch_size}", "batches_per_call": G, "launch_sets_of_a_pass": [y - x for x, y in zip(set_bounds(0, K)[:-1], set_bounds(0, K)[1:])][:8],
                   "streams": S, "pipeline": bool(args.pipeline),
                   "dedup_strategy": wss[0][0].strategy,
                   "sample_streams": args.sample_streams if args.pipeline else None,
                   "buffer_sets": depth,
                   "row_stride_bytes": int(feat.stride(0) * feat.element_size()),
                   "mean_nodes_per_batch": n_final / K, "mean_edges_per_batch": edges / K},
        "sampled_edges_per_s": edges / dt,
        "gather_GBps": gather_gbs,
        "path_algorithmic_GBps": alg / dt / 1e9,
        "path_frac_of_hbm_peak": alg / dt / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "k_gather", "achieved": gather_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": gather_gbs / HBM_PEAK_GBS,
                     "traffic": traffic_row * n_final * passes / max(1, gather_launches) if traffic_row else None,
                     "traffic_unit": "bytes per launch", "traffic_note": traffic_note,
                     "avg_launch_ms": gather_ms / max(1, gather_launches), "launches": gather_launches,
                     "note": "achieved = algorithmic bytes of all gather launches of the timed region / their summed "
                             "durations (HIP events on the launch's own stream).  With --pipeline 1 every one of them "
                             "but the very last shares the chip with the sampling kernels of the next launch set; "
                             "alone_* is the same launch repeated right after with nothing else running",
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
        run_calls(0, K)
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
            o.c.counts = counts_ring.data_ptr()
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

        share = os.environ.get("OMP_NUM_THREADS", "")
        threads = args.cpu_threads or (int(share) if share.isdigit() and int(share) > 0
                                       else len(os.sched_getaffinity(0)))
        result["cpu_baseline"] = cpu_baseline(w, graph, feat, batches, keys, args.cpu_seconds, threads, gpu_check)

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()

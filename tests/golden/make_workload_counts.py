#!/usr/bin/env python3
"""Writes tests/golden/workload_counts.json: per-batch node and edge counts of the two small
workloads as the CPU oracle computes them (calls only synth for inputs and oracle/ for results).

    python tests/golden/make_workload_counts.py

The file guards against silent drift of the input generators or of the oracle: the paper prints no
worked example, so these are not paper values.
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2110_08450_amd import synth  # noqa: E402


def main():
    out = {}
    for name, batch_ids in (("tiny", [0, 1, 2, 3]), ("mid", [0, 45, 90])):
        w = synth.WORKLOADS[name]
        g = synth.make_graph(w)
        batches = synth.make_seed_batches(w)
        orc = oracle.Oracle(g.indptr.numpy(), g.indices.numpy())
        rows = []
        for b in batch_ids:
            r = orc.sample_mfg(batches[b].numpy(), w.fanouts, synth.batch_rng_key(w, b))
            rows.append({"batch": b, "nodes": r.num_nodes, "edges": r.num_edges,
                         "node_ids_head": r.node_ids[:4].tolist(), "node_ids_tail": r.node_ids[-4:].tolist()})
        out[name] = {"num_edges": g.num_edges, "num_batches": len(batches), "batches": rows}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "workload_counts.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print(path)


if __name__ == "__main__":
    main()

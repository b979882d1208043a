"""Double-buffered hand-off of prepared batches (stream and event plumbing only).

The paper overlaps the hand-off of batch i+1 with the training of batch i by using separate streams
and synchronising so that an iteration starts only after its data has arrived (section 4.3).  Here
the data never leaves the GPU, so the same idea becomes: launch set i+1 is sampled on a side stream
and its feature rows are gathered on a second side stream while the consumer still works on set i.
Two buffer sets exist; a set is overwritten only after the consumer has moved past it.  All
computation happens inside libsmfg's kernels.
"""
from __future__ import annotations

from typing import Callable, Iterator, List, Optional, Sequence

import torch

from . import binding as smfg


class BatchPipeline:
    def __init__(self, g: smfg.Graph, fanouts: Sequence[int], batch_size: int, batches_per_set: int = 8,
                 node_capacity: Optional[int] = None, depth: int = 2, sample_capacity: int = 0,
                 sample_streams: int = 1):
        self.g, self.fanouts = g, tuple(fanouts)
        self.G = max(1, min(batches_per_set, smfg.MAX_BATCHES))
        self.depth = depth
        cap = 0 if node_capacity is None else node_capacity
        self.wss = [[smfg.workspace_create(g, batch_size, self.fanouts, cap, sample_capacity) for _ in range(self.G)]
                    for _ in range(depth)]
        self.outs = [[smfg.alloc_output(g, batch_size, self.fanouts, node_capacity) for _ in range(self.G)]
                     for _ in range(depth)]
        # launch sets alternate over the sampling streams, so that the short kernels of one set's
        # first hops can fill the gaps of another set's (depth must exceed their number)
        self.s_samples = [torch.cuda.Stream() for _ in range(max(1, min(sample_streams, depth - 1)))]
        self.s_sample = self.s_samples[0]
        self.s_gather = torch.cuda.Stream()
        self._issued = 0
        self.sampled = [torch.cuda.Event() for _ in range(depth)]
        self.gathered = [torch.cuda.Event() for _ in range(depth)]
        self.released = [torch.cuda.Event() for _ in range(depth)]   # consumer is done with the set

    def issue(self, q: int, seeds: Sequence[torch.Tensor], keys: Sequence[int],
              before_launch: Optional[Callable[[List[smfg.Output]], None]] = None) -> List[smfg.Output]:
        """Enqueues one launch set into buffer set q; returns its outputs (valid after gathered[q])."""
        k = len(seeds)
        outs = self.outs[q][:k]
        if before_launch is not None:
            before_launch(outs)
        ss = self.s_samples[self._issued % len(self.s_samples)]
        self._issued += 1
        ss.wait_event(self.released[q])
        ss.wait_event(self.gathered[q])
        smfg.sample_mfg_many(self.g, self.wss[q][:k], seeds, self.fanouts, keys, outs, stream=ss,
                             with_features=self.g.feat is None)
        self.sampled[q].record(ss)
        if self.g.feat is not None:
            self.s_gather.wait_event(self.sampled[q])
            smfg.gather_many(self.g, outs, stream=self.s_gather)
            self.gathered[q].record(self.s_gather)
        else:
            self.gathered[q].record(ss)
        return outs

    def run(self, seed_batches: Sequence[torch.Tensor], rng_keys: Sequence[int]) -> Iterator[List[smfg.Output]]:
        """Yields the outputs of one launch set at a time, ready on the caller's current stream.
        While the caller handles set i, set i+1 is already being prepared.  What is yielded stays
        valid until the caller asks for the set after the next one."""
        sets = [(list(seed_batches[i:i + self.G]), list(rng_keys[i:i + self.G]))
                for i in range(0, len(seed_batches), self.G)]
        # inputs must be complete before the side streams read them
        start = torch.cuda.Event()
        start.record(torch.cuda.current_stream())
        for ss in self.s_samples:
            ss.wait_event(start)
        pending = []
        nxt = 0
        while nxt < len(sets) and len(pending) < self.depth:
            pending.append((nxt % self.depth, self.issue(nxt % self.depth, *sets[nxt])))
            nxt += 1
        while pending:
            q, outs = pending.pop(0)
            torch.cuda.current_stream().wait_event(self.gathered[q])
            yield outs
            self.released[q].record(torch.cuda.current_stream())
            if nxt < len(sets):
                pending.append((nxt % self.depth, self.issue(nxt % self.depth, *sets[nxt])))
                nxt += 1

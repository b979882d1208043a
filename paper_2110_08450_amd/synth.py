"""Seeded synthetic inputs: power-law graphs, feature tables and seed splits.

This module only *makes inputs*.  It contains none of the sampling / relabel /
gather arithmetic, so the CPU oracle and the HIP path can both be fed from it
without sharing any part of the method.

Everything is derived from a counter-based 64-bit integer hash evaluated with
plain torch integer ops, so the same (seed, shape) gives the same graph on the
CPU and on the GPU, independent of chunk sizes.

The graphs stand in for the paper's OGB datasets (Table 4: ogbn-arxiv,
ogbn-products, ogbn-papers100M) whose shapes they copy; the datasets themselves
are never needed.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Tuple

import torch

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 holds for those bits."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)
_GOLD = _s64(0x9E3779B97F4A7C15)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 bit patterns."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """A bijective 64-bit finalizer (xor-shift / multiply), wrapping int64 arithmetic."""
    x = (x ^ _lsr(x, 30)) * _C1
    x = (x ^ _lsr(x, 27)) * _C2
    return x ^ _lsr(x, 31)


def _mix64_int(x: int) -> int:
    x &= _MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK64
    return x ^ (x >> 31)


def hash64(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """64 hashed bits per element of `idx` (int64), distinct for distinct idx."""
    base = _s64(_mix64_int(_mix64_int(seed) ^ ((stream * 0x9E3779B97F4A7C15) & _MASK64)))
    return _mix64(idx * _GOLD + base)


def uniform01(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """float64 in [0, 1) from the top 53 hashed bits."""
    return _lsr(hash64(seed, stream, idx), 11).to(torch.float64) * (1.0 / (1 << 53))


# ----------------------------------------------------------------------------------------
# graphs
# ----------------------------------------------------------------------------------------

@dataclass
class Graph:
    num_nodes: int
    indptr: torch.Tensor   # int64 [num_nodes + 1]
    indices: torch.Tensor  # int32 [num_edges], rows sorted, no duplicates, no self loops

    @property
    def num_edges(self) -> int:
        return int(self.indices.numel())


def _rank_mass(i0: float, alpha: float, n: int) -> Tuple[float, float]:
    e = 1.0 - alpha
    return i0 ** e, (n + i0) ** e


def _top_prob(i0: float, alpha: float, n: int) -> float:
    a, b = _rank_mass(i0, alpha, n)
    return ((1.0 + i0) ** (1.0 - alpha) - a) / (b - a)


def solve_i0(num_nodes: int, num_pairs: int, alpha_src: float, alpha_dst: float,
             max_degree: float) -> float:
    """Offset i0 of the rank weights w_r ~ (r + i0)^-alpha so that the heaviest node's
    expected degree is `max_degree` (bisection; expected degree falls as i0 grows)."""
    def top_deg(i0: float) -> float:
        return num_pairs * (_top_prob(i0, alpha_src, num_nodes) + _top_prob(i0, alpha_dst, num_nodes))
    lo, hi = 1e-6, float(num_nodes) * 64.0
    if top_deg(lo) <= max_degree:
        return lo
    for _ in range(200):
        mid = math.sqrt(lo * hi)
        if top_deg(mid) > max_degree:
            lo = mid
        else:
            hi = mid
    return math.sqrt(lo * hi)


def _draw_rank(u: torch.Tensor, i0: float, alpha: float, n: int) -> torch.Tensor:
    """Inverse CDF of the continuous density ~ (x + i0)^-alpha on [0, n), floored to a rank."""
    a, b = _rank_mass(i0, alpha, n)
    x = (u * (b - a) + a) ** (1.0 / (1.0 - alpha)) - i0
    return x.to(torch.int64).clamp_(0, n - 1)


def powerlaw_graph(num_nodes: int, num_directed_edges: int, max_degree: float, seed: int,
                   gamma_dst: float = 2.5, gamma_src: Optional[float] = None,
                   device: str = "cpu", chunk_pairs: int = 1 << 26,
                   bucket_keys: int = 1 << 28) -> Graph:
    """Symmetric simple power-law graph in CSR (int64 indptr, int32 indices, sorted rows).

    Chung-Lu by endpoint sampling: `num_directed_edges / 2` endpoint pairs (u, v), each
    endpoint a rank drawn with probability ~ (rank + i0)^(-1/(gamma-1)); ranks are mapped to
    node ids by a seeded permutation so hubs are spread over the id range; self loops are
    dropped, both directions are added, duplicates removed.  `gamma_src` (default =
    `gamma_dst`) gives the citation-style recipe: mild out-weights, heavy-tailed in-weights,
    then made symmetric.
    """
    n = int(num_nodes)
    pairs = int(num_directed_edges) // 2
    a_dst = 1.0 / (gamma_dst - 1.0)
    a_src = a_dst if gamma_src is None else 1.0 / (gamma_src - 1.0)
    i0 = solve_i0(n, pairs, a_src, a_dst, max_degree)
    dev = torch.device(device)

    perm = torch.argsort(hash64(seed, 0, torch.arange(n, dtype=torch.int64, device=dev)))

    # all directed keys src * n + dst, kept as a list of chunks (each far below 2^31 elements)
    chunks: List[torch.Tensor] = []
    for c0 in range(0, pairs, chunk_pairs):
        idx = torch.arange(c0, min(pairs, c0 + chunk_pairs), dtype=torch.int64, device=dev)
        u = perm[_draw_rank(uniform01(seed, 1, idx), i0, a_src, n)]
        v = perm[_draw_rank(uniform01(seed, 2, idx), i0, a_dst, n)]
        keep = u != v
        u, v = u[keep], v[keep]
        chunks.append(torch.cat([u * n + v, v * n + u]))
        del idx, u, v, keep
    del perm

    total_keys = sum(int(c.numel()) for c in chunks)
    n_buckets = max(1, -(-total_keys // bucket_keys))
    rows_per_bucket = -(-n // n_buckets)
    deg = torch.zeros(n, dtype=torch.int64, device=dev)
    parts: List[torch.Tensor] = []
    for b in range(n_buckets):
        r0, r1 = b * rows_per_bucket, min(n, (b + 1) * rows_per_bucket)
        if r0 >= r1:
            break
        lo, hi = r0 * n, r1 * n
        if n_buckets == 1:
            keys = torch.cat(chunks)
        else:
            keys = torch.cat([c[(c >= lo) & (c < hi)] for c in chunks])
        keys = torch.unique_consecutive(torch.sort(keys).values)
        src = torch.div(keys, n, rounding_mode="floor")
        deg[r0:r1] = torch.bincount(src - r0, minlength=r1 - r0)
        parts.append((keys - src * n).to(torch.int32))
        del keys, src
    del chunks
    indptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    torch.cumsum(deg, 0, out=indptr[1:])
    m = int(indptr[-1].item())
    indices = torch.empty(m, dtype=torch.int32, device=dev)
    o = 0
    for p in parts:
        indices[o:o + p.numel()] = p
        o += int(p.numel())
    assert o == m
    return Graph(n, indptr, indices)


# ----------------------------------------------------------------------------------------
# features and seed splits
# ----------------------------------------------------------------------------------------

def normal_features(num_nodes: int, dim: int, dtype: torch.dtype, seed: int,
                    device: str = "cpu", chunk_rows: Optional[int] = None) -> torch.Tensor:
    """Row-major dense [num_nodes, dim] table of ~N(0,1) values (Box-Muller on hashed uniforms)."""
    dev = torch.device(device)
    out = torch.empty((num_nodes, dim), dtype=dtype, device=dev)
    half = (dim + 1) // 2
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 25) // max(1, half))
    for r0 in range(0, num_nodes, chunk_rows):
        r1 = min(num_nodes, r0 + chunk_rows)
        idx = (torch.arange(r0, r1, dtype=torch.int64, device=dev)[:, None] * half
               + torch.arange(half, dtype=torch.int64, device=dev)[None, :])
        u1 = 1.0 - uniform01(seed, 3, idx)          # (0, 1]
        u2 = uniform01(seed, 4, idx)
        r = torch.sqrt(-2.0 * torch.log(u1))
        z = torch.cat([r * torch.cos(2.0 * math.pi * u2), r * torch.sin(2.0 * math.pi * u2)], dim=1)
        out[r0:r1] = z[:, :dim].to(dtype)
        del idx, u1, u2, r, z
    return out


def node_permutation(num_nodes: int, seed: int, device: str = "cpu") -> torch.Tensor:
    """A seeded permutation of [0, num_nodes) as int32; splits are disjoint slices of it."""
    dev = torch.device(device)
    h = hash64(seed, 5, torch.arange(num_nodes, dtype=torch.int64, device=dev))
    return torch.argsort(h).to(torch.int32)


def seed_batches(split: torch.Tensor, batch_size: int) -> List[torch.Tensor]:
    """Cut a split (already in random order) into batches; the partial last batch is kept."""
    return [split[i:i + batch_size].contiguous() for i in range(0, int(split.numel()), batch_size)]


# ----------------------------------------------------------------------------------------
# the five workloads
# ----------------------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    name: str
    num_nodes: int
    num_directed_edges: int
    max_degree: float
    gamma_src: Optional[float]
    feat_dim: int
    feat_dtype: torch.dtype
    fanouts: Tuple[int, ...]
    batch_size: int
    split_offset_frac: float   # where the seed split starts in the node permutation
    split_frac: float          # fraction of nodes that are seeds
    max_batches: Optional[int]
    graph_seed: int


WORKLOADS = {
    # Tiny: 4 batches of 256 seeds.
    "tiny": Workload("tiny", 10_000, 100_000, 300.0, None, 32, torch.float32, (10, 5), 256,
                     0.0, 0.1024, 4, 1001),
    # Shaped like ogbn-arxiv (Table 4; edges doubled by symmetrisation).
    "mid": Workload("mid", 169_000, 2_300_000, 13_000.0, None, 128, torch.float32, (15, 10, 5),
                    1024, 0.0, 0.55, None, 1002),
    # Shaped like ogbn-products.
    "large": Workload("large", 2_450_000, 124_000_000, 17_000.0, None, 100, torch.float16,
                      (15, 10, 5), 1024, 0.0, 0.08, None, 1003),
    # products-shaped graph with fanouts beyond 32 and with full neighbourhoods (Table 6 compares
    # fanouts (20,20,20), (100,100,100) and "all" for inference).
    "large_wide": Workload("large_wide", 2_450_000, 124_000_000, 17_000.0, None, 100, torch.float16,
                           (100, 100), 1024, 0.08, 0.02, None, 1003),
    "large_all": Workload("large_all", 2_450_000, 124_000_000, 17_000.0, None, 100, torch.float16,
                          (-1, -1), 256, 0.08, 0.005, None, 1003),
    # Shaped like ogbn-papers100M, training fanouts.
    "papers": Workload("papers", 111_000_000, 3_200_000_000, 100_000.0, 3.5, 128, torch.float16,
                       (15, 10, 5), 1024, 0.0, 0.011, None, 1004),
    # Same graph, inference-shaped sampling on a held-out split.
    "papers_infer": Workload("papers_infer", 111_000_000, 3_200_000_000, 100_000.0, 3.5, 128,
                             torch.float16, (20, 20, 20), 4096, 0.011, 0.002, None, 1004),
}


def make_graph(w: Workload, device: str = "cpu") -> Graph:
    return powerlaw_graph(w.num_nodes, w.num_directed_edges, w.max_degree, w.graph_seed,
                          gamma_src=w.gamma_src, device=device)


def make_features(w: Workload, device: str = "cpu") -> torch.Tensor:
    return normal_features(w.num_nodes, w.feat_dim, w.feat_dtype, w.graph_seed, device=device)


def make_seed_batches(w: Workload, device: str = "cpu") -> List[torch.Tensor]:
    perm = node_permutation(w.num_nodes, w.graph_seed, device=device)
    a = int(w.split_offset_frac * w.num_nodes)
    b = a + int(w.split_frac * w.num_nodes)
    batches = seed_batches(perm[a:b], w.batch_size)
    return batches if w.max_batches is None else batches[:w.max_batches]


def batch_rng_key(w: Workload, batch_index: int) -> int:
    """One key per batch: (graph seed << 32) | batch index."""
    return (w.graph_seed << 32) | (batch_index & 0xFFFFFFFF)

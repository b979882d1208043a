"""Thin ctypes binding of libsmfg.so: argument marshalling only.

Function names mirror include/smfg.h without the `smfg_` prefix.  PyTorch supplies device memory
(`torch.empty`) and the stream; every step of the path runs inside the library's kernels.  The
library must have been built (`python -m paper_2110_08450_amd.build` or `__graft_entry__.build()`);
loading fails loudly otherwise - there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

MAX_LAYERS = 8
MAX_FANOUT = 32
MAX_WIDE_FANOUT = 1024
FANOUT_ALL = -1
MAX_BATCHES = 16

OK = 0
ERR_INVALID_ARG, ERR_NULL_PTR, ERR_BAD_FANOUT, ERR_TOO_MANY_LAYERS = -1, -2, -3, -4
ERR_TOO_MANY_SEEDS, ERR_OOM, ERR_CAPACITY, ERR_BAD_GRAPH, ERR_HIP_BASE = -5, -6, -7, -8, -1000
ST_NODE_CAPACITY, ST_EDGE_CAPACITY, ST_TABLE_FULL, ST_SEED_OUT_OF_RANGE, ST_DUPLICATE_SEED = 1, 2, 3, 4, 5
ST_INTERNAL = 6
STRATEGY_TABLE, STRATEGY_PARTITION = 0, 1

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsmfg.so")

EXPORTS = [
    "smfg_graph_create", "smfg_graph_destroy", "smfg_graph_validate", "smfg_graph_set_labels", "smfg_bounds",
    "smfg_workspace_create", "smfg_workspace_create_sized",
    "smfg_workspace_destroy", "smfg_workspace_bytes", "smfg_workspace_strategy", "smfg_sample_mfg", "smfg_sample_mfg_many",
    "smfg_sample_mfg_static",
    "smfg_gather_rows", "smfg_gather_many", "smfg_mean_aggregate", "smfg_sage_layer", "smfg_sage_pack_weights",
    "smfg_sage_packed_bytes", "smfg_read_counts", "smfg_strerror", "smfg_profile_begin", "smfg_profile_end",
]
STAGES = ["clear", "seeds", "sample_insert", "flag_rows", "scan_tiles", "assemble", "gather",
          "mean_aggregate", "sage_layer", "partition", "dedup_buckets"]


class SmfgError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class _Output(ctypes.Structure):
    _fields_ = [
        ("indptr", ctypes.c_void_p * MAX_LAYERS),
        ("indices", ctypes.c_void_p * MAX_LAYERS),
        ("node_ids", ctypes.c_void_p),
        ("features", ctypes.c_void_p),
        ("counts", ctypes.c_void_p),
        ("node_capacity", ctypes.c_int64),
        ("edge_capacity", ctypes.c_int64 * MAX_LAYERS),
        ("labels", ctypes.c_void_p),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2110_08450_amd.build)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
        pp = ctypes.POINTER(ctypes.c_void_p)
        L.smfg_graph_create.argtypes = [pp, i64, i64, vp, vp, vp, i32, i32, i64]
        L.smfg_graph_destroy.argtypes = [vp]
        L.smfg_graph_validate.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32), vp]
        L.smfg_graph_set_labels.argtypes = [vp, vp, i32]
        L.smfg_bounds.argtypes = [i32, i32, ctypes.POINTER(i32), i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.smfg_workspace_create.argtypes = [pp, vp, i32, i32, ctypes.POINTER(i32), i64]
        L.smfg_workspace_create_sized.argtypes = [pp, vp, i32, i32, ctypes.POINTER(i32), i64, i64]
        L.smfg_workspace_destroy.argtypes = [vp]
        L.smfg_workspace_bytes.argtypes = [vp]
        L.smfg_workspace_bytes.restype = i64
        L.smfg_workspace_strategy.argtypes = [vp]
        L.smfg_sample_mfg.argtypes = [vp, vp, vp, i32, ctypes.POINTER(i32), i32, u64,
                                      ctypes.POINTER(_Output), vp]
        L.smfg_sample_mfg_static.argtypes = [vp, vp, i32, ctypes.POINTER(i32), i32, u64, ctypes.POINTER(_Output), vp]
        L.smfg_sample_mfg_many.argtypes = [vp, pp, pp, ctypes.POINTER(i32), ctypes.POINTER(i32), i32,
                                           ctypes.POINTER(u64), ctypes.POINTER(_Output), i32, vp]
        L.smfg_gather_rows.argtypes = [vp, vp, vp, i64, vp, vp]
        L.smfg_gather_many.argtypes = [vp, ctypes.POINTER(_Output), i32, i32, vp]
        L.smfg_mean_aggregate.argtypes = [vp, vp, i64, vp, i64, vp, i64, i32, i32, vp, vp]
        L.smfg_sage_layer.argtypes = [vp, vp, i64, vp, i64, vp, i64, i32, vp, vp, i32, i32, vp, i32, vp]
        L.smfg_sage_packed_bytes.argtypes = [i32, i32]
        L.smfg_sage_packed_bytes.restype = i64
        L.smfg_sage_pack_weights.argtypes = [vp, i32, i32, vp, vp]
        L.smfg_read_counts.argtypes = [ctypes.POINTER(_Output), i32, ctypes.POINTER(i64), vp]
        L.smfg_profile_begin.argtypes = [i32, i32]
        L.smfg_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        L.smfg_strerror.argtypes = [ctypes.c_int]
        L.smfg_strerror.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("smfg_workspace_bytes", "smfg_strerror", "smfg_sage_packed_bytes"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().smfg_strerror(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != OK:
        raise SmfgError(code, where)


def _fan(fanouts: Sequence[int]):
    return (ctypes.c_int32 * max(1, len(fanouts)))(*[int(d) for d in fanouts])


def _stream_ptr(stream: Optional[torch.cuda.Stream]):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(t.data_ptr()) if t is not None and t.numel() > 0 else ctypes.c_void_p(None)


class Graph:
    """Graph handle; keeps the borrowed device tensors alive."""

    def __init__(self, handle, indptr, indices, feat):
        self.handle, self.indptr, self.indices, self.feat = handle, indptr, indices, feat
        self.labels = None
        self.num_nodes = int(indptr.numel() - 1)
        self.row_bytes = int(feat.shape[1] * feat.element_size()) if feat is not None else 0

    def __del__(self):
        if getattr(self, "handle", None):
            lib().smfg_graph_destroy(self.handle)
            self.handle = None


def graph_create(indptr: torch.Tensor, indices: torch.Tensor, feat: Optional[torch.Tensor] = None) -> Graph:
    assert indptr.dtype == torch.int64 and indices.dtype == torch.int32
    assert indptr.is_contiguous() and indices.is_contiguous()
    h = ctypes.c_void_p()
    if feat is not None:
        assert feat.dim() == 2 and feat.stride(1) == 1
        fd, eb, stride = int(feat.shape[1]), int(feat.element_size()), int(feat.stride(0) * feat.element_size())
    else:
        fd, eb, stride = 0, 0, 0
    rc = lib().smfg_graph_create(ctypes.byref(h), indptr.numel() - 1, indices.numel(),
                                 ctypes.c_void_p(indptr.data_ptr()), _ptr(indices),
                                 ctypes.c_void_p(feat.data_ptr()) if feat is not None else None,
                                 fd, eb, stride)
    _check(rc, "smfg_graph_create")
    return Graph(h, indptr, indices, feat)


BAD_INDPTR_START, BAD_INDPTR_ORDER, BAD_INDPTR_END, BAD_INDEX_RANGE = 1, 2, 4, 8


def graph_validate(g: Graph, stream: Optional[torch.cuda.Stream] = None) -> int:
    """0 if the CSR arrays are consistent, else the OR of the BAD_* bits.  Synchronises the stream."""
    flags = ctypes.c_uint32(0)
    rc = lib().smfg_graph_validate(g.handle, ctypes.byref(flags), _stream_ptr(stream))
    if rc != OK and rc != ERR_BAD_GRAPH:
        _check(rc, "smfg_graph_validate")
    return int(flags.value)


def graph_set_labels(g: Graph, labels: Optional[torch.Tensor]) -> None:
    """y: one element per node (1, 2, 4 or 8 bytes each), on the graph's device."""
    if labels is None:
        _check(lib().smfg_graph_set_labels(g.handle, None, 0), "smfg_graph_set_labels")
    else:
        assert labels.dim() == 1 and labels.is_contiguous() and labels.numel() == g.num_nodes
        _check(lib().smfg_graph_set_labels(g.handle, ctypes.c_void_p(labels.data_ptr()), labels.element_size()),
               "smfg_graph_set_labels")
    g.labels = labels


def bounds(num_seeds: int, fanouts: Sequence[int], num_nodes: int):
    L = len(fanouts)
    mn = (ctypes.c_int64 * (L + 1))()
    me = (ctypes.c_int64 * max(1, L))()
    _check(lib().smfg_bounds(num_seeds, L, _fan(fanouts), num_nodes, mn, me), "smfg_bounds")
    return list(mn), list(me)[:L]


class Workspace:
    def __init__(self, handle):
        self.handle = handle

    @property
    def nbytes(self) -> int:
        return int(lib().smfg_workspace_bytes(self.handle))

    @property
    def strategy(self) -> str:
        """'partition' or 'table': how calls on this workspace dedup a hop."""
        return "partition" if lib().smfg_workspace_strategy(self.handle) == STRATEGY_PARTITION else "table"

    def __del__(self):
        if getattr(self, "handle", None):
            lib().smfg_workspace_destroy(self.handle)
            self.handle = None


def workspace_create(g: Graph, max_seeds: int, fanouts: Sequence[int], node_capacity: int = 0,
                     sample_capacity: int = 0) -> Workspace:
    """sample_capacity > 0 bounds the samples of one hop explicitly (needed with FANOUT_ALL)."""
    h = ctypes.c_void_p()
    if sample_capacity:
        rc = lib().smfg_workspace_create_sized(ctypes.byref(h), g.handle, max_seeds, len(fanouts), _fan(fanouts),
                                               node_capacity, sample_capacity)
    else:
        rc = lib().smfg_workspace_create(ctypes.byref(h), g.handle, max_seeds, len(fanouts), _fan(fanouts),
                                         node_capacity)
    _check(rc, "smfg_workspace_create")
    return Workspace(h)


@dataclass
class Output:
    """Caller-owned device buffers of one batch plus the C struct that points at them."""
    L: int
    node_capacity: int
    edge_capacity: List[int]
    indptr: List[torch.Tensor]
    indices: List[torch.Tensor]
    node_ids: torch.Tensor
    features: Optional[torch.Tensor]
    counts: torch.Tensor
    labels: Optional[torch.Tensor] = None
    c: _Output = field(repr=False, default=None)


def mfg_blocks(out: Output, counts: Sequence[int]):
    """Views of one prepared batch in the order a layer-by-layer consumer walks it (Appendix C,
    GraphSAGE listing): outermost hop first.  `counts` is what read_counts returned.  Each item is
    (indptr [n_dst + 1], indices [E], (n_src, n_dst)); the destinations of a block are the first
    n_dst of its n_src source nodes.  No copies."""
    L = out.L
    n, e = counts[:L + 1], counts[L + 1:2 * L + 1]
    return [(out.indptr[h][:n[h] + 1], out.indices[h][:e[h]], (n[h + 1], n[h])) for h in range(L - 1, -1, -1)]


def alloc_output(g: Graph, max_seeds: int, fanouts: Sequence[int], node_capacity: Optional[int] = None,
                 edge_capacity: Optional[Sequence[int]] = None, with_features: bool = True) -> Output:
    """torch.empty device buffers sized to the worst case unless capacities are given."""
    L = len(fanouts)
    mn, me = bounds(max_seeds, fanouts, g.num_nodes)
    ncap = max(1, int(node_capacity if node_capacity is not None else mn[L]))
    m = int(g.indices.numel())   # a hop never has more edges than the graph: destinations are distinct
    ecap = [int(x) for x in (edge_capacity if edge_capacity is not None
                             else [min(m, me[h], ncap * fanouts[h]) if fanouts[h] > 0 else m for h in range(L)])]
    dev = g.indptr.device
    indptr = [torch.empty(ncap + 1, dtype=torch.int32, device=dev) for _ in range(L)]
    indices = [torch.empty(max(1, ecap[h]), dtype=torch.int32, device=dev) for h in range(L)]
    node_ids = torch.empty(ncap, dtype=torch.int32, device=dev)
    counts = torch.zeros(2 * L + 2, dtype=torch.int64, device=dev)
    feats = None
    if with_features and g.feat is not None:
        feats = torch.empty((ncap, g.feat.shape[1]), dtype=g.feat.dtype, device=dev)
    c = _Output()
    for h in range(L):
        c.indptr[h] = indptr[h].data_ptr()
        c.indices[h] = indices[h].data_ptr()
        c.edge_capacity[h] = ecap[h]
    c.node_ids = node_ids.data_ptr()
    c.features = feats.data_ptr() if feats is not None else None
    c.counts = counts.data_ptr()
    c.node_capacity = ncap
    labels = None
    if g.labels is not None:
        labels = torch.empty(max(1, max_seeds), dtype=g.labels.dtype, device=dev)
        c.labels = labels.data_ptr()
    return Output(L, ncap, ecap, indptr, indices, node_ids, feats, counts, labels, c)


def sample_mfg(g: Graph, ws: Workspace, seeds: torch.Tensor, fanouts: Sequence[int], rng_key: int,
               out: Output, stream: Optional[torch.cuda.Stream] = None) -> None:
    assert seeds.dtype == torch.int32 and seeds.is_contiguous()
    rc = lib().smfg_sample_mfg(g.handle, ws.handle, _ptr(seeds), seeds.numel(), _fan(fanouts), len(fanouts),
                               ctypes.c_uint64(rng_key & 0xFFFFFFFFFFFFFFFF), ctypes.byref(out.c),
                               _stream_ptr(stream))
    _check(rc, "smfg_sample_mfg")


STATIC_SCRATCH_BYTES = 64 << 20


def sample_mfg_static(g: Graph, seeds: torch.Tensor, fanouts: Sequence[int], rng_key: int, out: Output,
                      stream: Optional[torch.cuda.Stream] = None) -> None:
    """sample_mfg without a workspace: scratch is the library's fixed per-GPU array; allocates nothing."""
    assert seeds.dtype == torch.int32 and seeds.is_contiguous()
    rc = lib().smfg_sample_mfg_static(g.handle, _ptr(seeds), seeds.numel(), _fan(fanouts), len(fanouts),
                                      ctypes.c_uint64(rng_key & 0xFFFFFFFFFFFFFFFF), ctypes.byref(out.c),
                                      _stream_ptr(stream))
    _check(rc, "smfg_sample_mfg_static")


def _out_array(outs: Sequence[Output], with_features: bool = True):
    a = (_Output * len(outs))()
    for i, o in enumerate(outs):
        ctypes.memmove(ctypes.byref(a[i]), ctypes.byref(o.c), ctypes.sizeof(_Output))
        if not with_features:
            a[i].features = None
    return a


def gather_many(g: Graph, outs: Sequence[Output], stream: Optional[torch.cuda.Stream] = None) -> None:
    rc = lib().smfg_gather_many(g.handle, _out_array(outs), len(outs), outs[0].L, _stream_ptr(stream))
    _check(rc, "smfg_gather_many")


def sample_mfg_many(g: Graph, wss: Sequence[Workspace], seeds: Sequence[torch.Tensor], fanouts: Sequence[int],
                    rng_keys: Sequence[int], outs: Sequence[Output],
                    stream: Optional[torch.cuda.Stream] = None, with_features: bool = True) -> None:
    n = len(wss)
    assert len(seeds) == n and len(rng_keys) == n and len(outs) == n
    for s in seeds:
        assert s.dtype == torch.int32 and s.is_contiguous()
    a_ws = (ctypes.c_void_p * n)(*[w.handle for w in wss])
    a_seeds = (ctypes.c_void_p * n)(*[_ptr(s) for s in seeds])
    a_ns = (ctypes.c_int32 * n)(*[s.numel() for s in seeds])
    a_keys = (ctypes.c_uint64 * n)(*[k & 0xFFFFFFFFFFFFFFFF for k in rng_keys])
    a_outs = _out_array(outs, with_features)
    rc = lib().smfg_sample_mfg_many(g.handle, a_ws, a_seeds, a_ns, _fan(fanouts), len(fanouts), a_keys,
                                    a_outs, n, _stream_ptr(stream))
    _check(rc, "smfg_sample_mfg_many")


def gather_rows(g: Graph, node_ids: torch.Tensor, num_rows: torch.Tensor, max_rows: int, out: torch.Tensor,
                stream: Optional[torch.cuda.Stream] = None) -> None:
    assert node_ids.dtype == torch.int32 and num_rows.dtype == torch.int64
    rc = lib().smfg_gather_rows(g.handle, _ptr(node_ids), ctypes.c_void_p(num_rows.data_ptr()), max_rows,
                                ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream))
    _check(rc, "smfg_gather_rows")


def mean_aggregate(indptr: torch.Tensor, indices: torch.Tensor, num_dst: torch.Tensor, max_dst: int,
                   x: torch.Tensor, out: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """out[i] = mean of x[indices[e]] over the block row i (float32 out; x is float16 or float32)."""
    assert indptr.dtype == torch.int32 and indices.dtype == torch.int32 and num_dst.dtype == torch.int64
    assert x.dim() == 2 and x.is_contiguous() and x.dtype in (torch.float16, torch.float32)
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape[1] == x.shape[1]
    assert out.shape[0] >= max_dst
    assert indptr.numel() >= max_dst + 1
    rc = lib().smfg_mean_aggregate(ctypes.c_void_p(indptr.data_ptr()), ctypes.c_void_p(indices.data_ptr()),
                                   indices.numel(), ctypes.c_void_p(num_dst.data_ptr()), max_dst,
                                   ctypes.c_void_p(x.data_ptr()), x.shape[0], x.shape[1], x.element_size(),
                                   ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream))
    _check(rc, "smfg_mean_aggregate")


@dataclass
class PackedWeights:
    """A linear layer's weight [out_dim x 2 dim] re-arranged for smfg_sage_layer."""
    data: torch.Tensor
    dim: int
    out_dim: int


def sage_pack_weights(w: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> PackedWeights:
    assert w.dim() == 2 and w.is_contiguous() and w.dtype == torch.float16 and w.shape[1] % 2 == 0
    out_dim, dim = int(w.shape[0]), int(w.shape[1] // 2)
    nbytes = int(lib().smfg_sage_packed_bytes(dim, out_dim))
    if nbytes == 0:
        raise SmfgError(ERR_INVALID_ARG, "smfg_sage_packed_bytes")
    packed = torch.empty(nbytes // 2, dtype=torch.float16, device=w.device)
    _check(lib().smfg_sage_pack_weights(ctypes.c_void_p(w.data_ptr()), dim, out_dim, ctypes.c_void_p(packed.data_ptr()),
                                        _stream_ptr(stream)), "smfg_sage_pack_weights")
    return PackedWeights(packed, dim, out_dim)


def sage_layer(indptr: torch.Tensor, indices: torch.Tensor, num_dst: torch.Tensor, max_dst: int,
               x: torch.Tensor, w: PackedWeights, bias: Optional[torch.Tensor], relu: bool, out: torch.Tensor,
               stream: Optional[torch.cuda.Stream] = None) -> None:
    """out[i] = act([x[i] | mean of x[indices[e]] over block row i] w^T + bias); x float16, w from
    sage_pack_weights, bias float32 or None, out float16 or float32 [>= max_dst x out_dim]."""
    assert indptr.dtype == torch.int32 and indices.dtype == torch.int32 and num_dst.dtype == torch.int64
    assert x.dim() == 2 and x.is_contiguous() and x.dtype == torch.float16 and x.shape[1] == w.dim
    assert bias is None or (bias.dtype == torch.float32 and bias.is_contiguous() and bias.numel() == w.out_dim)
    assert out.dtype in (torch.float16, torch.float32) and out.is_contiguous() and out.shape[1] == w.out_dim
    assert out.shape[0] >= max_dst and indptr.numel() >= max_dst + 1
    rc = lib().smfg_sage_layer(ctypes.c_void_p(indptr.data_ptr()), ctypes.c_void_p(indices.data_ptr()),
                               indices.numel(), ctypes.c_void_p(num_dst.data_ptr()), max_dst,
                               ctypes.c_void_p(x.data_ptr()), x.shape[0], x.shape[1],
                               ctypes.c_void_p(w.data.data_ptr()),
                               ctypes.c_void_p(bias.data_ptr()) if bias is not None else None, w.out_dim,
                               int(bool(relu)), ctypes.c_void_p(out.data_ptr()), out.element_size(),
                               _stream_ptr(stream))
    _check(rc, "smfg_sage_layer")


def read_counts(out: Output, stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> List[int]:
    """Synchronises; returns [n_0..n_L, E_0..E_{L-1}, status]."""
    h = (ctypes.c_int64 * (2 * out.L + 2))()
    rc = lib().smfg_read_counts(ctypes.byref(out.c), out.L, h, _stream_ptr(stream))
    if rc < 0 or (check and rc != 0):
        raise SmfgError(rc, "smfg_read_counts")
    return list(h)


def profile_begin(level: int, max_records: int) -> None:
    _check(lib().smfg_profile_begin(level, max_records), "smfg_profile_begin")


def profile_end():
    """Synchronises; returns {stage: (milliseconds, launches)}."""
    ms = (ctypes.c_double * len(STAGES))()
    n = (ctypes.c_int64 * len(STAGES))()
    _check(lib().smfg_profile_end(ms, n), "smfg_profile_end")
    return {s: (float(ms[i]), int(n[i])) for i, s in enumerate(STAGES)}

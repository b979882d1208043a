"""ctypes front end of the CPU oracle (`smfg_oracle.c`).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package; the
product package never does.  Arrays are numpy, on the host.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "smfg_oracle.c")
_LIB = os.path.join(_HERE, "libsmfg_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no vector or threading flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", _LIB, _SRC])
    return _LIB


def _configure(lib):
    """Declares the argument types of the oracle's exports on a loaded library."""
    if True:
        u32p = ctypes.POINTER(ctypes.c_uint32)
        lib.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_floyd_positions.argtypes = [ctypes.c_uint32, ctypes.c_uint32, u32p, u32p]
        lib.oracle_floyd_positions.restype = ctypes.c_int32
        lib.oracle_sample_positions.argtypes = [ctypes.c_uint32, ctypes.c_int32, ctypes.c_uint64,
                                                ctypes.c_uint32, ctypes.c_uint32, u32p]
        lib.oracle_sample_positions.restype = ctypes.c_int32
        lib.oracle_slice_labels.restype = ctypes.c_int32
        lib.oracle_slice_labels.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p,
                                            ctypes.c_int32, ctypes.c_void_p]
        lib.oracle_half_to_double.restype = ctypes.c_double
        lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.oracle_mean_aggregate.restype = ctypes.c_int32
        lib.oracle_mean_aggregate.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                              ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_sage_layer.restype = ctypes.c_int32
        lib.oracle_sage_layer.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_sample_mfg.restype = ctypes.c_int32
        lib.oracle_sample_mfg.argtypes = [
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint64,
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p]
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _configure(ctypes.CDLL(build()))
    return _lib


ST_OK, ST_NODE_CAPACITY, ST_EDGE_CAPACITY, ST_SEED_RANGE, ST_DUP_SEED = 0, 1, 2, 4, 5


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> List[int]:
    c = (ctypes.c_uint32 * 4)(*[x & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[x & 0xFFFFFFFF for x in key])
    o = (ctypes.c_uint32 * 4)()
    _load().oracle_philox4x32_10(c, k, o)
    return list(o)


def floyd_positions(deg: int, k: int, words: Sequence[int]) -> List[int]:
    w = (ctypes.c_uint32 * max(1, k))(*[x & 0xFFFFFFFF for x in words[:k]])
    p = (ctypes.c_uint32 * max(1, k))()
    n = _load().oracle_floyd_positions(deg, k, w, p)
    return list(p[:n])


def sample_positions(deg: int, fanout: int, rng_key: int, v: int, h: int) -> List[int]:
    p = (ctypes.c_uint32 * max(1, min(deg, fanout) if fanout >= 0 else deg))()
    n = _load().oracle_sample_positions(deg, fanout, rng_key, v, h, p)
    if n < 0:
        raise ValueError("bad fanout")
    return list(p[:n])


def slice_labels(labels: np.ndarray, seeds: np.ndarray) -> np.ndarray:
    """ys = y[ids[:batch_size]] for a 1-D label array of any fixed-size dtype."""
    labels = np.ascontiguousarray(labels)
    seeds = np.ascontiguousarray(seeds, dtype=np.int32)
    out = np.empty(len(seeds), dtype=labels.dtype)
    rc = _load().oracle_slice_labels(labels.ctypes.data, labels.itemsize, len(labels), seeds.ctypes.data,
                                     len(seeds), out.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_slice_labels: {rc}")
    return out


def half_to_double(bits: int) -> float:
    return float(_load().oracle_half_to_double(bits & 0xFFFF))


def mean_aggregate(indptr: np.ndarray, indices: np.ndarray, x: np.ndarray):
    """(mean, mag) in float64 for one block; x is a 2-D float16 or float32 array of source rows."""
    indptr = np.ascontiguousarray(indptr, dtype=np.int32)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    assert x.ndim == 2 and x.flags["C_CONTIGUOUS"] and x.dtype in (np.float16, np.float32)
    n, dim = len(indptr) - 1, x.shape[1]
    mean = np.zeros((n, dim), dtype=np.float64)
    mag = np.zeros((n, dim), dtype=np.float64)
    rc = _load().oracle_mean_aggregate(indptr.ctypes.data, indices.ctypes.data, n, x.ctypes.data, dim,
                                       x.itemsize, mean.ctypes.data, mag.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_mean_aggregate: {rc}")
    return mean, mag


def sage_layer(indptr: np.ndarray, indices: np.ndarray, x: np.ndarray, w: np.ndarray,
               bias: Optional[np.ndarray], relu: bool):
    """(out, mag) in float64 for one GraphSAGE layer over a block: x [n_src x dim] float16/float32,
    w [out_dim x 2 dim] (columns [0, dim) act on the node's own row, [dim, 2 dim) on the mean),
    bias [out_dim] or None."""
    indptr = np.ascontiguousarray(indptr, dtype=np.int32)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    assert x.ndim == 2 and x.flags["C_CONTIGUOUS"] and x.dtype in (np.float16, np.float32)
    n, dim = len(indptr) - 1, x.shape[1]
    w = np.ascontiguousarray(w, dtype=np.float64)
    assert w.ndim == 2 and w.shape[1] == 2 * dim
    out_dim = w.shape[0]
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    assert b is None or b.shape == (out_dim,)
    tmp = np.zeros((2, max(1, n), dim), dtype=np.float64)
    out = np.zeros((n, out_dim), dtype=np.float64)
    mag = np.zeros((n, out_dim), dtype=np.float64)
    rc = _load().oracle_sage_layer(indptr.ctypes.data, indices.ctypes.data, n, x.ctypes.data, dim, x.itemsize,
                                   w.ctypes.data, None if b is None else b.ctypes.data, out_dim, int(bool(relu)),
                                   tmp[0].ctypes.data, tmp[1].ctypes.data, out.ctypes.data, mag.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_sage_layer: {rc}")
    return out, mag


@dataclass
class OracleMFG:
    status: int
    counts: np.ndarray               # int64 [2L+2]
    node_ids: np.ndarray             # int32 [n_L]
    indptr: List[np.ndarray]         # hop h: int32 [n_h + 1]
    indices: List[np.ndarray]        # hop h: int32 [E_h]
    features: Optional[np.ndarray]   # uint8 [n_L, row_bytes]

    @property
    def num_nodes(self) -> List[int]:
        L = len(self.indptr)
        return [int(x) for x in self.counts[:L + 1]]

    @property
    def num_edges(self) -> List[int]:
        L = len(self.indptr)
        return [int(x) for x in self.counts[L + 1:2 * L + 1]]


def worst_case(num_seeds: int, fanouts: Sequence[int], num_nodes: int):
    """n_{h+1} <= min(N, n_h (1 + d_h)) and E_h <= n_h d_h (disjoint-neighbourhood worst case).
    From the first fanout -1 (all neighbours) on: N nodes, and -1 (unknown) edges for such a hop."""
    nodes, edges = [min(num_seeds, num_nodes)], []
    everything = False
    for d in fanouts:
        everything = everything or d == -1
        if everything:
            edges.append(-1 if d == -1 else num_nodes * d)
            nodes.append(num_nodes)
        else:
            edges.append(nodes[-1] * d)
            nodes.append(min(num_nodes, nodes[-1] * (1 + d)))
    return nodes, edges


class Oracle:
    """Holds one graph (+ optional feature table) and the [num_nodes] scratch map."""

    def __init__(self, indptr: np.ndarray, indices: np.ndarray, feat: Optional[np.ndarray] = None):
        self.indptr = np.ascontiguousarray(indptr, dtype=np.int64)
        self.indices = np.ascontiguousarray(indices, dtype=np.int32)
        self.num_nodes = int(self.indptr.shape[0] - 1)
        self.feat = None
        self.row_bytes = self.row_stride = 0
        if feat is not None:
            assert feat.ndim == 2 and feat.flags["C_CONTIGUOUS"]
            self.feat = feat
            self.row_bytes = self.row_stride = int(feat.shape[1] * feat.itemsize)
        self.local_of = np.full(self.num_nodes, -1, dtype=np.int32)

    def clone_scratch(self) -> "Oracle":
        """Same graph, own scratch map: one per thread when batches run side by side."""
        o = Oracle.__new__(Oracle)
        o.__dict__.update(self.__dict__)
        o.local_of = np.full(self.num_nodes, -1, dtype=np.int32)
        return o

    def sample_mfg(self, seeds: np.ndarray, fanouts: Sequence[int], rng_key: int,
                   node_capacity: Optional[int] = None,
                   edge_capacity: Optional[Sequence[int]] = None,
                   with_features: bool = True) -> OracleMFG:
        seeds = np.ascontiguousarray(seeds, dtype=np.int32)
        L = len(fanouts)
        wc_nodes, wc_edges = worst_case(len(seeds), fanouts, self.num_nodes)
        ncap = int(node_capacity) if node_capacity is not None else max(1, wc_nodes[-1])
        if edge_capacity is None:   # a hop never has more edges than the graph: destinations are distinct
            edge_capacity = [min(e, len(self.indices)) if e >= 0 else len(self.indices) for e in wc_edges]
        ecap = np.asarray(edge_capacity, dtype=np.int64)
        fan = np.asarray(fanouts, dtype=np.int32)
        node_ids = np.empty(ncap, dtype=np.int32)
        indptr = [np.zeros(ncap + 1, dtype=np.int32) for _ in range(L)]
        indices = [np.empty(max(1, int(ecap[h])), dtype=np.int32) for h in range(L)]
        counts = np.zeros(2 * L + 2, dtype=np.int64)
        want_feat = with_features and self.feat is not None
        out_feat = np.empty((ncap, self.row_bytes), dtype=np.uint8) if want_feat else None
        pp = (ctypes.c_void_p * L)(*[a.ctypes.data for a in indptr])
        pi = (ctypes.c_void_p * L)(*[a.ctypes.data for a in indices])
        st = _load().oracle_sample_mfg(
            self.num_nodes, self.indptr.ctypes.data, self.indices.ctypes.data,
            self.feat.ctypes.data if want_feat else None, self.row_bytes, self.row_stride,
            seeds.ctypes.data, len(seeds), fan.ctypes.data, L, rng_key & 0xFFFFFFFFFFFFFFFF,
            self.local_of.ctypes.data, ncap, ecap.ctypes.data,
            node_ids.ctypes.data, pp, pi,
            out_feat.ctypes.data if want_feat else None, counts.ctypes.data)
        n = [int(x) for x in counts[:L + 1]]
        e = [int(x) for x in counts[L + 1:2 * L + 1]]
        return OracleMFG(
            status=int(st), counts=counts, node_ids=node_ids[:n[L]] if st == 0 else node_ids[:0],
            indptr=[indptr[h][:n[h] + 1] for h in range(L)],
            indices=[indices[h][:e[h]] for h in range(L)],
            features=out_feat[:n[L]] if (want_feat and st == 0) else None)

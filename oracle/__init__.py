"""CPU oracle for the beam-search hot path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package; the product (paper_2512_02278_amd) never does.  It wraps
``beam_search.c`` and ``graph_optimize.c`` (plain C, compiled with gcc) through
ctypes and takes numpy arrays that live in host memory.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "beam_search.c"), os.path.join(_HERE, "graph_optimize.c")]
_LIB = os.path.join(_HERE, "liboracle.so")

DT_U8, DT_F16, DT_F32 = 0, 1, 2
L2, IP = 0, 1

_NP_OF = {DT_U8: np.uint8, DT_F16: np.float16, DT_F32: np.float32}


def build(force: bool = True) -> str:
    """Compile the C sources into liboracle.so next to them (gcc, OpenMP over queries / graph rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, *_SRCS, "-lm"],
            check=True,
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        lib.oracle_search.restype = ctypes.c_int
        lib.oracle_search_routed.restype = ctypes.c_int
        lib.oracle_bruteforce.restype = ctypes.c_int
        lib.oracle_entries.restype = ctypes.c_int
        lib.oracle_route.restype = ctypes.c_int
        lib.oracle_threads.restype = ctypes.c_int
        lib.oracle_keys.restype = None
        _lib = lib
    return _lib


def dtype_code(arr: np.ndarray) -> int:
    for code, t in _NP_OF.items():
        if arr.dtype == t:
            return code
    raise TypeError(f"unsupported dtype {arr.dtype}")


def _p(arr):
    return None if arr is None else arr.ctypes.data_as(ctypes.c_void_p)


def _c(arr, dtype=None):
    if arr is None:
        return None
    a = np.ascontiguousarray(arr) if dtype is None else np.ascontiguousarray(arr, dtype=dtype)
    return a


class Index:
    """Host-side description of one partition: vectors, graph, entry rule."""

    def __init__(self, vectors, graph, metric=L2, n_entry=32, entry_mode=0, seed=0, centroids=None,
                 cluster_offsets=None, route_c=0):
        assert vectors.ndim == 2 and graph.ndim == 2 and graph.shape[0] == vectors.shape[0]
        assert vectors.strides[1] == vectors.itemsize, "rows must be dense along dim"
        self.vectors = vectors  # rows may be padded: the row stride is taken from .strides[0]
        self.graph = _c(graph, np.int32)
        self.metric, self.n_entry, self.entry_mode, self.seed = metric, n_entry, entry_mode, seed
        self.dtype = dtype_code(vectors)
        self.n, self.dim = vectors.shape
        self.degree = graph.shape[1]
        self.centroids = _c(centroids)
        self.cluster_offsets = _c(cluster_offsets, np.int64)
        self.n_clusters = 0 if centroids is None else centroids.shape[0]
        self.route_c = route_c
        if centroids is not None:
            assert centroids.dtype == vectors.dtype and centroids.shape[1] == self.dim
            assert self.cluster_offsets.shape[0] == self.n_clusters + 1

    def _head(self):
        return (_p(self.vectors), ctypes.c_int64(self.n), ctypes.c_int32(self.dim), ctypes.c_int32(self.dtype),
                ctypes.c_int64(self.vectors.strides[0]), _p(self.graph), ctypes.c_int32(self.degree),
                ctypes.c_int32(self.metric), ctypes.c_int32(self.n_entry), ctypes.c_int32(self.entry_mode),
                ctypes.c_uint64(self.seed), _p(self.centroids), _p(self.cluster_offsets),
                ctypes.c_int32(self.n_clusters), ctypes.c_int32(self.route_c))


def search(index: Index, queries, k, itopk, width, max_iters, forget_visited=False, n_threads=0, routes=None):
    """Returns (ids[nq,k] int32, dists[nq,k] int32|float32, counters dict of int64[nq]).

    routes (int32 [nq, route_c], routed entry mode only): cluster ids used instead of the oracle's own
    routing step; an id outside [0, n_clusters) names no cluster."""
    q = _c(queries)
    assert q.dtype == index.vectors.dtype and q.ndim == 2 and q.shape[1] == index.dim
    nq = q.shape[0]
    ids = np.empty((nq, k), np.int32)
    dists = np.empty((nq, k), np.int32 if index.dtype == DT_U8 else np.float32)
    iters, ndist, npar = (np.zeros(nq, np.int64) for _ in range(3))
    r = None
    if routes is not None:
        r = _c(routes, np.int32)
        assert index.entry_mode == 1 and r.shape == (nq, index.route_c)
    rc = _load().oracle_search_routed(*index._head(), _p(q), ctypes.c_int64(nq), ctypes.c_int32(k), ctypes.c_int32(itopk),
                                      ctypes.c_int32(width), ctypes.c_int32(max_iters), ctypes.c_int32(int(forget_visited)),
                                      _p(ids), _p(dists), _p(iters), _p(ndist), _p(npar), ctypes.c_int32(n_threads), _p(r))
    if rc != 0:
        raise ValueError("oracle_search rejected its arguments")
    return ids, dists, {"iters": iters, "n_dist": ndist, "n_parents": npar}


def bruteforce(vectors, queries, k, metric=L2):
    """Exact top-k under (key, id) over all rows of `vectors`."""
    q = _c(queries)
    assert q.dtype == vectors.dtype and vectors.strides[1] == vectors.itemsize
    nq = q.shape[0]
    code = dtype_code(vectors)
    ids = np.empty((nq, k), np.int32)
    dists = np.empty((nq, k), np.int32 if code == DT_U8 else np.float32)
    rc = _load().oracle_bruteforce(_p(vectors), ctypes.c_int64(vectors.shape[0]), ctypes.c_int32(vectors.shape[1]),
                                   ctypes.c_int32(code), ctypes.c_int64(vectors.strides[0]), ctypes.c_int32(metric),
                                   _p(q), ctypes.c_int64(nq), ctypes.c_int32(k), _p(ids), _p(dists))
    if rc != 0:
        raise ValueError("oracle_bruteforce rejected its arguments")
    return ids, dists


def keys(vectors, queries, ids, metric=L2):
    """key(q_i, x_id) as float64 for ids[nq, r]; +inf where id < 0."""
    q = _c(queries)
    ids = _c(ids, np.int32)
    out = np.empty(ids.shape, np.float64)
    _load().oracle_keys(_p(vectors), ctypes.c_int32(vectors.shape[1]), ctypes.c_int32(dtype_code(vectors)),
                        ctypes.c_int64(vectors.strides[0]), ctypes.c_int32(metric), _p(q),
                        ctypes.c_int64(q.shape[0]), ctypes.c_int32(ids.shape[1]), _p(ids), _p(out))
    return out


def entries(index: Index, queries):
    """Entry ids per query, [nq, n_entry] int32 (-1 where a slot produced none)."""
    q = _c(queries)
    out = np.empty((q.shape[0], index.n_entry), np.int32)
    rc = _load().oracle_entries(ctypes.c_int64(index.n), ctypes.c_int32(index.dim), ctypes.c_int32(index.dtype),
                                ctypes.c_int32(index.metric), ctypes.c_int32(index.n_entry),
                                ctypes.c_int32(index.entry_mode), ctypes.c_uint64(index.seed), _p(index.centroids),
                                _p(index.cluster_offsets), ctypes.c_int32(index.n_clusters),
                                ctypes.c_int32(index.route_c), _p(q), ctypes.c_int64(q.shape[0]), _p(out))
    if rc != 0:
        raise ValueError("oracle_entries rejected its arguments")
    return out


def route(centroids, queries, route_c, metric=L2):
    """The route_c nearest clusters per query under (key, cluster index)."""
    q = _c(queries)
    c = _c(centroids)
    out = np.empty((q.shape[0], route_c), np.int32)
    rc = _load().oracle_route(ctypes.c_int32(c.shape[1]), ctypes.c_int32(dtype_code(c)), ctypes.c_int32(metric),
                              _p(c), ctypes.c_int32(c.shape[0]), ctypes.c_int32(route_c), _p(q),
                              ctypes.c_int64(q.shape[0]), _p(out))
    if rc != 0:
        raise ValueError("oracle_route rejected its arguments")
    return out


def threads(n_threads=0) -> int:
    return int(_load().oracle_threads(ctypes.c_int32(n_threads)))


def merge_topk(ids, keys, k):
    """Final top-k of [nq, per_query] candidates under (key, id); id < 0 is padding."""
    ids = _c(ids, np.int32)
    keys = _c(keys)
    assert ids.shape == keys.shape and keys.dtype in (np.int32, np.float32)
    nq, per_query = ids.shape
    out_ids = np.empty((nq, k), np.int32)
    out_keys = np.empty((nq, k), keys.dtype)
    _load().oracle_merge_topk.restype = ctypes.c_int
    rc = _load().oracle_merge_topk(ctypes.c_int32(int(keys.dtype == np.float32)), _p(ids), _p(keys), ctypes.c_int64(nq),
                                   ctypes.c_int32(per_query), ctypes.c_int32(k), _p(out_ids), _p(out_keys))
    if rc != 0:
        raise ValueError("oracle_merge_topk rejected its arguments")
    return out_ids, out_keys


def gather(vectors, ids):
    """Rows of `vectors` for every id (zeros where the id is outside the partition)."""
    ids = _c(ids, np.int32)
    out = np.empty((*ids.shape, vectors.shape[1]), vectors.dtype)
    _load().oracle_gather.restype = None
    _load().oracle_gather(_p(vectors), ctypes.c_int64(vectors.shape[0]), ctypes.c_int32(vectors.shape[1]),
                          ctypes.c_int32(dtype_code(vectors)), ctypes.c_int64(vectors.strides[0]), _p(ids),
                          ctypes.c_int64(ids.size), _p(out))
    return out


def _graph_call(name, *args):
    fn = getattr(_load(), name)
    fn.restype = ctypes.c_int
    if fn(*args) != 0:
        raise ValueError(f"{name} rejected its arguments")


def graph_detours(knn):
    """c(x, j) for every entry of knn[n, d_in]: two-hop routes of smaller rank (-1 where absent)."""
    knn = _c(knn, np.int32)
    n, d_in = knn.shape
    counts = np.empty((n, d_in), np.int32)
    _graph_call("oracle_graph_detours", _p(knn), ctypes.c_int64(n), ctypes.c_int32(d_in), _p(counts))
    return counts


def graph_prune(knn, d_out):
    """Rows cut to d_out by ascending (detour count, rank)."""
    knn = _c(knn, np.int32)
    n, d_in = knn.shape
    out = np.empty((n, d_out), np.int32)
    _graph_call("oracle_graph_prune", _p(knn), ctypes.c_int64(n), ctypes.c_int32(d_in), ctypes.c_int32(d_out), _p(out))
    return out


def graph_reverse(pruned):
    """Per node, the sources of its first d in-edges in ascending (position in the source's row, source)."""
    pruned = _c(pruned, np.int32)
    n, d = pruned.shape
    out = np.empty((n, d), np.int32)
    _graph_call("oracle_graph_reverse", _p(pruned), ctypes.c_int64(n), ctypes.c_int32(d), _p(out))
    return out


def graph_merge(pruned, rev):
    """Forward half, then up to d/2 reverse edges, then the forward tail."""
    pruned, rev = _c(pruned, np.int32), _c(rev, np.int32)
    assert pruned.shape == rev.shape
    n, d = pruned.shape
    out = np.empty((n, d), np.int32)
    _graph_call("oracle_graph_merge", _p(pruned), _p(rev), ctypes.c_int64(n), ctypes.c_int32(d), _p(out))
    return out


def graph_optimize(knn, d_out):
    """knn[n, d_in] (rank order) -> search graph [n, d_out]: prune, reverse, merge."""
    knn = _c(knn, np.int32)
    n, d_in = knn.shape
    out = np.empty((n, d_out), np.int32)
    _graph_call("oracle_graph_optimize", _p(knn), ctypes.c_int64(n), ctypes.c_int32(d_in), ctypes.c_int32(d_out),
                _p(out))
    return out

"""ctypes binding of libann (include/ann.h): argument marshalling only.

The functions carry the names of the C entry points.  Tensors are torch tensors
on the GPU; torch is used for device memory and streams, nothing else.  There is
no CPU fallback: without the built library, or with host tensors, calls raise.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libann.so")

ANN_U8, ANN_F16, ANN_F32 = 0, 1, 2
ANN_L2, ANN_IP = 0, 1
ANN_ENTRY_UNIFORM, ANN_ENTRY_ROUTED = 0, 1
(ANN_OPT_CLUSTER_ORDER_MIN_QUERIES, ANN_OPT_VISITED_WINDOW_BITS, ANN_OPT_VISITED_HASH_BITS_BIAS,
 ANN_OPT_MATRIX_CORE_ROUTING, ANN_OPT_LANES_PER_ROW, ANN_OPT_WAVEFRONTS_PER_QUERY) = range(6)
ANN_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024
ANN_OK, ANN_EINVAL, ANN_EUNSUPPORTED, ANN_ENOMEM, ANN_EHIP = 0, -1, -2, -3, -4

_DTYPES = {torch.uint8: ANN_U8, torch.float16: ANN_F16, torch.float32: ANN_F32}

EXPORTS = ("ann_index_load", "ann_search", "ann_search_counters", "ann_search_routed", "ann_route", "ann_free",
           "ann_last_error", "ann_lds_bytes", "ann_calibration_copy", "ann_gather_vectors", "ann_merge_topk",
           "ann_graph_prune", "ann_graph_optimize", "ann_graph_optimize_workspace_bytes", "ann_calibration_gather",
           "ann_index_set_option", "ann_search_static")


class ann_index_desc_t(ctypes.Structure):
    _fields_ = [
        ("vectors", ctypes.c_void_p), ("n", ctypes.c_int64), ("dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("row_stride_bytes", ctypes.c_int64), ("graph", ctypes.c_void_p), ("degree", ctypes.c_int32),
        ("metric", ctypes.c_int32), ("n_entry", ctypes.c_int32), ("entry_mode", ctypes.c_int32),
        ("seed", ctypes.c_uint64), ("centroids", ctypes.c_void_p), ("cluster_offsets", ctypes.c_void_p),
        ("n_clusters", ctypes.c_int32), ("route_c", ctypes.c_int32),
    ]


class AnnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libann error {code}: {text}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libann.so; raises if it has not been built (python -m paper_2512_02278_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with paper_2512_02278_amd/build.py")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.ann_index_load.argtypes = [ctypes.POINTER(ann_index_desc_t), ctypes.POINTER(vp)]
        L.ann_index_load.restype = ctypes.c_int
        L.ann_search.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, vp, vp]
        L.ann_search.restype = ctypes.c_int
        L.ann_search_static.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, vp, vp]
        L.ann_search_static.restype = ctypes.c_int
        L.ann_search_counters.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, vp, vp, vp]
        L.ann_search_counters.restype = ctypes.c_int
        L.ann_search_routed.argtypes = [vp, vp, i64, vp, i32, i32, i32, i32, vp, vp, vp, vp]
        L.ann_search_routed.restype = ctypes.c_int
        L.ann_route.argtypes = [vp, vp, i64, vp, vp]
        L.ann_route.restype = ctypes.c_int
        L.ann_index_set_option.argtypes = [vp, i32, i64]
        L.ann_index_set_option.restype = ctypes.c_int
        L.ann_free.argtypes = [vp]
        L.ann_free.restype = ctypes.c_int
        L.ann_last_error.argtypes = []
        L.ann_last_error.restype = ctypes.c_char_p
        L.ann_gather_vectors.argtypes = [vp, vp, i64, vp, vp]
        L.ann_gather_vectors.restype = ctypes.c_int
        L.ann_merge_topk.argtypes = [i32, vp, vp, i64, i32, i32, vp, vp, vp]
        L.ann_merge_topk.restype = ctypes.c_int
        L.ann_calibration_copy.argtypes = [vp, vp, i64, vp]
        L.ann_calibration_copy.restype = ctypes.c_int
        L.ann_lds_bytes.argtypes = [vp, i32, i32]
        L.ann_lds_bytes.restype = ctypes.c_int64
        L.ann_calibration_gather.argtypes = [vp, vp, i64, vp, vp]
        L.ann_calibration_gather.restype = ctypes.c_int
        L.ann_graph_prune.argtypes = [vp, i64, i32, i32, vp, vp]
        L.ann_graph_prune.restype = ctypes.c_int
        L.ann_graph_optimize_workspace_bytes.argtypes = [i64, i32, i32]
        L.ann_graph_optimize_workspace_bytes.restype = ctypes.c_int64
        L.ann_graph_optimize.argtypes = [vp, i64, i32, i32, vp, vp, i64, vp]
        L.ann_graph_optimize.restype = ctypes.c_int
        _lib = L
    return _lib


def ann_last_error() -> str:
    return lib().ann_last_error().decode()


def _check(rc: int) -> None:
    if rc != ANN_OK:
        raise AnnError(rc, ann_last_error())


def _dev_ptr(t, what: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{what} must live on the GPU")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


class Handle:
    """An ann_index_t* plus references to the tensors it borrows (so they stay alive)."""

    def __init__(self, ptr, keep, dtype, dim, route_c):
        self.ptr, self._keep, self.dtype, self.dim, self.route_c = ptr, keep, dtype, dim, route_c


def ann_index_load(vectors: torch.Tensor, graph: torch.Tensor, metric: int = ANN_L2, n_entry: int = 32,
                   entry_mode: int = ANN_ENTRY_UNIFORM, seed: int = 0, centroids: torch.Tensor = None,
                   cluster_offsets: torch.Tensor = None, route_c: int = 0) -> Handle:
    """vectors [n, dim] (rows may be padded: stride(0) is the row stride), graph [n, degree] int32."""
    if vectors.dim() != 2 or vectors.stride(1) != 1 or vectors.dtype not in _DTYPES:
        raise ValueError("vectors must be [n, dim] uint8/float16/float32 with unit stride along dim")
    if graph.dim() != 2 or graph.dtype != torch.int32 or not graph.is_contiguous() or graph.shape[0] != vectors.shape[0]:
        raise ValueError("graph must be a contiguous [n, degree] int32 tensor")
    d = ann_index_desc_t()
    d.vectors, d.n, d.dim = _dev_ptr(vectors, "vectors"), vectors.shape[0], vectors.shape[1]
    d.dtype, d.row_stride_bytes = _DTYPES[vectors.dtype], vectors.stride(0) * vectors.element_size()
    d.graph, d.degree, d.metric = _dev_ptr(graph, "graph"), graph.shape[1], metric
    d.n_entry, d.entry_mode, d.seed = n_entry, entry_mode, seed
    if entry_mode == ANN_ENTRY_ROUTED:
        if centroids is None or cluster_offsets is None:
            raise ValueError("routed entries need centroids and cluster_offsets")
        if centroids.dtype != vectors.dtype or not centroids.is_contiguous() or centroids.shape[1] != vectors.shape[1]:
            raise ValueError("centroids must be contiguous [n_clusters, dim] of the vectors' dtype")
        if cluster_offsets.dtype != torch.int64 or cluster_offsets.numel() != centroids.shape[0] + 1:
            raise ValueError("cluster_offsets must be int64 [n_clusters + 1]")
        d.centroids, d.cluster_offsets = _dev_ptr(centroids, "centroids"), _dev_ptr(cluster_offsets, "cluster_offsets")
        d.n_clusters, d.route_c = centroids.shape[0], route_c
    h = ctypes.c_void_p()
    _check(lib().ann_index_load(ctypes.byref(d), ctypes.byref(h)))
    return Handle(h, (vectors, graph, centroids, cluster_offsets), vectors.dtype, vectors.shape[1], route_c)


def ann_index_set_option(h: Handle, option: int, value: int) -> None:
    _check(lib().ann_index_set_option(h.ptr, option, value))


def _queries_ok(h: Handle, queries: torch.Tensor):
    if queries.dim() != 2 or queries.dtype != h.dtype or queries.shape[1] != h.dim or not queries.is_contiguous():
        raise ValueError("queries must be a contiguous [nq, dim] tensor of the index dtype")


def ann_search(h: Handle, queries: torch.Tensor, k: int, itopk: int, width: int, max_iters: int,
               out_ids: torch.Tensor = None, out_dists: torch.Tensor = None, stream=None, counters: torch.Tensor = None,
               routes: torch.Tensor = None):
    """Enqueues the search on `stream` (default: torch's current stream); returns (out_ids, out_dists).

    With `counters` (int32 [nq, 4]) the call goes to ann_search_counters; with `routes`
    (int32 [nq, route_c] from ann_route) it goes to ann_search_routed."""
    _queries_ok(h, queries)
    nq = queries.shape[0]
    dd = torch.int32 if h.dtype == torch.uint8 else torch.float32
    if out_ids is None:
        out_ids = torch.empty((nq, k), dtype=torch.int32, device=queries.device)
    if out_dists is None:
        out_dists = torch.empty((nq, k), dtype=dd, device=queries.device)
    if out_ids.dtype != torch.int32 or out_dists.dtype != dd or out_ids.numel() != nq * k or out_dists.numel() != nq * k:
        raise ValueError("out_ids / out_dists have the wrong dtype or size")
    if not (out_ids.is_contiguous() and out_dists.is_contiguous()):
        raise ValueError("outputs must be contiguous")
    if counters is not None and (counters.dtype != torch.int32 or counters.numel() != nq * 4 or not counters.is_contiguous()):
        raise ValueError("counters must be a contiguous int32 [nq, 4] tensor")
    if routes is not None:
        if routes.dtype != torch.int32 or routes.numel() != nq * h.route_c or not routes.is_contiguous():
            raise ValueError("routes must be a contiguous int32 [nq, route_c] tensor")
        rc = lib().ann_search_routed(h.ptr, _dev_ptr(queries, "queries"), nq, _dev_ptr(routes, "routes"), k, itopk, width,
                                     max_iters, _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_dists, "out_dists"),
                                     _dev_ptr(counters, "counters"), _stream(stream))
    elif counters is None:
        rc = lib().ann_search(h.ptr, _dev_ptr(queries, "queries"), nq, k, itopk, width, max_iters,
                              _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_dists, "out_dists"), _stream(stream))
    else:
        rc = lib().ann_search_counters(h.ptr, _dev_ptr(queries, "queries"), nq, k, itopk, width, max_iters,
                                       _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_dists, "out_dists"),
                                       _dev_ptr(counters, "counters"), _stream(stream))
    _check(rc)
    return out_ids, out_dists


def ann_search_static(h: Handle, queries: torch.Tensor, k: int, itopk: int, width: int, max_iters: int,
                      out_ids: torch.Tensor, out_dists: torch.Tensor, stream=None):
    """ann_search with the library's static scratch: the caller passes every buffer, nothing is allocated."""
    _queries_ok(h, queries)
    nq = queries.shape[0]
    dd = torch.int32 if h.dtype == torch.uint8 else torch.float32
    if out_ids.dtype != torch.int32 or out_dists.dtype != dd or out_ids.numel() != nq * k or out_dists.numel() != nq * k:
        raise ValueError("out_ids / out_dists have the wrong dtype or size")
    if not (out_ids.is_contiguous() and out_dists.is_contiguous()):
        raise ValueError("outputs must be contiguous")
    _check(lib().ann_search_static(h.ptr, _dev_ptr(queries, "queries"), nq, k, itopk, width, max_iters,
                                   _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_dists, "out_dists"), _stream(stream)))
    return out_ids, out_dists


def ann_route(h: Handle, queries: torch.Tensor, out_clusters: torch.Tensor = None, stream=None) -> torch.Tensor:
    _queries_ok(h, queries)
    if out_clusters is None:
        out_clusters = torch.empty((queries.shape[0], h.route_c), dtype=torch.int32, device=queries.device)
    _check(lib().ann_route(h.ptr, _dev_ptr(queries, "queries"), queries.shape[0], _dev_ptr(out_clusters, "out"),
                           _stream(stream)))
    return out_clusters


def ann_lds_bytes(h: Handle, itopk: int, width: int) -> int:
    v = lib().ann_lds_bytes(h.ptr, itopk, width)
    if v < 0:
        raise AnnError(int(v), ann_last_error())
    return int(v)


def ann_free(h: Handle) -> None:
    if h is not None and h.ptr:
        _check(lib().ann_free(h.ptr))
        h.ptr = None
        h._keep = None


def ann_calibration_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """Plain copy kernel of known size, for calibrating a profiler's byte counters."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (dst.is_contiguous() and src.is_contiguous()):
        raise ValueError("dst and src must be contiguous and of equal size")
    _check(lib().ann_calibration_copy(_dev_ptr(dst, "dst"), _dev_ptr(src, "src"), nbytes, _stream(stream)))


def ann_gather_vectors(h: Handle, ids: torch.Tensor, out_vectors: torch.Tensor = None, stream=None) -> torch.Tensor:
    """Rows of the index for every id in `ids` (any shape, int32); zeros where id < 0."""
    if ids.dtype != torch.int32 or not ids.is_contiguous():
        raise ValueError("ids must be a contiguous int32 tensor")
    if out_vectors is None:
        out_vectors = torch.empty((*ids.shape, h.dim), dtype=h.dtype, device=ids.device)
    if out_vectors.dtype != h.dtype or out_vectors.numel() != ids.numel() * h.dim or not out_vectors.is_contiguous():
        raise ValueError("out_vectors must be contiguous, of the index dtype, with ids.numel() * dim elements")
    _check(lib().ann_gather_vectors(h.ptr, _dev_ptr(ids, "ids"), ids.numel(), _dev_ptr(out_vectors, "out_vectors"),
                                    _stream(stream)))
    return out_vectors


def ann_merge_topk(ids: torch.Tensor, keys: torch.Tensor, k: int, out_ids: torch.Tensor = None,
                   out_keys: torch.Tensor = None, stream=None):
    """ids, keys: [nq, per_query] candidates (int32 ids; int32 or float32 keys) -> ([nq, k], [nq, k])."""
    if ids.dim() != 2 or ids.shape != keys.shape or ids.dtype != torch.int32 or keys.dtype not in (torch.int32, torch.float32):
        raise ValueError("ids [nq, per_query] int32 and keys of the same shape, int32 or float32")
    if not (ids.is_contiguous() and keys.is_contiguous()):
        raise ValueError("ids and keys must be contiguous")
    nq, per_query = ids.shape
    if out_ids is None:
        out_ids = torch.empty((nq, k), dtype=torch.int32, device=ids.device)
    if out_keys is None:
        out_keys = torch.empty((nq, k), dtype=keys.dtype, device=ids.device)
    if out_ids.dtype != torch.int32 or out_keys.dtype != keys.dtype or out_ids.numel() != nq * k or out_keys.numel() != nq * k:
        raise ValueError("out_ids / out_keys have the wrong dtype or size")
    key_dtype = ANN_U8 if keys.dtype == torch.int32 else ANN_F32
    _check(lib().ann_merge_topk(key_dtype, _dev_ptr(ids, "ids"), _dev_ptr(keys, "keys"), nq, per_query, k,
                                _dev_ptr(out_ids, "out_ids"), _dev_ptr(out_keys, "out_keys"), _stream(stream)))
    return out_ids, out_keys


def _check_knn(knn: torch.Tensor):
    if knn.dim() != 2 or knn.dtype != torch.int32 or not knn.is_contiguous():
        raise ValueError("knn must be a contiguous [n, d_in] int32 tensor")
    return knn.shape


def ann_graph_prune(knn: torch.Tensor, d_out: int, pruned: torch.Tensor = None, stream=None) -> torch.Tensor:
    """knn [n, d_in] int32 in rank order -> [n, d_out]: each row's edges by ascending (detour count, rank)."""
    n, d_in = _check_knn(knn)
    if pruned is None:
        pruned = torch.empty((n, d_out), dtype=torch.int32, device=knn.device)
    if pruned.dtype != torch.int32 or pruned.numel() != n * d_out or not pruned.is_contiguous():
        raise ValueError("pruned must be a contiguous int32 tensor of n * d_out elements")
    _check(lib().ann_graph_prune(_dev_ptr(knn, "knn"), n, d_in, d_out, _dev_ptr(pruned, "pruned"), _stream(stream)))
    return pruned


def ann_graph_optimize_workspace_bytes(n: int, d_in: int, d_out: int) -> int:
    need = lib().ann_graph_optimize_workspace_bytes(n, d_in, d_out)
    if need < 0:
        raise AnnError(int(need), ann_last_error())
    return int(need)


def ann_graph_optimize(knn: torch.Tensor, d_out: int, out_graph: torch.Tensor = None, workspace: torch.Tensor = None,
                       stream=None) -> torch.Tensor:
    """knn [n, d_in] int32 in rank order -> search graph [n, d_out] (pruned edges plus reverse edges).

    workspace: a uint8 tensor of at least ann_graph_optimize_workspace_bytes(n, d_in, d_out) bytes; one is
    allocated (and released when the work is done) if none is given."""
    n, d_in = _check_knn(knn)
    if out_graph is None:
        out_graph = torch.empty((n, d_out), dtype=torch.int32, device=knn.device)
    if out_graph.dtype != torch.int32 or out_graph.numel() != n * d_out or not out_graph.is_contiguous():
        raise ValueError("out_graph must be a contiguous int32 tensor of n * d_out elements")
    if workspace is None:
        workspace = torch.empty(ann_graph_optimize_workspace_bytes(n, d_in, d_out), dtype=torch.uint8, device=knn.device)
    if workspace.dtype != torch.uint8 or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 tensor")
    _check(lib().ann_graph_optimize(_dev_ptr(knn, "knn"), n, d_in, d_out, _dev_ptr(out_graph, "out_graph"),
                                    _dev_ptr(workspace, "workspace"), workspace.numel(), _stream(stream)))
    if stream is not None:
        workspace.record_stream(stream)
    return out_graph


def ann_calibration_gather(h: Handle, ids: torch.Tensor, sink: torch.Tensor = None, stream=None) -> torch.Tensor:
    """Reads the rows of `ids` (int32, any shape) and xors them into `sink` (one int32, zeroed here if not given)."""
    if ids.dtype != torch.int32 or not ids.is_contiguous():
        raise ValueError("ids must be a contiguous int32 tensor")
    if sink is None:
        sink = torch.zeros(1, dtype=torch.int32, device=ids.device)
    if sink.dtype != torch.int32 or sink.numel() != 1:
        raise ValueError("sink must hold one int32")
    _check(lib().ann_calibration_gather(h.ptr, _dev_ptr(ids, "ids"), ids.numel(), _dev_ptr(sink, "sink"), _stream(stream)))
    return sink

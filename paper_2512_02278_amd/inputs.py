"""Seeded synthetic inputs: vector partitions, proximity graphs, queries, ground truth.

Nothing here belongs to the search method.  These generators produce the
*inputs* that both the GPU library and the CPU oracle are run on (the same
arrays go to both), plus exact brute-force neighbours for recall.  They stand in
for SIFT-, Deep- and text-embedding-style collections, which are not available
offline; only their shapes, dtypes and clustered structure are imitated.

All functions take a torch device, so the tiny cases run on the CPU and the
large ones are generated directly in HBM.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import torch

L2, IP = 0, 1


@dataclasses.dataclass
class Partition:
    """One GPU's share of an index, stored cluster-sorted (cluster = contiguous id range)."""

    vectors: torch.Tensor  # [n, dim] uint8 / float16 / float32
    centres: torch.Tensor  # [n_clusters, dim], same dtype as vectors
    offsets: torch.Tensor  # [n_clusters + 1] int64
    metric: int
    graph: Optional[torch.Tensor] = None  # [n, degree] int32


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _cluster_sizes(n: int, n_centres: int, g: torch.Generator, device) -> torch.Tensor:
    """Sizes of a uniform mixture: every vector picks its centre uniformly at random."""
    sizes = torch.zeros(n_centres, dtype=torch.int64, device=device)
    step = 1 << 26
    for lo in range(0, n, step):
        lab = torch.randint(0, n_centres, (min(step, n - lo),), generator=g, device=device)
        sizes += torch.bincount(lab, minlength=n_centres)
    return sizes


def _offsets(sizes: torch.Tensor) -> torch.Tensor:
    off = torch.zeros(sizes.numel() + 1, dtype=torch.int64, device=sizes.device)
    off[1:] = torch.cumsum(sizes, 0)
    return off


def _fill_clustered(out: torch.Tensor, centres_f32: torch.Tensor, offsets: torch.Tensor, sigma: float,
                    g: torch.Generator, finish) -> None:
    """out[off[c]:off[c+1]] = finish(centre_c + sigma * N(0, I)), a few million rows at a time."""
    n, dim = out.shape
    n_centres = centres_f32.shape[0]
    sizes = offsets[1:] - offsets[:-1]
    rows_per_step = 1 << 21
    off_cpu = offsets.cpu()
    c = 0
    while c < n_centres:
        c_hi = c + 1
        while c_hi < n_centres and int(off_cpu[c_hi + 1] - off_cpu[c]) <= rows_per_step:
            c_hi += 1
        lo, hi = int(off_cpu[c]), int(off_cpu[c_hi])
        if hi > lo:
            lab = torch.repeat_interleave(torch.arange(c, c_hi, device=out.device), sizes[c:c_hi])
            x = centres_f32[lab] + sigma * torch.randn((hi - lo, dim), generator=g, device=out.device)
            out[lo:hi] = finish(x)
        c = c_hi


def _u8(x: torch.Tensor) -> torch.Tensor:
    return x.round().clamp_(0, 255).to(torch.uint8)


def sift_like(n: int, n_centres: int, dim: int = 128, sigma: float = 20.0, seed: int = 20251202,
              device="cpu") -> Partition:
    """uint8 Gaussian mixture: centres uniform on 0..255, noise sigma, rounded and clipped."""
    g = _gen(seed, device)
    centres = torch.randint(0, 256, (n_centres, dim), generator=g, device=device, dtype=torch.uint8)
    offsets = _offsets(_cluster_sizes(n, n_centres, g, device))
    vectors = torch.empty((n, dim), dtype=torch.uint8, device=device)
    _fill_clustered(vectors, centres.float(), offsets, sigma, g, _u8)
    return Partition(vectors, centres, offsets, L2)


def sift_like_queries(part: Partition, nq: int, sigma: float = 20.0, seed: int = 20251203) -> torch.Tensor:
    """Queries from the same mixture, in drawn (random-cluster) order."""
    dev = part.vectors.device
    g = _gen(seed, dev)
    lab = torch.randint(0, part.centres.shape[0], (nq,), generator=g, device=dev)
    x = part.centres.float()[lab] + sigma * torch.randn((nq, part.centres.shape[1]), generator=g, device=dev)
    return _u8(x)


def unit_mixture(n: int, n_centres: int, dim: int, dtype: torch.dtype, metric: int, rho: float = 0.5,
                 seed: int = 20251202, device="cpu") -> Partition:
    """Unit-normalised Gaussian mixture (Deep-like fp32 d=96, text-like fp16 d=768).

    Centres are unit vectors; a vector is normalise(centre + sigma * N(0, I)) with
    sigma = rho / sqrt(dim), i.e. rho is the noise norm relative to the centre norm.
    """
    g = _gen(seed, device)
    centres = torch.nn.functional.normalize(torch.randn((n_centres, dim), generator=g, device=device), dim=1)
    offsets = _offsets(_cluster_sizes(n, n_centres, g, device))
    vectors = torch.empty((n, dim), dtype=dtype, device=device)
    sigma = rho / dim ** 0.5
    _fill_clustered(vectors, centres, offsets, sigma, g,
                    lambda x: torch.nn.functional.normalize(x, dim=1).to(dtype))
    return Partition(vectors, centres.to(dtype), offsets, metric)


def unit_mixture_queries(part: Partition, nq: int, rho: float = 0.5, seed: int = 20251203) -> torch.Tensor:
    dev = part.vectors.device
    dim = part.centres.shape[1]
    g = _gen(seed, dev)
    lab = torch.randint(0, part.centres.shape[0], (nq,), generator=g, device=dev)
    x = part.centres.float()[lab] + (rho / dim ** 0.5) * torch.randn((nq, dim), generator=g, device=dev)
    return torch.nn.functional.normalize(x, dim=1).to(part.vectors.dtype)


# --------------------------------------------------------------------------- exact neighbours


def _keys_block(x: torch.Tensor, y: torch.Tensor, metric: int) -> torch.Tensor:
    """key(x_i, y_j) as fp32 [len(x), len(y)].

    uint8 rows: computed through an fp16 GEMM with fp32 accumulation, which is exact
    (every value and every partial sum is an integer below 2^24 for dim <= 128).
    Float rows: an fp32 GEMM; good to rounding, which is all a ground truth for
    recall needs.
    """
    if x.dtype == torch.uint8:
        if x.device.type == "cpu":
            xf, yf = x.float(), y.float()
            g = xf @ yf.T
        else:
            xf, yf = x.half(), y.half()
            g = torch.mm(xf, yf.T, out_dtype=torch.float32)
            xf, yf = x.float(), y.float()
    else:
        xf, yf = x.float(), y.float()
        g = xf @ yf.T
    if metric == IP:
        return g.neg_()
    xx = (xf * xf).sum(1, keepdim=True)
    yy = (yf * yf).sum(1, keepdim=True)
    return g.mul_(-2.0).add_(xx).add_(yy.T)


def _topk_by_key_then_id(keys: torch.Tensor, ids: torch.Tensor, k: int) -> torch.Tensor:
    """Per row, the ids of the k smallest keys with ties broken by smaller id.

    keys [r, m] fp32, ids [m] int64 (strictly increasing or not: compared by value).
    Rows whose k-th and (k+1)-th keys tie are redone with an exact two-level sort;
    the others only need their k winners put in (key, id) order.
    """
    r, m = keys.shape
    kk = min(k + 1, m)
    vals, idx = torch.topk(keys, kk, dim=1, largest=False, sorted=True)
    got = ids[idx]
    if kk > k:
        tie = vals[:, k - 1] == vals[:, k]
        if bool(tie.any()):
            rows = tie.nonzero().squeeze(1)
            sub = keys[rows]
            order = torch.argsort(ids, stable=True)
            sub = sub[:, order]
            sid = ids[order]
            o2 = torch.argsort(sub, dim=1, stable=True)[:, :kk]  # stable: equal keys stay in id order
            vals[rows] = torch.gather(sub, 1, o2)
            got[rows] = sid[o2]
    vals, got = vals[:, :k], got[:, :k]
    # order each row's winners by (key, id): sort by id first, then stably by key
    o = torch.argsort(got, dim=1, stable=True)
    vals, got = torch.gather(vals, 1, o), torch.gather(got, 1, o)
    o = torch.argsort(vals, dim=1, stable=True)
    return torch.gather(got, 1, o)


def knn_graph_exact(part: Partition, degree: int, block: int = 4096) -> torch.Tensor:
    """Out-graph of the exact `degree` nearest neighbours over the whole set, self excluded."""
    x = part.vectors
    n = x.shape[0]
    ids = torch.arange(n, device=x.device)
    graph = torch.full((n, degree), -1, dtype=torch.int32, device=x.device)
    for lo in range(0, n, block):
        hi = min(n, lo + block)
        keys = _keys_block(x[lo:hi], x, part.metric)
        keys[torch.arange(hi - lo, device=x.device), torch.arange(lo, hi, device=x.device)] = float("inf")
        kk = min(degree, n - 1)
        graph[lo:hi, :kk] = _topk_by_key_then_id(keys, ids, kk).to(torch.int32)
    part.graph = graph
    return graph


def knn_graph_clustered(part: Partition, degree: int, n_near: int = 4, row_block: int = 8192,
                        progress=None) -> torch.Tensor:
    """Cluster-restricted exact kNN graph.

    A vector's candidates are the members of its own cluster and of the n_near
    clusters whose centres are nearest to its own cluster's centre; among them the
    `degree` nearest under (key, id), self excluded.  Rows with fewer candidates
    are padded with -1.
    """
    x = part.vectors
    dev = x.device
    n = x.shape[0]
    n_clusters = part.centres.shape[0]
    graph = torch.full((n, degree), -1, dtype=torch.int32, device=dev)
    ck = _keys_block(part.centres, part.centres, part.metric)
    ck.fill_diagonal_(float("inf"))
    near = torch.topk(ck, min(n_near, n_clusters - 1), dim=1, largest=False).indices.cpu() if n_clusters > 1 else None
    off = part.offsets.cpu().tolist()
    for c in range(n_clusters):
        lo, hi = off[c], off[c + 1]
        if hi == lo:
            continue
        members = [c] + (near[c].tolist() if near is not None else [])
        ids = torch.cat([torch.arange(off[m], off[m + 1], device=dev) for m in members])
        y = x[ids]
        for rlo in range(lo, hi, row_block):
            rhi = min(hi, rlo + row_block)
            keys = _keys_block(x[rlo:rhi], y, part.metric)
            # own cluster comes first in `ids`, so row r's own column is (r - lo)
            keys[torch.arange(rhi - rlo, device=dev), torch.arange(rlo - lo, rhi - lo, device=dev)] = float("inf")
            kk = min(degree, ids.numel() - 1)
            if kk > 0:
                graph[rlo:rhi, :kk] = _topk_by_key_then_id(keys, ids, kk).to(torch.int32)
        if progress is not None and (c + 1) % progress[1] == 0:
            progress[0](c + 1, n_clusters)
    part.graph = graph
    return graph


def ground_truth(part: Partition, queries: torch.Tensor, k: int, col_block: int = 1 << 20,
                 row_block: int = 1024) -> torch.Tensor:
    """Exact top-k ids [nq, k] int32 over the whole partition under (key, id).

    row_block * col_block stays below 2^31 elements (index arithmetic of the library's nonzero)."""
    x = part.vectors
    dev = x.device
    n = x.shape[0]
    out = torch.empty((queries.shape[0], k), dtype=torch.int32, device=dev)
    for qlo in range(0, queries.shape[0], row_block):
        q = queries[qlo:qlo + row_block]
        # pass 1: the k-th smallest key per query (its value does not depend on tie order)
        best = torch.full((q.shape[0], k), float("inf"), device=dev)
        for lo in range(0, n, col_block):
            keys = _keys_block(q, x[lo:lo + col_block], part.metric)
            v = torch.topk(keys, min(k, keys.shape[1]), dim=1, largest=False).values
            best = torch.topk(torch.cat([best, v], 1), k, dim=1, largest=False).values
        kth = best[:, k - 1:k]
        # pass 2: everything at or below that key, then cut by (key, id)
        rows, cols, vals = [], [], []
        for lo in range(0, n, col_block):
            keys = _keys_block(q, x[lo:lo + col_block], part.metric)
            r, c = (keys <= kth).nonzero(as_tuple=True)
            rows.append(r)
            cols.append(c + lo)
            vals.append(keys[r, c])
        rows, cols, vals = torch.cat(rows), torch.cat(cols), torch.cat(vals)
        o = torch.argsort(cols, stable=True)
        rows, cols, vals = rows[o], cols[o], vals[o]
        o = torch.argsort(vals, stable=True)
        rows, cols, vals = rows[o], cols[o], vals[o]
        o = torch.argsort(rows, stable=True)
        rows, cols = rows[o], cols[o]
        start = torch.searchsorted(rows, torch.arange(q.shape[0], device=dev))
        pick = start[:, None] + torch.arange(k, device=dev)[None, :]
        valid = pick < rows.numel()
        pick = pick.clamp_(max=max(rows.numel() - 1, 0))
        ok = valid & (rows[pick] == torch.arange(q.shape[0], device=dev)[:, None])
        out[qlo:qlo + q.shape[0]] = torch.where(ok, cols[pick], torch.full_like(pick, -1)).to(torch.int32)
    return out


def recall_per_query(found: torch.Tensor, truth: torch.Tensor) -> torch.Tensor:
    """|found ∩ truth| / k for every query, float64 [nq] (ids of -1 never match; a repeated id counts once)."""
    f = found.to(torch.int64)
    t = truth.to(torch.int64).to(f.device)
    out = torch.empty(t.shape[0], dtype=torch.float64, device=f.device)
    for lo in range(0, t.shape[0], 4096):
        tt, ff = t[lo:lo + 4096], f[lo:lo + 4096]
        out[lo:lo + 4096] = ((tt[:, :, None] == ff[:, None, :]) & (tt[:, :, None] >= 0)).any(2).double().sum(1) / t.shape[1]
    return out


def recall(found: torch.Tensor, truth: torch.Tensor) -> float:
    """Mean over queries of |found ∩ truth| / k."""
    return float(recall_per_query(found, truth).mean())


def graph_stats(part: Partition) -> dict:
    """Fraction of edges that leave their cluster, and the fraction of empty slots."""
    g = part.graph.to(torch.int64)
    n = g.shape[0]
    lab = torch.searchsorted(part.offsets, torch.arange(n, device=g.device), right=True) - 1
    valid = g >= 0
    cross = (lab[g.clamp(min=0)] != lab[:, None]) & valid
    return {"cross_cluster_edge_fraction": float(cross.sum() / valid.sum().clamp(min=1)),
            "empty_slot_fraction": float((~valid).float().mean())}

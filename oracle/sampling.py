"""Rows of the optimized graph for a few nodes of a large graph, by the oracle.  TEST INFRASTRUCTURE ONLY.

A row of the result depends on little of the input: the node's own kNN row, the rows of every node
that lists it (they may point back at it after pruning), and the rows of all those nodes' neighbours
(their detour counts read them).  This module cuts that subgraph out (torch tensor ops on whatever
device holds the kNN lists; no arithmetic of the method), relabels its ids in ascending order, which
keeps the order of sources that the reverse lists use, and hands it to oracle.graph_optimize.  An id
outside the subgraph becomes absent in place: ranks stay what they were, and no count of a row that
matters can change, because every neighbour of such a row is inside.
"""
from __future__ import annotations

import numpy as np
import torch

from . import graph_optimize


def optimized_rows(knn: torch.Tensor, nodes, d_out: int) -> np.ndarray:
    """knn [n, d_in] int32 (any device), nodes: distinct ids -> rows of the optimized graph, [len(nodes), d_out]."""
    n = knn.shape[0]
    nodes = np.asarray(nodes, dtype=np.int64)
    nodes_t = torch.as_tensor(nodes, device=knn.device, dtype=torch.int32)
    listing = torch.zeros(n, dtype=torch.bool, device=knn.device)
    step = max(1, (1 << 28) // knn.shape[1])  # bound the size of the temporary mask
    for lo in range(0, n, step):
        listing[lo:lo + step] = torch.isin(knn[lo:lo + step], nodes_t).any(dim=1)
    first = torch.unique(torch.cat([listing.nonzero().flatten(), nodes_t.long()]))
    nb = knn[first].flatten().long()
    nb = nb[(nb >= 0) & (nb < n)]
    keep = torch.unique(torch.cat([first, nb]))  # ascending
    sub = knn[keep].long()
    pos = torch.searchsorted(keep, sub.clamp(0, n - 1)).clamp(max=keep.numel() - 1)
    inside = (sub >= 0) & (sub < n) & (keep[pos] == sub)
    sub = torch.where(inside, pos, torch.full_like(pos, -1)).to(torch.int32).cpu().numpy()
    out = graph_optimize(sub, d_out)
    keep_np = keep.cpu().numpy()
    rows = out[np.searchsorted(keep_np, nodes)]
    return np.where(rows >= 0, keep_np[np.clip(rows, 0, None)], -1).astype(np.int32)

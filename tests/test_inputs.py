"""The seeded input generators: what the workload recipe promises, checked on the CPU."""
import numpy as np
import torch

from paper_2512_02278_amd import inputs


def test_sift_like_is_seeded_cluster_sorted_uint8():
    a = inputs.sift_like(5000, 20, seed=3)
    b = inputs.sift_like(5000, 20, seed=3)
    c = inputs.sift_like(5000, 20, seed=4)
    assert torch.equal(a.vectors, b.vectors) and torch.equal(a.offsets, b.offsets) and torch.equal(a.centres, b.centres)
    assert not torch.equal(a.vectors, c.vectors)
    assert a.vectors.dtype == torch.uint8 and a.vectors.shape == (5000, 128) and a.centres.shape == (20, 128)
    off = a.offsets.tolist()
    assert off[0] == 0 and off[-1] == 5000 and all(x <= y for x, y in zip(off, off[1:]))
    # members of a cluster sit around their centre (sigma 20, clipped): far closer than to other centres
    x, cen = a.vectors.float(), a.centres.float()
    lab = torch.searchsorted(a.offsets, torch.arange(5000), right=True) - 1
    d = torch.cdist(x, cen)
    assert (d.argmin(1) == lab).all()
    assert 150 < d[torch.arange(5000), lab].mean() < 300     # about 20 * sqrt(128) = 226


def test_queries_come_from_the_same_mixture_in_drawn_order():
    part = inputs.sift_like(2000, 50, seed=1)
    q = inputs.sift_like_queries(part, 400, seed=2)
    assert q.dtype == torch.uint8 and q.shape == (400, 128)
    lab = torch.cdist(q.float(), part.centres.float()).argmin(1)
    assert len(set(lab.tolist())) > 30                       # many clusters
    assert (lab[1:] < lab[:-1]).any()                        # not sorted by cluster


def test_unit_mixture_is_unit_norm_and_typed():
    for dtype, metric in ((torch.float32, inputs.L2), (torch.float16, inputs.IP)):
        part = inputs.unit_mixture(3000, 16, 64, dtype, metric, seed=5)
        assert part.vectors.dtype == dtype and part.centres.dtype == dtype and part.metric == metric
        n = part.vectors.float().norm(dim=1)
        assert (n - 1).abs().max() < (2e-3 if dtype == torch.float16 else 1e-5)
        q = inputs.unit_mixture_queries(part, 10, seed=6)
        assert q.dtype == dtype and ((q.float().norm(dim=1) - 1).abs() < 2e-3).all()


def test_clustered_graph_is_exact_knn_among_its_candidates():
    part = inputs.sift_like(3000, 12, dim=32, seed=7)
    g = inputs.knn_graph_clustered(part, 8, n_near=2)
    assert g.dtype == torch.int32 and g.shape == (3000, 8)
    x = part.vectors.numpy().astype(np.int64)
    cen = part.centres.numpy().astype(np.int64)
    off = part.offsets.numpy()
    cd = ((cen[:, None, :] - cen[None, :, :]) ** 2).sum(2)
    np.fill_diagonal(cd, np.iinfo(np.int64).max)
    for i in (0, 777, 1500, 2999):
        c = int(np.searchsorted(off, i, side="right") - 1)
        near = np.argsort(cd[c], kind="stable")[:2]
        cand = np.concatenate([np.arange(off[m], off[m + 1]) for m in [c, *near]])
        cand = cand[cand != i]
        d = ((x[cand] - x[i]) ** 2).sum(1)
        want = cand[np.lexsort((cand, d))[:8]]
        assert g[i].tolist() == want.tolist()
    assert (g != torch.arange(3000, dtype=torch.int32)[:, None]).all()   # self excluded
    stats = inputs.graph_stats(part)
    assert 0.0 <= stats["cross_cluster_edge_fraction"] <= 1.0 and stats["empty_slot_fraction"] == 0.0


def test_recall_counts_matches_and_ignores_padding():
    found = torch.tensor([[1, 2, 3, -1], [9, 9, 9, 9]], dtype=torch.int32)
    truth = torch.tensor([[3, 2, 7, 8], [9, 1, 2, 3]], dtype=torch.int32)
    # query 0 finds two of four; query 1 lists one true neighbour four times: it counts once
    assert abs(inputs.recall(found, truth) - (2 + 1) / 8) < 1e-9


def test_bench_refuses_more_than_one_gpu():
    """The build covers one GPU's partition: bench.py --gpus N (N > 1) must say so and exit non-zero."""
    import os
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and not r.stdout.strip()

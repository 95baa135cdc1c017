"""GPU graph construction (ann_graph_prune, ann_graph_optimize) against the CPU oracle: integer work,
so every entry must be identical."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    if not torch.cuda.is_available():
        pytest.fail("these tests need the MI355X (run with -m 'not gpu' elsewhere)")
    return torch


def random_knn(rng, n, d_in, holes=0.0, junk=0.0):
    """Rows of distinct ids != x in random order, some entries absent (-1, out of range, self)."""
    if d_in < n:
        knn = np.stack([rng.permutation(np.delete(np.arange(n), x))[:d_in] for x in range(n)]).astype(np.int32)
    else:
        knn = np.full((n, d_in), -1, np.int32)
        for x in range(n):
            knn[x, : n - 1] = rng.permutation(np.delete(np.arange(n), x))
    if holes:
        knn[rng.random(knn.shape) < holes] = -1
    if junk:
        m = rng.random(knn.shape) < junk
        knn[m] = rng.choice(np.array([-7, n, n + 3, 2**31 - 1], dtype=np.int64), size=int(m.sum())).astype(np.int32)
        rows = np.nonzero(rng.random(n) < junk)[0]
        knn[rows, rng.integers(0, d_in, rows.size)] = rows
    return knn


def data_knn(n, n_centres, d_in, seed):
    """Exact kNN lists of clustered uint8 vectors: the real input, with many mutual edges and shared neighbours."""
    import torch

    from paper_2512_02278_amd import inputs

    part = inputs.sift_like(n, n_centres, seed=seed, device=torch.device("cuda:0"))
    return inputs.knn_graph_exact(part, d_in).cpu().numpy()


def gpu_prune(torch, knn, d_out):
    from paper_2512_02278_amd import ann

    out = ann.ann_graph_prune(torch.from_numpy(knn).to("cuda:0"), d_out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_optimize(torch, knn, d_out):
    from paper_2512_02278_amd import ann

    out = ann.ann_graph_optimize(torch.from_numpy(knn).to("cuda:0"), d_out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check_both(oracle, torch, knn, d_out):
    want = oracle.graph_prune(knn, d_out)
    got = gpu_prune(torch, knn, d_out)
    assert np.array_equal(got, want), f"pruned rows differ: {np.argwhere(got != want)[:5].tolist()}"
    want = oracle.graph_optimize(knn, d_out)
    got = gpu_optimize(torch, knn, d_out)
    assert np.array_equal(got, want), f"optimized rows differ: {np.argwhere(got != want)[:5].tolist()}"


@pytest.mark.parametrize("n,n_centres,d_in,d_out,seed", [
    (3000, 10, 64, 32, 1),    # the headline shape: 64 -> 32
    (2500, 5, 128, 64, 2),    # two registers per lane, the largest degrees
    (2000, 8, 48, 17, 3),     # degrees that are no power of two, odd d_out
    (1500, 6, 96, 40, 4),
    (1000, 4, 16, 16, 5),     # no cut: the row is only reordered
])
def test_knn_lists_of_clustered_data(oracle, torch_cuda, n, n_centres, d_in, d_out, seed):
    check_both(oracle, torch_cuda, data_knn(n, n_centres, d_in, seed), d_out)


@pytest.mark.parametrize("n,d_in,d_out,holes,junk,seed", [
    (1, 4, 2, 0.0, 0.0, 1),        # a single node: every entry absent
    (2, 1, 1, 0.0, 0.0, 2),
    (33, 8, 3, 0.0, 0.0, 3),       # one node beyond a run of 32
    (261, 20, 7, 0.2, 0.05, 4),    # eight runs and a ragged ninth
    (700, 64, 64, 0.3, 0.05, 5),
    (300, 128, 1, 0.1, 0.0, 6),
    (90, 128, 64, 0.0, 0.0, 7),    # rows longer than the graph has nodes
    (500, 30, 9, 0.1, 0.05, 8),    # row length no multiple of four: one id per lane and load
    (400, 70, 33, 0.1, 0.0, 9),    # the same with two registers per lane
])
def test_random_lists_with_absent_entries(oracle, torch_cuda, n, d_in, d_out, holes, junk, seed):
    rng = np.random.default_rng(seed)
    check_both(oracle, torch_cuda, random_knn(rng, n, d_in, holes, junk), d_out)


def test_rows_that_do_not_start_on_16_bytes(oracle, torch_cuda):
    """kNN lists whose base address is only 4-byte aligned take the one-id-per-lane loads."""
    from paper_2512_02278_amd import ann

    torch = torch_cuda
    rng = np.random.default_rng(12)
    knn = random_knn(rng, 600, 32, holes=0.1)
    flat = torch.empty(600 * 32 + 1, dtype=torch.int32, device="cuda:0")
    view = flat[1:].view(600, 32)
    view.copy_(torch.from_numpy(knn))
    assert view.data_ptr() % 16 == 4 and view.is_contiguous()
    got = ann.ann_graph_optimize(view, 16)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.graph_optimize(knn, 16))


def test_hubs_with_thousands_of_in_edges(oracle, torch_cuda):
    """Every node lists the same few hubs first, so their reverse lists are cut from thousands of
    candidates that arrive in many 64-word chunks."""
    rng = np.random.default_rng(11)
    n, d_in, d_out = 5000, 24, 12
    knn = random_knn(rng, n, d_in)
    for x in range(n):
        hubs = [hb for hb in (0, 1, 2, 4999) if hb != x]
        rest = [v for v in knn[x].tolist() if v not in hubs]
        knn[x] = (hubs + rest)[:d_in]
    check_both(oracle, torch_cuda, knn, d_out)


def test_bad_workspace_is_refused(torch_cuda):
    from paper_2512_02278_amd import ann

    torch = torch_cuda
    knn = torch.zeros((100, 8), dtype=torch.int32, device="cuda:0")
    need = ann.ann_graph_optimize_workspace_bytes(100, 8, 4)
    with pytest.raises(ann.AnnError):
        ann.ann_graph_optimize(knn, 4, workspace=torch.empty(need - 1, dtype=torch.uint8, device="cuda:0"))
    with pytest.raises(ann.AnnError):
        ann.ann_graph_optimize(knn, 4, workspace=torch.empty(need + 64, dtype=torch.uint8, device="cuda:0")[8:])
    with pytest.raises(ann.AnnError):
        ann.ann_graph_optimize(knn, 9)


def test_million_node_graph_sampled(oracle, torch_cuda):
    """The 1M-vector configuration's shape (cluster-restricted kNN, 64 -> 32), checked on sampled rows."""
    torch = torch_cuda
    from paper_2512_02278_amd import ann, inputs

    part = inputs.sift_like(1_000_000, 1000, seed=5, device=torch.device("cuda:0"))
    knn = inputs.knn_graph_clustered(part, 64)
    out = ann.ann_graph_optimize(knn, 32)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    nodes = np.unique(np.concatenate([[0, 31, 32, 999_999], rng.integers(0, 1_000_000, 60)]))
    from oracle import sampling

    want = sampling.optimized_rows(knn, nodes, 32)
    got = out[torch.as_tensor(nodes, device=out.device)].cpu().numpy()
    assert np.array_equal(got, want)
    # whole-graph properties: full rows, distinct ids, no self loops
    assert int((out < 0).sum()) == 0
    srt = torch.sort(out, dim=1).values
    assert int((srt[:, 1:] == srt[:, :-1]).sum()) == 0
    assert int((out == torch.arange(out.shape[0], device=out.device, dtype=torch.int32)[:, None]).sum()) == 0


def test_search_on_the_graph_the_gpu_built(oracle, torch_cuda):
    """The whole path at small size: kNN lists -> ann_graph_optimize -> ann_search on that graph, both against
    the oracle (graph rows identical, then ids and int32 keys of the search identical)."""
    torch = torch_cuda
    from paper_2512_02278_amd import ann, inputs

    part = inputs.sift_like(20_000, 20, seed=9, device=torch.device("cuda:0"))
    knn = inputs.knn_graph_clustered(part, 48)
    graph = ann.ann_graph_optimize(knn, 24)
    torch.cuda.synchronize()
    want_graph = oracle.graph_optimize(knn.cpu().numpy(), 24)
    assert np.array_equal(graph.cpu().numpy(), want_graph)
    q = inputs.sift_like_queries(part, 500)
    h = ann.ann_index_load(part.vectors, graph, n_entry=32, entry_mode=ann.ANN_ENTRY_ROUTED, seed=5,
                           centroids=part.centres, cluster_offsets=part.offsets, route_c=2)
    cnt = torch.zeros((500, 4), dtype=torch.int32, device="cuda:0")
    ids, dists = ann.ann_search(h, q, 10, 96, 4, 100, counters=cnt)
    torch.cuda.synchronize()
    ann.ann_free(h)
    ix = oracle.Index(part.vectors.cpu().numpy(), want_graph, n_entry=32, entry_mode=1, seed=5,
                      centroids=part.centres.cpu().numpy(), cluster_offsets=part.offsets.cpu().numpy(), route_c=2)
    oi, od, oc = oracle.search(ix, q.cpu().numpy(), 10, 96, 4, 100)
    assert np.array_equal(ids.cpu().numpy(), oi) and np.array_equal(dists.cpu().numpy(), od)
    assert np.array_equal(cnt[:, 0].cpu().numpy(), oc["iters"])
    truth = inputs.ground_truth(part, q, 10)
    assert inputs.recall(ids, truth) > 0.95

"""Pins for the CPU oracle: what the mathematics and the paper fix, checked without a GPU.

Each test is built so that a plausible mistake in oracle/beam_search.c (a dropped
term or wrong sign in the key, a transposed index, a broken tie-break, a merge that
loses entries, a termination or flag bug, a wrong counter) fails at least one.
"""
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
NP_DT = {"u8": np.uint8, "f16": np.float16, "f32": np.float32}


# ----------------------------------------------------------------------------- helpers
def np_keys(q, x, metric):
    """key(q, x_i) for every row: the textbook definition in int64 / float64."""
    if x.dtype == np.uint8:
        a, b = q.astype(np.int64), x.astype(np.int64)
        return ((a[None, :] - b) ** 2).sum(1) if metric == 0 else -(a[None, :] * b).sum(1)
    a, b = q.astype(np.float64), x.astype(np.float64)
    k = ((a[None, :] - b) ** 2).sum(1) if metric == 0 else -(a[None, :] * b).sum(1)
    return k.astype(np.float32)


def np_topk(q, x, ids, metric, k):
    """Brute-force top-k over the rows listed in `ids`, ordered by (key, id)."""
    ids = np.asarray(sorted(ids), dtype=np.int64)
    keys = np_keys(q, x[ids], metric)
    order = np.lexsort((ids, keys))[:k]
    return ids[order], keys[order]


def random_vectors(rng, n, dim, dt):
    if dt == "u8":
        return rng.integers(0, 256, (n, dim), dtype=np.uint8)
    return rng.standard_normal((n, dim)).astype(NP_DT[dt])


def random_graph(rng, n, degree, ring=True, holes=0.0):
    g = rng.integers(0, n, (n, degree), dtype=np.int32)
    if ring:
        g[:, 0] = (np.arange(n) + 1) % n  # a ring edge makes the graph strongly connected
    if holes:
        g[rng.random((n, degree)) < holes] = -1
        if ring:
            g[:, 0] = (np.arange(n) + 1) % n
    return g


def reachable(graph, entries):
    seen, todo = set(int(e) for e in entries), [int(e) for e in entries]
    while todo:
        for v in graph[todo.pop()]:
            v = int(v)
            if 0 <= v < graph.shape[0] and v not in seen:
                seen.add(v)
                todo.append(v)
    return seen


def pad_expect(ids, keys, k, is_u8):
    out_i = np.full(k, -1, np.int64)
    out_k = np.full(k, np.iinfo(np.int32).max if is_u8 else np.inf, np.float64)
    out_i[: len(ids)] = ids
    out_k[: len(ids)] = keys
    return out_i, out_k


# ----------------------------------------------------------------------------- generator
def test_entry_generator_published_vectors(oracle):
    """Entry ids come from the splitmix64 stream of `seed`; for seed 0 its first three
    outputs are the widely published test values of that generator."""
    first3 = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    n = 2**31 - 1
    x = np.zeros((n.bit_length(), 4), np.uint8)  # vectors are not read by the entry rule
    ix = oracle.Index(x, np.zeros((x.shape[0], 1), np.int32), n_entry=3, seed=0)
    ix.n = n
    e = oracle.entries(ix, np.zeros((2, 4), np.uint8))
    assert e[0].tolist() == [z % n for z in first3]
    # query 1 continues the same stream at counter n_entry*1 + j (outputs 4..6): all distinct from query 0
    assert len(set(e[0].tolist()) | set(e[1].tolist())) == 6


def test_entries_differ_per_query_and_seed(oracle):
    x = np.zeros((1000, 4), np.uint8)
    g = np.zeros((1000, 1), np.int32)
    q = np.zeros((5, 4), np.uint8)
    a = oracle.entries(oracle.Index(x, g, n_entry=32, seed=7), q)
    b = oracle.entries(oracle.Index(x, g, n_entry=32, seed=8), q)
    assert a.min() >= 0 and a.max() < 1000
    assert not np.array_equal(a[0], a[1]) and not np.array_equal(a, b)
    # uniform over [0, n): a crude chi-square-free check on the mean
    big = oracle.entries(oracle.Index(x, g, n_entry=64, seed=1), np.zeros((500, 4), np.uint8))
    assert abs(big.mean() - 499.5) < 10


# ----------------------------------------------------------------------------- brute force (P8)
@pytest.mark.parametrize("dt", ["u8", "f16", "f32"])
@pytest.mark.parametrize("metric", [0, 1])
def test_bruteforce_is_the_definition(oracle, dt, metric):
    rng = np.random.default_rng(1)
    x = random_vectors(rng, 300, 24, dt)
    if dt == "u8":
        x[:, :] = rng.integers(0, 4, x.shape)  # few distinct values: many exact key ties
    q = x[rng.integers(0, 300, 7)].copy() if dt == "u8" else random_vectors(rng, 7, 24, dt)
    ids, dists = oracle.bruteforce(x, q, 12, metric)
    for i in range(len(q)):
        ei, ek = np_topk(q[i], x, range(300), metric, 12)
        assert ids[i].tolist() == ei.tolist()
        assert np.array_equal(dists[i].astype(np.float64), ek.astype(np.float64))


def test_bruteforce_padded_rows_and_k_above_n(oracle):
    rng = np.random.default_rng(2)
    buf = rng.integers(0, 256, (5, 48), dtype=np.uint8)
    x = buf[:, :16]  # row stride 48 bytes, 16 used
    q = rng.integers(0, 256, (2, 16), dtype=np.uint8)
    ids, dists = oracle.bruteforce(x, q, 8, 0)
    for i in range(2):
        ei, ek = np_topk(q[i], np.ascontiguousarray(x), range(5), 0, 8)
        wi, wk = pad_expect(ei, ek, 8, True)
        assert ids[i].tolist() == wi.tolist() and dists[i].tolist() == wk.tolist()


def test_ground_truth_generator_agrees_with_bruteforce(oracle):
    """The torch ground truth used for recall at scale equals the oracle's brute force."""
    import torch

    from paper_2512_02278_amd import inputs

    part = inputs.sift_like(3000, 10, dim=32, seed=5)
    q = inputs.sift_like_queries(part, 40, seed=6)
    gt = inputs.ground_truth(part, q, 10, col_block=700, row_block=16)
    ids, _ = oracle.bruteforce(part.vectors.numpy(), q.numpy(), 10, 0)
    assert np.array_equal(gt.numpy(), ids)
    # tie-heavy case: 2-bit coordinates
    part.vectors = torch.randint(0, 4, (3000, 32), dtype=torch.uint8, generator=torch.Generator().manual_seed(1))
    gt = inputs.ground_truth(part, part.vectors[:25], 10, col_block=700, row_block=16)
    ids, _ = oracle.bruteforce(part.vectors.numpy(), part.vectors[:25].numpy(), 10, 0)
    assert np.array_equal(gt.numpy(), ids)


# ----------------------------------------------------------------------------- P1 reachable-set rule
@pytest.mark.parametrize("dt", ["u8", "f16", "f32"])
@pytest.mark.parametrize("metric", [0, 1])
@pytest.mark.parametrize("ring", [True, False])
def test_reachable_set_rule(oracle, dt, metric, ring):
    """With itopk and max_iters >= |R| (R = nodes reachable from the entries) the list ends
    up holding all of R, so the output is brute force over R under (key, id).  On a
    strongly connected graph this is exact kNN."""
    rng = np.random.default_rng(10 + ring)
    n, dim, degree = 400, 20, 3
    x = random_vectors(rng, n, dim, dt)
    if dt == "u8":
        x %= 8  # ties
    g = random_graph(rng, n, degree, ring=ring, holes=0.2)
    q = random_vectors(rng, 12, dim, dt)
    ix = oracle.Index(x, g, metric=metric, n_entry=2, seed=3)
    ent = oracle.entries(ix, q)
    for width in (1, 3):
        ids, dists, cnt = oracle.search(ix, q, k=15, itopk=n, width=width, max_iters=n)
        for i in range(len(q)):
            R = reachable(g, ent[i])
            if ring:
                assert len(R) == n
            ei, ek = np_topk(q[i], x, R, metric, 15)
            wi, wk = pad_expect(ei, ek, 15, dt == "u8")
            assert ids[i].tolist() == wi.tolist()
            assert np.array_equal(dists[i].astype(np.float64), wk)
            assert cnt["n_dist"][i] == len(R)  # every reachable node scored exactly once
            assert cnt["n_parents"][i] == len(R)  # and expanded exactly once


def test_fewer_reachable_than_k_is_padded(oracle):
    n = 50
    x = np.arange(n, dtype=np.uint8)[:, None].repeat(4, 1)
    g = np.full((n, 2), -1, np.int32)  # no edges at all: R = the entries
    ix = oracle.Index(x, g, n_entry=3, seed=11)
    q = np.zeros((4, 4), np.uint8)
    ent = oracle.entries(ix, q)
    ids, dists, cnt = oracle.search(ix, q, k=6, itopk=8, width=2, max_iters=10)
    for i in range(4):
        R = sorted(set(ent[i].tolist()))
        assert ids[i].tolist() == R + [-1] * (6 - len(R))
        assert dists[i].tolist() == [4 * r * r for r in R] + [2**31 - 1] * (6 - len(R))
        assert cnt["n_dist"][i] == len(R)


# ----------------------------------------------------------------------------- P2 complete graph
@pytest.mark.parametrize("dt", ["u8", "f32"])
def test_complete_graph_one_round(oracle, dt):
    rng = np.random.default_rng(4)
    n = 60
    x = random_vectors(rng, n, 16, dt)
    g = np.array([[j for j in range(n) if j != i] for i in range(n)], np.int32)
    q = random_vectors(rng, 9, 16, dt)
    ix = oracle.Index(x, g, n_entry=1, seed=5)
    ids, dists, cnt = oracle.search(ix, q, k=10, itopk=n, width=1, max_iters=1)
    for i in range(9):
        ei, ek = np_topk(q[i], x, range(n), 0, 10)
        assert ids[i].tolist() == ei.tolist()
        assert np.array_equal(dists[i].astype(np.float64), ek.astype(np.float64))
        assert cnt["iters"][i] == 1 and cnt["n_dist"][i] == n and cnt["n_parents"][i] == 1


# ----------------------------------------------------------------------------- P3 path graph
@pytest.mark.parametrize("t", [0, 1, 7, 40])
def test_path_graph_closed_form(oracle, t):
    """x_i = i on a line, neighbours {i-1, i+1}, one entry at node 0 (routed mode with a
    single one-node cluster pins the entry), itopk = width = 1.  The walk takes one
    step right per round until the query position t, then one more round that finds
    nothing better: result t, t+1 rounds, t+2 keys computed, t+1 graph rows read."""
    n = 64
    x = np.zeros((n, 4), np.float32)
    x[:, 0] = np.arange(n)
    g = np.stack([np.arange(n) - 1, np.arange(n) + 1], 1).astype(np.int32)
    g[g >= n] = -1
    q = np.zeros((1, 4), np.float32)
    q[0, 0] = t
    ix = oracle.Index(x, g, n_entry=1, entry_mode=1, seed=9, centroids=x[:1].copy(),
                      cluster_offsets=np.array([0, 1]), route_c=1)
    ids, dists, cnt = oracle.search(ix, q, k=1, itopk=1, width=1, max_iters=1000)
    assert ids[0, 0] == t and dists[0, 0] == 0.0
    assert cnt["iters"][0] == t + 1 and cnt["n_dist"][0] == t + 2 and cnt["n_parents"][0] == t + 1
    # max_iters cuts the walk short: after m rounds the best node seen is min(m, t)
    ids, _, cnt = oracle.search(ix, q, k=1, itopk=1, width=1, max_iters=3)
    assert ids[0, 0] == min(3, t) and cnt["iters"][0] == min(3, t + 1)
    # max_iters = 0: only the entries are scored
    ids, _, cnt = oracle.search(ix, q, k=1, itopk=1, width=1, max_iters=0)
    assert ids[0, 0] == 0 and cnt["iters"][0] == 0 and cnt["n_dist"][0] == 1


# ----------------------------------------------------------------------------- P4 / P5 / P6
def _clustered_case(rng, dt, n=1500, dim=24, degree=8):
    centres = rng.integers(40, 216, (6, dim)).astype(np.float64)
    lab = np.sort(rng.integers(0, 6, n))
    x = centres[lab] + rng.standard_normal((n, dim)) * 12
    if dt == "u8":
        x = np.clip(np.rint(x), 0, 255).astype(np.uint8)
    else:
        x = (x / 64).astype(NP_DT[dt])
    # kNN graph by the textbook definition (float64), self excluded
    xx = x.astype(np.float64)
    d = ((xx[:, None, :] - xx[None, :, :]) ** 2).sum(2)
    np.fill_diagonal(d, np.inf)
    g = np.argsort(d, 1, kind="stable")[:, :degree].astype(np.int32)
    q = x[rng.integers(0, n, 30)].copy()
    if dt != "u8":
        q = (q.astype(np.float64) + rng.standard_normal(q.shape) * 0.05).astype(NP_DT[dt])
    else:
        q = np.clip(q.astype(np.int64) + rng.integers(-6, 7, q.shape), 0, 255).astype(np.uint8)
    return x, g, q


@pytest.mark.parametrize("dt", ["u8", "f16", "f32"])
@pytest.mark.parametrize("metric", [0, 1])
def test_output_invariants_and_slot_order(oracle, dt, metric):
    rng = np.random.default_rng(21)
    x, g, q = _clustered_case(rng, dt)
    ix = oracle.Index(x, g, metric=metric, n_entry=8, seed=2)
    ids, dists, cnt = oracle.search(ix, q, k=10, itopk=32, width=2, max_iters=40)
    n = x.shape[0]
    for i in range(len(q)):
        real = ids[i][ids[i] >= 0]
        assert len(set(real.tolist())) == len(real) and real.max() < n
        assert (ids[i] >= 0).all()  # 8 entries + neighbours always give at least k nodes here
        want = np_keys(q[i], x[real], metric).astype(np.float64)
        assert np.array_equal(dists[i].astype(np.float64), want)  # reported distance = recomputed key
        pairs = list(zip(dists[i].tolist(), ids[i].tolist()))
        assert pairs == sorted(pairs)  # ascending by (key, id)
        assert cnt["n_parents"][i] <= 2 * cnt["iters"][i] and cnt["iters"][i] <= 40
    # permuting the neighbour slots inside every graph row changes nothing
    perm = np.stack([rng.permutation(g.shape[1]) for _ in range(n)])
    g2 = np.take_along_axis(g, perm, 1)
    ids2, dists2, cnt2 = oracle.search(oracle.Index(x, g2, metric=metric, n_entry=8, seed=2), q, 10, 32, 2, 40)
    assert np.array_equal(ids, ids2) and np.array_equal(dists, dists2)
    assert np.array_equal(cnt["n_dist"], cnt2["n_dist"])
    # thread count changes nothing
    ids3, dists3, _ = oracle.search(ix, q, 10, 32, 2, 40, n_threads=1)
    assert np.array_equal(ids, ids3) and np.array_equal(dists, dists3)


@pytest.mark.parametrize("dt", ["u8", "f32"])
def test_keys_never_get_worse_with_more_rounds(oracle, dt):
    rng = np.random.default_rng(22)
    x, g, q = _clustered_case(rng, dt)
    ix = oracle.Index(x, g, n_entry=4, seed=5)
    prev = None
    for m in (0, 1, 2, 4, 8, 16, 64):
        _, dists, _ = oracle.search(ix, q, k=10, itopk=24, width=2, max_iters=m)
        d = dists.astype(np.float64)
        if prev is not None:
            assert (d <= prev).all()
        prev = d


@pytest.mark.parametrize("dt", ["u8", "f16", "f32"])
@pytest.mark.parametrize("width,itopk", [(1, 16), (4, 32), (3, 7)])
def test_forgetful_visited_set_gives_the_same_result(oracle, dt, width, itopk):
    """The list always holds the itopk best of everything scored so far and its worst key
    never rises, so a node scored twice is either still in the list or rejected again:
    forgetting the visited set (except list members) cannot change the outcome, only
    the number of keys computed.  This is what lets a GPU use a small visited table."""
    rng = np.random.default_rng(23)
    x, g, q = _clustered_case(rng, dt)
    if dt == "u8":
        x //= 16  # heavy ties
        q //= 16
    ix = oracle.Index(x, g, n_entry=6, seed=8)
    a = oracle.search(ix, q, k=min(10, itopk), itopk=itopk, width=width, max_iters=60)
    b = oracle.search(ix, q, k=min(10, itopk), itopk=itopk, width=width, max_iters=60, forget_visited=True)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(a[2]["iters"], b[2]["iters"]) and np.array_equal(a[2]["n_parents"], b[2]["n_parents"])
    assert (b[2]["n_dist"] >= a[2]["n_dist"]).all() and (b[2]["n_dist"] > a[2]["n_dist"]).any()


# ----------------------------------------------------------------------------- routing
@pytest.mark.parametrize("dt", ["u8", "f32"])
def test_routed_entries_fall_in_the_nearest_clusters(oracle, dt):
    rng = np.random.default_rng(30)
    n_clusters, dim = 12, 16
    cen = random_vectors(rng, n_clusters, dim, dt)
    sizes = rng.integers(0, 9, n_clusters)
    sizes[3] = 0  # an empty cluster yields no entries
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    x = random_vectors(rng, n, dim, dt)
    q = random_vectors(rng, 20, dim, dt)
    near = oracle.route(cen, q, 3, 0)
    ix = oracle.Index(x, np.zeros((n, 1), np.int32), n_entry=9, entry_mode=1, seed=4, centroids=cen,
                      cluster_offsets=off, route_c=3)
    ent = oracle.entries(ix, q)
    for i in range(20):
        keys = np_keys(q[i], cen, 0)
        assert near[i].tolist() == np.lexsort((np.arange(n_clusters), keys))[:3].tolist()
        owners = {int(np.searchsorted(off, e, side="right") - 1) for e in ent[i] if e >= 0}
        assert owners <= set(near[i].tolist())
        want = sum(3 for c in near[i] if sizes[c] > 0)  # 9 slots, 3 per routed cluster
        assert (ent[i] >= 0).sum() == want


def _splitmix64_stream(seed, count):
    """The published splitmix64 generator, written out here on its own: state += golden-ratio
    constant, output = the three-step xor-shift-multiply finaliser of the new state."""
    m = (1 << 64) - 1
    out, state = [], seed & m
    for _ in range(count):
        state = (state + 0x9E3779B97F4A7C15) & m
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
        out.append(z ^ (z >> 31))
    return out


def test_routed_entry_ids_follow_the_slot_rule_and_the_generator(oracle):
    """Entry j of the query at batch position i takes output number i*n_entry + j of the splitmix64
    stream started at the seed, goes to the (j mod route_c)-th nearest cluster c, and is
    off[c] + z mod |c|; an empty cluster gives no entry for its slots."""
    rng = np.random.default_rng(31)
    n_clusters, dim, n_entry, route_c, seed, nq = 9, 8, 7, 3, 0xDEADBEEFCAFE, 11
    cen = random_vectors(rng, n_clusters, dim, "f32")
    sizes = rng.integers(1, 40, n_clusters)
    sizes[[2, 5]] = 0
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    x = random_vectors(rng, n, dim, "f32")
    q = random_vectors(rng, nq, dim, "f32")
    ix = oracle.Index(x, np.zeros((n, 1), np.int32), n_entry=n_entry, entry_mode=1, seed=seed, centroids=cen,
                      cluster_offsets=off, route_c=route_c)
    ent = oracle.entries(ix, q)
    z = _splitmix64_stream(seed, nq * n_entry)
    saw_empty = False
    for i in range(nq):
        keys = np_keys(q[i], cen, 0)
        near = np.lexsort((np.arange(n_clusters), keys))[:route_c]
        want = []
        for j in range(n_entry):
            c = int(near[j % route_c])
            if sizes[c] == 0:
                saw_empty = True
                continue
            want.append(int(off[c]) + z[i * n_entry + j] % int(sizes[c]))
        got = [int(e) for e in ent[i] if e >= 0]
        assert got == want, (i, got, want)
    assert saw_empty
    # uniform mode, same stream: z mod n
    ix0 = oracle.Index(x, np.zeros((n, 1), np.int32), n_entry=n_entry, entry_mode=0, seed=seed)
    ent0 = oracle.entries(ix0, q)
    assert ent0.tolist() == [[z[i * n_entry + j] % n for j in range(n_entry)] for i in range(nq)]


def test_given_routes_replace_the_routing_step(oracle):
    """Searching with the oracle's own routes handed in gives the oracle's own answer; a route id
    outside the clusters names no cluster (no entries from it; padding if a query has no other)."""
    rng = np.random.default_rng(32)
    x, g, q = _clustered_case(rng, "u8")
    n = len(x)
    off = np.array([0, n // 3, n // 3, n], np.int64)  # cluster 1 is empty
    cen = np.stack([x[: n // 3].mean(0), x[0] * 0, x[n // 3:].mean(0)]).astype(np.uint8)
    ix = oracle.Index(x, g, n_entry=8, entry_mode=1, seed=3, centroids=cen, cluster_offsets=off, route_c=2)
    a = oracle.search(ix, q, 5, 16, 2, 30)
    r = oracle.route(cen, q, 2, 0)
    b = oracle.search(ix, q, 5, 16, 2, 30, routes=r)
    assert all(np.array_equal(u, v) for u, v in zip(a[:2], b[:2]))
    bad = r.copy()
    bad[0] = [-1, 3]
    bad[1, 1] = 7
    c = oracle.search(ix, q, 5, 16, 2, 30, routes=bad)
    assert (c[0][0] == -1).all() and (c[1][0] == np.iinfo(np.int32).max).all() and c[2]["n_dist"][0] == 0
    ix1 = oracle.Index(x, g, n_entry=8, entry_mode=1, seed=3, centroids=cen, cluster_offsets=off, route_c=2)
    ent = oracle.entries(ix1, q[1:2])  # query 0 of that call: other stream positions, so compare through the search only
    assert np.array_equal(c[0][2:], a[0][2:]) and np.array_equal(c[1][2:], a[1][2:])
    assert ent.shape == (1, 8)


def test_half_precision_decoding_on_explicit_bit_patterns(oracle):
    """fp16 inputs are decoded by the format's definition; checked against numpy's float16 on
    zeros, the smallest and largest subnormals, the smallest normal, 1, the largest finite value
    and both infinities, through key = -q*x with q = 1."""
    bits = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x03FF, 0x83FF, 0x0200, 0x0400, 0x8400, 0x3C00, 0xBC00, 0x3555,
                     0x7BFF, 0xFBFF, 0x7C00, 0xFC00], np.uint16)
    x = bits.view(np.float16).reshape(-1, 1)
    q = np.ones((1, 1), np.float16)
    got = oracle.keys(x, q, np.arange(len(bits), dtype=np.int32)[None, :], metric=1)[0]
    want = -x[:, 0].astype(np.float64)
    assert np.array_equal(got, want)
    assert got[2] == -2.0 ** -24 and got[4] == -(1023 * 2.0 ** -24) and got[12] == -65504.0 and np.isneginf(got[14])


# ----------------------------------------------------------------------------- P7 the paper's worked example
def _golden():
    vals = {}
    with open(os.path.join(HERE, "golden", "paper_stage3_traffic.txt")) as f:
        for line in f:
            if "=" in line and not line.startswith("#"):
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    return vals


def test_paper_stage3_worked_example(oracle):
    """Sec. 3.2 Stage 3: with I = 6 rounds, beam width w = 6 and out-degree 32, a query
    whose parents are always fresh fetches V = 6*6*32 = 1152 vectors; at d = 1536 fp16
    that is 3.539 MB and 1.55e12 B/s gives about 4.37e5 queries/s, 68.5 ms for 30k.
    A layered no-revisit graph reproduces V with the oracle's counters."""
    from paper_2512_02278_amd import metrics

    gold = _golden()
    I, w, deg, dim = int(gold["iterations"]), int(gold["width"]), int(gold["degree"]), int(gold["dim"])
    n = w + I * w * deg
    x = np.zeros((n, dim), np.float16)
    g = np.full((n, deg), -1, np.int32)
    # layer 0: the w entries; layer l+1: the children of the w best nodes of layer l.
    # deeper layers are nearer to the query (at the origin), so parents are always new nodes.
    x[:w, 0] = 8 + np.arange(w) / 256
    start = 0
    for layer in range(I):
        child0 = w + layer * w * deg
        for p in range(w):  # the w best of a layer are its first w nodes
            g[start + p] = child0 + p * deg + np.arange(deg)
        x[child0:child0 + w * deg, 0] = (7 - layer) + np.arange(w * deg) / 256
        start = child0
    cen = x[:w].copy()
    ix = oracle.Index(x, g, n_entry=w, entry_mode=1, seed=1, centroids=cen,
                      cluster_offsets=np.arange(w + 1), route_c=w)
    q = np.zeros((1, dim), np.float16)
    ids, dists, cnt = oracle.search(ix, q, k=10, itopk=64, width=w, max_iters=I)
    assert cnt["iters"][0] == I and cnt["n_parents"][0] == I * w
    fetched = int(cnt["n_dist"][0]) - w  # neighbour vectors, entries aside
    assert fetched == gold["vectors_per_query"] == metrics.paper_model_vectors(I, w, deg)
    nbytes = metrics.paper_model_bytes(fetched, dim, int(gold["bytes_per_elem"]))
    assert nbytes == 3538944 and round(nbytes / 1e6, 3) == gold["megabytes_per_query"]
    qps = metrics.paper_model_qps(gold["hbm_bytes_per_s"], nbytes)
    assert abs(qps - gold["qps"]) / gold["qps"] < 0.005  # the paper rounds 4.38e5 down to 4.37e5
    assert abs(gold["queries_per_rank"] / qps * 1e3 - gold["search_ms"]) < 0.1
    # the result is the 10 nodes nearest the origin: the first 10 of the last layer
    last = w + (I - 1) * w * deg
    assert ids[0].tolist() == list(range(last, last + 10))
    # the refined count adds graph rows, query and results to the rows scored
    b = metrics.algorithmic_bytes_per_query(cnt["n_dist"][0], cnt["n_parents"][0], dim * 2, deg, dim * 2, 10)
    assert b == (w + fetched) * dim * 2 + I * w * deg * 4 + dim * 2 + 80


# ----------------------------------------------------------------------------- the tiny config
def test_tiny_sift_like_config_behaves_as_expected(oracle):
    """Config 1 (N=10k uint8 d=128, 100 centres, degree-32 exact kNN graph, 100 queries,
    k=10, itopk=64, width 1, 50 rounds, 32 entries).  The mixture's clusters are far
    apart, so the kNN graph has no edges between clusters: uniform entries reach the
    query's cluster only by luck, routed entries always do."""
    import torch

    from paper_2512_02278_amd import inputs

    part = inputs.sift_like(10_000, 100)
    inputs.knn_graph_exact(part, 32)
    q = inputs.sift_like_queries(part, 100)
    stats = inputs.graph_stats(part)
    assert stats["cross_cluster_edge_fraction"] == 0.0 and stats["empty_slot_fraction"] == 0.0
    x, g, qn = part.vectors.numpy(), part.graph.numpy(), q.numpy()
    # the graph generator equals the definition on a few rows
    for i in (0, 1234, 9999):
        ei, _ = np_topk(x[i], x, [j for j in range(10_000) if j != i], 0, 32)
        assert g[i].tolist() == ei.tolist()
    gt, _ = oracle.bruteforce(x, qn, 10, 0)
    uni = oracle.Index(x, g, n_entry=32, entry_mode=0, seed=20251204)
    ids_u, _, _ = oracle.search(uni, qn, 10, 64, 1, 50)
    rec_u = inputs.recall(torch.from_numpy(ids_u), torch.from_numpy(gt))
    rt = oracle.Index(x, g, n_entry=32, entry_mode=1, seed=20251204, centroids=part.centres.numpy(),
                      cluster_offsets=part.offsets.numpy(), route_c=1)
    ids_r, _, cnt = oracle.search(rt, qn, 10, 64, 1, 50)
    rec_r = inputs.recall(torch.from_numpy(ids_r), torch.from_numpy(gt))
    assert 0.1 < rec_u < 0.5  # about 1 - (1 - 1/100)^32 = 0.28
    assert rec_r > 0.97
    assert cnt["iters"].max() <= 50


# ----------------------------------------------------------------------------- stage 4, local half
@pytest.mark.parametrize("dt", ["u8", "f32"])
def test_merge_of_partition_results_is_global_bruteforce(oracle, dt):
    """Merging the exact top-k of disjoint partitions (ids made global) gives the exact top-k of
    their union: the definition of the combine step.  Also checked directly against a numpy
    lexsort, with padding and ties."""
    rng = np.random.default_rng(40)
    n, dim, k, parts = 900, 16, 10, 3
    x = random_vectors(rng, n, dim, dt)
    if dt == "u8":
        x %= 6
    q = random_vectors(rng, 25, dim, dt)
    if dt == "u8":
        q %= 6
    bounds = [0, 250, 255, 900]  # the middle partition has fewer than k vectors: its list is padded
    ids_p, keys_p = [], []
    for p in range(parts):
        lo, hi = bounds[p], bounds[p + 1]
        i, d = oracle.bruteforce(np.ascontiguousarray(x[lo:hi]), q, k, 0)
        ids_p.append(np.where(i >= 0, i + lo, -1))
        keys_p.append(d)
    ids = np.concatenate(ids_p, 1).astype(np.int32)
    keys = np.concatenate(keys_p, 1)
    got_i, got_k = oracle.merge_topk(ids, keys, k)
    want_i, want_k = oracle.bruteforce(x, q, k, 0)
    assert np.array_equal(got_i, want_i) and np.array_equal(got_k, want_k)
    for r in range(len(q)):
        real = ids[r] >= 0
        order = np.lexsort((ids[r][real], keys[r][real]))[:k]
        assert got_i[r].tolist() == ids[r][real][order].tolist()
    # fewer candidates than k: padded
    gi, gk = oracle.merge_topk(np.array([[5, -1, 3, -1]], np.int32), np.array([[7, 0, 7, 0]], np.int32), 3)
    assert gi.tolist() == [[3, 5, -1]] and gk.tolist() == [[7, 7, 2**31 - 1]]


def test_gather_returns_the_rows(oracle):
    rng = np.random.default_rng(41)
    buf = rng.standard_normal((50, 24)).astype(np.float16)
    x = buf[:, :16]  # padded rows
    ids = np.array([[3, 49, -1], [0, 0, 50]], np.int32)
    out = oracle.gather(x, ids)
    assert out.shape == (2, 3, 16)
    assert np.array_equal(out[0, 0], x[3]) and np.array_equal(out[0, 1], x[49]) and np.array_equal(out[1, 1], x[0])
    assert not out[0, 2].any() and not out[1, 2].any()

"""Benchmark of the search hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--nq N]

A step is one ann_search call (routing + execution order + beam search: every stage of the
hot path) over one batch of synthetic queries that already sits in HBM.  The default
workload is the 100M-vector uint8 partition ("one GPU's tenth of a billion-scale SIFT-like
index").  Prints ONE JSON line; progress goes to stderr.

The line carries: queries/s at the smallest itopk whose recall@k, less two standard errors,
reaches 0.95 on 10 000 exactly solved queries; bytes per query (algorithmic, from the oracle's
counters; gathered, from the kernel's); the roofline of the beam-search kernel; a batch-size
sweep, alone and with four batches in flight on four streams; and the CPU oracle timed on this machine's host cores on a sample of the same batch, which
is also checked bit for bit against the GPU's answers.

Roofline.  The timed step runs the batch grouped by cluster, so most gathers hit L2 and the
kernel is bound by vector-ALU instruction issue, not by HBM: "roofline" reports that resource
(issued vector instructions x 64 lanes per second against 256 CUs x 4 SIMDs x 16 lanes x
2.4 GHz), with the HBM view of the same launch ("hbm": measured L2<->fabric traffic / kernel
time) and the same kernel in drawn order ("drawn_order": every gather goes to HBM, algorithmic
bytes / kernel time against the 8 TB/s peak) beside it.  Instruction and byte counts come from
rocprofv3 --pmc runs of `bench.py --profile` (summaries under profiles/); they are used only if
the kernel sources they were taken on are the ones this run uses (a hash of the sources is
stored with them), otherwise the fields are null and "roofline" falls back to the drawn-order
HBM figure.

"value" is measured on the workload's own graph (the cluster-restricted kNN graph).  Where
the workload names a longer kNN list to start from, "optimized_graph" adds the same
measurement on the graph that ann_graph_optimize builds from it at the same degree.

--workload embed1536 is the shape of the paper's own cost example for this stage (Sec. 3.2); for it alone
"vs_baseline" relates the measured rate to the paper's analytic estimate for an A100 ("paper_model").

--profile runs only what the counters are for (a few searches in each configuration, the graph
construction, a copy of known size) with fixed --itopk / --opt-itopk and prints which launch is
which; it is the program the rocprofv3 commands in profiles/ run.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak
# Vector-ALU issue: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second (a wave64
# instruction occupies its SIMD for 4 cycles); the published 157.3 TFLOP/s fp32 figure is this x 2 (FMA) x 2 (packed).
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
RECALL_TARGET = 0.95
N_TRUTH = 10_000

WORKLOADS = {
    # name: generator settings and search parameters (benchmark configs)
    "sift100m": dict(kind="sift", n=100_000_000, centres=16384, dim=128, degree=32, nq=1_000_000, k=10, width=4,
                     max_iters=200, itopk_sweep=(128, 144, 160, 176, 184, 192, 200, 208, 224, 256),
                     sweep=(1_000, 10_000, 100_000, 1_000_000),
                     optimize_from=64, opt_itopk_sweep=(96, 104, 112, 120, 128, 144, 160, 184),
                     text="100M x 128 uint8 SIFT-like partition, 16384 centres, degree-32 cluster-restricted kNN graph"),
    "sift1m": dict(kind="sift", n=1_000_000, centres=1000, dim=128, degree=32, nq=10_000, k=10, width=4, max_iters=100,
                   itopk_sweep=(128, 160, 192, 256), sweep=(1_000, 10_000),
                   optimize_from=64, opt_itopk_sweep=(32, 48, 64, 96, 128),
                   text="1M x 128 uint8 SIFT-like index, 1000 centres, degree-32 cluster-restricted kNN graph"),
    "tiny": dict(kind="sift", n=10_000, centres=100, dim=128, degree=32, nq=100, k=10, width=1, max_iters=50,
                 itopk_sweep=(64,), sweep=(100,), exact_graph=True,
                 text="10k x 128 uint8 SIFT-like index, 100 centres, exact degree-32 kNN graph"),
    "deep10m": dict(kind="unit", dtype="f32", metric="l2", n=10_000_000, centres=4096, dim=96, degree=64, nq=100_000,
                    k=10, width=4, max_iters=150, itopk_sweep=(256,), sweep=(1_000, 10_000, 100_000),
                    optimize_from=128, opt_itopk_sweep=(32, 48, 64, 96, 128, 192, 256),
                    text="10M x 96 fp32 Deep-like index (unit-norm mixture, 4096 centres, rho 0.5), degree-64 "
                         "cluster-restricted kNN graph, L2"),
    "text20m": dict(kind="unit", dtype="f16", metric="ip", n=20_000_000, centres=8192, dim=768, degree=64, nq=50_000,
                    k=100, width=8, max_iters=200, itopk_sweep=(256,), sweep=(1_000, 10_000, 50_000),
                    optimize_from=128, opt_itopk_sweep=(100, 104, 112, 128, 160, 192, 256),
                    text="20M x 768 fp16 text-embedding-like index (unit-norm mixture, 8192 centres, rho 0.5), "
                         "degree-64 cluster-restricted kNN graph, inner product, fp32 accumulation"),
    # The shape of the paper's own cost example for this stage (Sec. 3.2, stage 3): fp16 rows of d = 1536, out-degree 32,
    # 6 rounds of beam width 6 (at most 1152 rows = 3.539 MB per query), c * bs = 30 000 queries per rank.  The paper
    # gives no list size, metric or recall for it; the list is 64 and the recall is reported as it comes out.
    "embed1536": dict(kind="unit", dtype="f16", metric="ip", n=8_000_000, centres=4096, dim=1536, degree=32, nq=30_000,
                      k=10, width=6, max_iters=6, itopk_sweep=(64,), sweep=(1_000, 10_000, 30_000),
                      paper_model=dict(rows_per_query=1152, qps_a100=4.37e5, a100_hbm_gbps=1550.0),
                      text="8M x 1536 fp16 embedding-like index (unit-norm mixture, 4096 centres, rho 0.5), degree-32 "
                           "cluster-restricted kNN graph, inner product: the row, degree, width and round count of the "
                           "paper's stage-3 cost example"),
}
FLOAT_TOL = {"f32": 1e-5, "f16": 1e-3}
SEED = 20251202


def log(msg: str) -> None:
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def sources_sha() -> str:
    """Hash of everything the kernels are compiled from: counters taken on other sources are not this build's."""
    h = hashlib.sha256()
    base = os.path.join(ROOT, "paper_2512_02278_amd")
    for path in sorted(glob.glob(os.path.join(base, "csrc", "*")) + [os.path.join(base, "build.py")]):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


def read_profile(kernel: str, workload: str) -> dict:
    """`key = value` lines of the committed rocprofv3 --pmc summary of this kernel and workload (profiles/)."""
    out = {}
    try:
        for ln in open(os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")):
            key, sep, val = ln.partition(" = ")
            if sep and key and " " not in key.strip():
                val = val.strip()
                try:
                    out[key.strip()] = float(val)
                except ValueError:
                    out[key.strip()] = val
    except OSError:
        pass
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="sift100m", choices=sorted(WORKLOADS))
    ap.add_argument("--nq", type=int, default=0, help="queries per step (default: the workload's batch)")
    ap.add_argument("--oracle-seconds", type=float, default=15.0, help="wall-clock aim for the CPU oracle sample")
    ap.add_argument("--no-oracle", action="store_true", help="skip the CPU baseline and the sampled parity check")
    ap.add_argument("--no-optimized-graph", action="store_true", help="skip the optimized-graph measurement")
    ap.add_argument("--itopk", type=int, default=0, help="fix the list size instead of choosing it by recall")
    ap.add_argument("--opt-itopk", type=int, default=0, help="the same for the optimized graph")
    ap.add_argument("--profile", action="store_true", help="only the launches the profiler's counters are for")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's partition; it has no multi-GPU path, run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2512_02278_amd import ann, inputs, metrics

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ann.lib()  # fail early if the library is not built
    dev = "cuda:0"
    w = WORKLOADS[args.workload]
    nq = args.nq or w["nq"]
    k, width, max_iters, degree = w["k"], w["width"], w["max_iters"], w["degree"]
    sha = sources_sha()

    # ------------------------------------------------------------------ inputs (resident in HBM)
    t0 = time.time()
    dt = w.get("dtype", "u8")
    metric = ann.ANN_IP if w.get("metric") == "ip" else ann.ANN_L2
    if w["kind"] == "sift":
        part = inputs.sift_like(w["n"], w["centres"], dim=w["dim"], seed=SEED, device=dev)
    else:
        part = inputs.unit_mixture(w["n"], w["centres"], w["dim"], torch.float32 if dt == "f32" else torch.float16,
                                   inputs.IP if metric == ann.ANN_IP else inputs.L2, seed=SEED, device=dev)
    log(f"vectors generated in {time.time() - t0:.1f} s")
    d_in = w.get("optimize_from") if not args.no_optimized_graph else None
    if w.get("exact_graph"):
        inputs.knn_graph_exact(part, degree)
    else:
        inputs.knn_graph_clustered(part, d_in or degree, progress=(lambda c, t: log(f"graph: cluster {c}/{t}"),
                                                                   max(1, w["centres"] // 8)))

    def event_ms(fn, reps):
        """Mean duration of fn() by HIP events on the stream the library launches on (torch's current stream)."""
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evs:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in evs) / reps

    opt = None
    if d_in:
        # the kNN lists are built d_in long; their first `degree` columns are the workload's kNN graph
        knn = part.graph
        torch.cuda.synchronize()
        log(f"kNN lists of length {d_in} built in {time.time() - t0:.1f} s")
        ws = torch.empty(ann.ann_graph_optimize_workspace_bytes(w["n"], d_in, degree), dtype=torch.uint8, device=dev)
        opt_graph = torch.empty((w["n"], degree), dtype=torch.int32, device=dev)
        ann.ann_graph_prune(knn, degree, pruned=opt_graph)  # warm-up
        prune_ms = event_ms(lambda: ann.ann_graph_prune(knn, degree, pruned=opt_graph), 1)
        ann.ann_graph_optimize(knn, degree, out_graph=opt_graph, workspace=ws)
        build_ms = event_ms(lambda: ann.ann_graph_optimize(knn, degree, out_graph=opt_graph, workspace=ws), 1)
        del ws
        opt = {"from_degree": d_in, "degree": degree,
               "build_ms": {"graph_prune_kernel": round(prune_ms, 2), "reverse_edges_and_merge": round(build_ms - prune_ms, 2),
                            "ann_graph_optimize": round(build_ms, 2)}}
        log(f"graph optimisation {d_in} -> {degree}: prune {prune_ms:.1f} ms, whole build {build_ms:.1f} ms")
        opt["build_roofline"] = prune_roofline(args.workload, sha, w["n"], d_in, degree, prune_ms)
        if not args.no_oracle and not args.profile:
            from oracle import sampling

            t1 = time.time()
            rng = np.random.default_rng(SEED)
            nodes = np.unique(np.concatenate([[0, w["n"] - 1], rng.integers(0, w["n"], 62)]))
            want = sampling.optimized_rows(knn, nodes, degree)
            got = opt_graph[torch.as_tensor(nodes, device=dev)].cpu().numpy()
            opt["parity"] = {"rows_checked": int(nodes.size), "bit_identical": bool(np.array_equal(got, want))}
            log(f"optimized graph: {opt['parity']} against the oracle in {time.time() - t1:.1f} s")
        part.graph = knn[:, :degree].contiguous()
        del knn
    nq_max = max(nq, max(w["sweep"]))
    if w["kind"] == "sift":
        queries = inputs.sift_like_queries(part, nq_max, seed=SEED + 1)
    else:
        queries = inputs.unit_mixture_queries(part, nq_max, seed=SEED + 1)
    torch.cuda.synchronize()
    log(f"index and {nq_max} queries generated in {time.time() - t0:.1f} s")

    def load(graph):
        return ann.ann_index_load(part.vectors, graph, metric=metric, n_entry=32, entry_mode=ann.ANN_ENTRY_ROUTED,
                                  seed=SEED + 2, centroids=part.centres, cluster_offsets=part.offsets, route_c=1)

    h = load(part.graph)
    row_bytes = w["dim"] * part.vectors.element_size()
    q = queries[:nq]
    out_ids = torch.empty((nq, k), dtype=torch.int32, device=dev)
    out_d = torch.empty((nq, k), dtype=torch.int32 if dt == "u8" else torch.float32, device=dev)

    def search(handle, it, **kw):
        return ann.ann_search(handle, q, k, it, width, max_iters, out_ids=out_ids, out_dists=out_d, **kw)

    if args.profile:
        return profile_pass(args, ann, torch, h, load(opt_graph) if opt is not None else None, q, search, sha)

    # ------------------------------------------------------------------ smallest itopk with recall - 2 SE >= 0.95
    n_gt = min(N_TRUTH, nq)
    t0 = time.time()
    truth = inputs.ground_truth(part, queries[:n_gt], k)
    torch.cuda.synchronize()
    log(f"exact ground truth for {n_gt} queries in {time.time() - t0:.1f} s")

    def recall_of(ids):
        per_query = inputs.recall_per_query(ids, truth)
        return float(per_query.mean()), float(per_query.std(unbiased=True) / per_query.numel() ** 0.5)

    def choose_itopk(handle, candidates, fixed):
        table, chosen = {}, None
        for cand in ([fixed] if fixed else candidates):
            ids, _ = ann.ann_search(handle, queries[:n_gt], k, cand, width, max_iters)
            torch.cuda.synchronize()
            r, se = recall_of(ids)
            table[cand] = [round(r, 4), round(se, 4)]
            if r - 2 * se >= RECALL_TARGET:
                chosen = cand
                break
        return table, chosen

    recall_by_itopk, itopk = choose_itopk(h, w["itopk_sweep"], args.itopk)
    log(f"recall@{k} [mean, standard error] by itopk: {recall_by_itopk}")
    target_met = itopk is not None
    if itopk is None:
        itopk = args.itopk or w["itopk_sweep"][-1]

    # ------------------------------------------------------------------ timed steps: whole hot path
    for _ in range(args.warmup):
        search(h, itopk)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        search(h, itopk)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    qps = nq / (wall / args.steps)
    rec, rec_se = recall_of(out_ids[:n_gt])
    log(f"{nq} queries/step, itopk {itopk}: {ms_per_step:.2f} ms/step, {qps:.3e} q/s, recall@{k} {rec:.4f} +- {rec_se:.4f}")

    # ------------------------------------------------------------------ the stages on their own (HIP events on the launch stream)
    routes = ann.ann_route(h, q)
    route_ms = event_ms(lambda: ann.ann_route(h, q, out_clusters=routes), args.steps)
    search_ms = event_ms(lambda: search(h, itopk, routes=routes), args.steps)
    # the same kernel without the cluster-grouped execution order: every gather goes to HBM
    ann.ann_index_set_option(h, ann.ANN_OPT_CLUSTER_ORDER_MIN_QUERIES, -1)
    search(h, itopk, routes=routes)
    drawn_ms = event_ms(lambda: search(h, itopk, routes=routes), max(2, args.steps // 2))
    ann.ann_index_set_option(h, ann.ANN_OPT_CLUSTER_ORDER_MIN_QUERIES, 16384)
    counters = torch.zeros((nq, 4), dtype=torch.int32, device=dev)
    search(h, itopk, counters=counters)
    torch.cuda.synchronize()
    cm = counters.double().mean(0).tolist()
    actual_bq = metrics.algorithmic_bytes_per_query(cm[1], cm[2], row_bytes, degree, row_bytes, k)
    log(f"stages: route {route_ms:.3f} ms, order + beam search {search_ms:.3f} ms (drawn order {drawn_ms:.3f} ms); per query: "
        f"rounds {cm[0]:.1f}, rows gathered {cm[1]:.0f}, graph rows {cm[2]:.0f}, table resets {cm[3]:.2f}")

    # ------------------------------------------------------------------ stage 1 of the next batch under stage 3 of this one
    # (two streams; the single-GPU shadow of the paper's two-microbatch pipeline, Sec. 3.2)
    s_route, s_search = torch.cuda.Stream(), torch.cuda.Stream()
    bufs = [torch.empty_like(routes) for _ in range(2)]
    routed = [torch.cuda.Event() for _ in range(2)]
    searched = [torch.cuda.Event() for _ in range(2)]
    torch.cuda.synchronize()
    ann.ann_route(h, q, out_clusters=bufs[0], stream=s_route)
    routed[0].record(s_route)
    t0 = time.perf_counter()
    for i in range(args.steps):
        cur, nxt = i % 2, (i + 1) % 2
        s_search.wait_event(routed[cur])
        search(h, itopk, routes=bufs[cur], stream=s_search)
        searched[cur].record(s_search)
        if i >= 1:
            s_route.wait_event(searched[nxt])  # the search that read bufs[nxt] has finished
        ann.ann_route(h, q, out_clusters=bufs[nxt], stream=s_route)
        routed[nxt].record(s_route)
    torch.cuda.synchronize()
    overlapped_qps = nq * args.steps / (time.perf_counter() - t0)
    log(f"two streams (stage 1 of the next batch under stage 3): {overlapped_qps:.3e} q/s")

    # ------------------------------------------------------------------ batch-size sweep (whole hot path)
    sweep = {}
    for b in w["sweep"]:
        if b > nq_max:
            continue
        qb = queries[:b]
        reps = max(3, min(20, int(2e6 // b)))
        for _ in range(2):
            ann.ann_search(h, qb, k, itopk, width, max_iters, out_ids=out_ids[:b], out_dists=out_d[:b])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            ann.ann_search(h, qb, k, itopk, width, max_iters, out_ids=out_ids[:b], out_dists=out_d[:b])
        torch.cuda.synchronize()
        sweep[str(b)] = round(b * reps / (time.perf_counter() - t0), 1)
    log(f"q/s by batch size: {sweep}")
    # Small batches are bound by the latency of a query's chain of rounds, not by the chip: several of them in flight at
    # once (one stream each, as micro-batches of a pipeline are; Sec. 3.2) share it.  Aggregate queries/s of 4 streams.
    streams4 = {}
    small = [b for b in w["sweep"] if b <= 10_000 and 4 * b <= nq_max]
    if small:
        ss = [torch.cuda.Stream() for _ in range(4)]
        for b in small:
            views = [(queries[i * b:(i + 1) * b], out_ids[i * b:(i + 1) * b], out_d[i * b:(i + 1) * b]) for i in range(4)]

            def round_of_four():
                for st, (qv, oi, od) in zip(ss, views):
                    ann.ann_search(h, qv, k, itopk, width, max_iters, out_ids=oi, out_dists=od, stream=st)
            torch.cuda.synchronize()
            round_of_four()
            torch.cuda.synchronize()
            reps = max(3, min(20, int(1e6 // b)))
            t0 = time.perf_counter()
            for _ in range(reps):
                round_of_four()
            torch.cuda.synchronize()
            streams4[str(b)] = round(4 * b * reps / (time.perf_counter() - t0), 1)
        log(f"q/s by batch size, four batches in flight on four streams: {streams4}")
    # leave the outputs of the full batch in place for the parity check
    search(h, itopk)
    torch.cuda.synchronize()

    # ------------------------------------------------------------------ CPU oracle: baseline, parity sample, algorithmic counters
    cpu_baseline = None
    parity = None
    algo = dict(n_dist=None, n_parents=None)
    if not args.no_oracle:
        import oracle

        t0 = time.time()
        ix = oracle.Index(part.vectors.cpu().numpy(), part.graph.cpu().numpy(), metric=metric, n_entry=32, entry_mode=1,
                          seed=SEED + 2, centroids=part.centres.cpu().numpy(),
                          cluster_offsets=part.offsets.cpu().numpy(), route_c=1)
        log(f"index copied to host in {time.time() - t0:.1f} s")
        qh = q.cpu().numpy()
        cores = oracle.threads()
        probe = min(nq, 256)
        t0 = time.perf_counter()
        oracle.search(ix, qh[:probe], k, itopk, width, max_iters)
        per_q = (time.perf_counter() - t0) / probe
        sample = int(max(probe, min(nq, args.oracle_seconds / per_q)))
        t0 = time.perf_counter()
        oi, od, oc = oracle.search(ix, qh[:sample], k, itopk, width, max_iters)
        cpu_s = time.perf_counter() - t0
        cpu_baseline = {"value": round(sample / cpu_s, 1), "unit": "queries/s", "cores": cores, "kind": "oracle",
                        "sample": f"first {sample} queries of the timed batch, same index, itopk {itopk}; "
                                  f"{cpu_s:.1f} s on {cores} threads"}
        gi, gd = out_ids[:sample].cpu().numpy(), out_d[:sample].cpu().numpy()
        if dt == "u8":
            same = bool(np.array_equal(gi, oi) and np.array_equal(gd, od))
            parity = {"queries_checked": sample, "bit_identical": same}
        else:
            # keys of the GPU's ids recomputed by the oracle: the reported keys, and the sorted keys rank by
            # rank against the oracle's own answer, must agree within the tolerance of the dtype
            tol = FLOAT_TOL[dt]
            gk = oracle.keys(ix.vectors, qh[:sample], gi, metric)
            fin = np.isfinite(gk) & np.isfinite(od)
            ok_reported = bool((np.abs(gd - gk)[fin] <= tol * np.maximum(np.abs(gk[fin]), 1e-30)).all())
            ok_ranks = bool((np.abs(np.sort(gk, 1) - od)[fin] <= tol * np.maximum(np.abs(od[fin]), 1e-30)).all()
                            and np.array_equal(gi < 0, oi < 0))
            same = ok_reported and ok_ranks
            parity = {"queries_checked": sample, "keys_within_tolerance": same, "tolerance": tol,
                      "identical_id_lists": round(float((gi == oi).all(1).mean()), 4)}
        algo = dict(n_dist=float(oc["n_dist"].mean()), n_parents=float(oc["n_parents"].mean()))
        log(f"oracle: {sample} queries in {cpu_s:.1f} s on {cores} threads; parity: {parity}")
        del ix

    ann.ann_free(h)

    # ------------------------------------------------------------------ the same measurement on the optimized graph
    if opt is not None:
        h2 = load(opt_graph)
        opt_recalls, opt_itopk = choose_itopk(h2, w["opt_itopk_sweep"], args.opt_itopk)
        opt["recall_target_met"] = opt_itopk is not None
        opt_itopk = opt_itopk or args.opt_itopk or w["opt_itopk_sweep"][-1]
        for _ in range(args.warmup):
            search(h2, opt_itopk)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            search(h2, opt_itopk)
        torch.cuda.synchronize()
        opt_wall = (time.perf_counter() - t0) / args.steps
        opt_routes = ann.ann_route(h2, q)
        opt_search_ms = event_ms(lambda: search(h2, opt_itopk, routes=opt_routes), args.steps)
        search(h2, opt_itopk, counters=counters)
        torch.cuda.synchronize()
        ocm = counters.double().mean(0).tolist()
        orec, orec_se = recall_of(out_ids[:n_gt])
        opt.update({"itopk": opt_itopk, "recall_by_itopk": opt_recalls, "recall_at_k": round(orec, 4), "recall_se": round(orec_se, 4),
                    "qps": round(nq / opt_wall, 1), "ms_per_step": round(opt_wall * 1e3, 3),
                    "per_query": {"rounds": round(ocm[0], 2), "rows_gathered": round(ocm[1], 1), "graph_rows": round(ocm[2], 1)}})
        opt_sweep = {}
        for b in w["sweep"]:
            if b > nq_max or b == nq:
                continue
            qb = queries[:b]
            reps = max(3, min(20, int(2e6 // b)))
            for _ in range(2):
                ann.ann_search(h2, qb, k, opt_itopk, width, max_iters, out_ids=out_ids[:b], out_dists=out_d[:b])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                ann.ann_search(h2, qb, k, opt_itopk, width, max_iters, out_ids=out_ids[:b], out_dists=out_d[:b])
            torch.cuda.synchronize()
            opt_sweep[str(b)] = round(b * reps / (time.perf_counter() - t0), 1)
        opt_sweep[str(nq)] = opt["qps"]
        opt["qps_by_batch"] = opt_sweep
        gathered = metrics.algorithmic_bytes_per_query(ocm[1], ocm[2], row_bytes, degree, row_bytes, k) * nq
        opt["roofline"] = search_roofline(read_profile("beam_search_kernel", args.workload), "optimized", sha, nq, opt_search_ms,
                                          gathered, None, None, opt_itopk)
        log(f"optimized graph: itopk {opt_itopk}, recall {orec:.4f}, {opt['qps']:.3e} q/s, rounds {ocm[0]:.1f}")
        ann.ann_free(h2)

    # ------------------------------------------------------------------ what random whole-row reads reach on this table
    hg = ann.ann_index_load(part.vectors, part.graph, metric=metric, n_entry=32)
    n_rows = int(min(1 << 26, (8 << 30) // row_bytes))
    rnd = torch.randint(0, w["n"], (n_rows,), dtype=torch.int32, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    ann.ann_calibration_gather(hg, rnd, sink=sink)  # warm-up
    gather_ms = min(event_ms(lambda: ann.ann_calibration_gather(hg, rnd, sink=sink), 1) for _ in range(5))
    gather_gbps = n_rows * row_bytes / gather_ms / 1e6
    log(f"random row gather ({n_rows} rows of {row_bytes} B): {gather_ms:.3f} ms, {gather_gbps:.0f} GB/s")
    ann.ann_free(hg)
    del rnd

    # ------------------------------------------------------------------ roofline of the dominant kernel
    algo_bytes = None
    if algo["n_dist"] is not None:
        algo_bytes = metrics.algorithmic_bytes_per_query(algo["n_dist"], algo["n_parents"], row_bytes, degree, row_bytes, k) * nq
    roofline = search_roofline(read_profile("beam_search_kernel", args.workload), "grouped", sha, nq, search_ms,
                               actual_bq * nq, algo_bytes, drawn_ms, itopk)
    roofline["random_row_gather"] = {
        "achieved": round(gather_gbps, 1), "unit": "GB/s", "rows": n_rows,
        "note": "ann_calibration_gather: a plain kernel that reads uniformly random whole rows of the same vector table "
                "and nothing else (non-temporal, eight loads in flight per lane): what this access pattern gets without "
                "any search work, a reference rather than a hard limit"}
    if roofline.get("drawn_order"):
        roofline["drawn_order"]["vs_random_row_gather"] = round(roofline["drawn_order"]["achieved"] / gather_gbps, 4)

    line = {
        "metric": f"queries/sec at recall@{k}>=0.95 on 1 MI355X", "value": round(qps, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dt, "data": "synthetic",
        "config": {"workload": f"{args.workload}: {w['text']}; {nq} queries per step in drawn order, k={k}, "
                               f"itopk={itopk}, width={width}, max_iters={max_iters}, 32 routed entries (route_c=1)",
                   "itopk": itopk, "queries_per_step": nq},
        "recall_at_k": round(rec, 4), "recall_se": round(rec_se, 4), "recall_queries": n_gt, "k": k,
        "recall_rule": f"smallest itopk of the sweep whose recall - 2 standard errors >= {RECALL_TARGET}",
        "recall_target_met": target_met, "recall_by_itopk": recall_by_itopk,
        "bytes_per_query": {"algorithmic": None if algo_bytes is None else round(algo_bytes / nq), "gathered": round(actual_bq)},
        "per_query": {"rounds": round(cm[0], 2), "rows_gathered": round(cm[1], 1), "graph_rows": round(cm[2], 1),
                      "rows_scored_by_oracle": algo["n_dist"]},
        "stage_ms": {"route": round(route_ms, 3), "order_and_beam_search": round(search_ms, 3)},
        "qps_two_streams": round(overlapped_qps, 1), "qps_by_batch": sweep, "qps_by_batch_four_streams": streams4, "parity": parity, "optimized_graph": opt,
        "sources_sha": sha, "roofline": roofline, "cpu_baseline": cpu_baseline,
    }
    pm = w.get("paper_model")
    if pm:
        model_bytes = pm["rows_per_query"] * row_bytes
        line["vs_baseline"] = round(qps / pm["qps_a100"], 3)
        line["paper_model"] = {
            "source": "Sec. 3.2, stage 3: an analytic bandwidth estimate for an A100 (HBM 1.55 TB/s), not a measurement",
            "rows_per_query": pm["rows_per_query"], "bytes_per_query": model_bytes, "qps_a100": pm["qps_a100"],
            "same_model_at_mi355x_hbm_peak_qps": round(HBM_PEAK_GBPS * 1e9 / model_bytes, 1),
            "measured_rows_per_query": round(cm[1], 1), "measured_bytes_per_query": round(actual_bq),
            "note": "vs_baseline = measured queries/s of the whole hot path (routing included) / the paper's estimate; the search "
                    "scores fewer rows than the model counts because ids seen before are not gathered again"}
    print(json.dumps(line), flush=True)
    return 0


def search_roofline(prof: dict, leg: str, sha: str, nq: int, kernel_ms: float, gathered_bytes: float, algo_bytes,
                    drawn_ms, itopk: int) -> dict:
    """Roofline object of one timed configuration of beam_search_kernel ("grouped" or "optimized").

    prof: the committed counter summary; its figures are per launch of `nq_profiled` queries at `itopk_profiled`
    and are used only if they were taken on these sources, this batch size and this list size."""
    fresh = bool(prof) and prof.get("sources_sha") == sha and prof.get(f"{leg}.nq") == nq and prof.get(f"{leg}.itopk") == itopk
    sec = kernel_ms * 1e-3
    counters = {"file": "profiles/beam_search_kernel_*_pmc.txt", "fresh": fresh,
                "why": None if fresh else ("no counters recorded" if not prof else
                                           "recorded on other kernel sources, batch or list size: not used")}
    hbm_view = {"traffic": None, "achieved": None, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": None, "dram_read_bytes": None,
                "gathered_bytes_per_launch": round(gathered_bytes),
                "note": "measured bytes between L2 and the fabric (FETCH_SIZE + WRITE_SIZE, scaled by the same counters on a "
                        "copy of known size) / kernel time; bytes the kernel gathers beyond this were L2 hits"}
    drawn = None
    if drawn_ms is not None and algo_bytes is not None:
        gbps = algo_bytes / (drawn_ms * 1e-3) / 1e9
        drawn = {"bound": "hbm", "kernel_ms": round(drawn_ms, 3), "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                 "frac": round(gbps / HBM_PEAK_GBPS, 4), "algorithmic_bytes_per_launch": round(algo_bytes),
                 "traffic": prof.get("drawn.traffic_bytes") if fresh else None,
                 "note": "the same kernel with the cluster grouping switched off: every gather goes to HBM and the measured "
                         "traffic equals the algorithmic bytes; this is the figure to hold against the HBM roofline"}
    if fresh:
        traffic = prof[f"{leg}.traffic_bytes"]
        hbm_view.update({"traffic": traffic, "achieved": round(traffic / sec / 1e9, 1), "frac": round(traffic / sec / 1e9 / HBM_PEAK_GBPS, 4),
                         "dram_read_bytes": prof.get(f"{leg}.dram_read_bytes")})
        valu = prof[f"{leg}.valu_insts"]  # wavefront instructions per launch
        tops = valu * 64 / sec / 1e12
        alu_view = {"achieved": round(tops, 2), "peak": round(VALU_PEAK_TOPS, 2), "unit": "TOP/s", "frac": round(tops / VALU_PEAK_TOPS, 4),
                    "valu_insts_per_query": round(valu / nq, 1), "valu_busy_frac_by_counter": prof.get(f"{leg}.valu_busy_frac"),
                    "note": "vector-ALU issue: vector instructions the launch issued (rocprofv3 SQ_INSTS_VALU) x 64 lanes / kernel time, "
                            "against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz"}
        # the binding resource is the one that is nearer to its peak
        if alu_view["frac"] >= hbm_view["frac"]:
            out = {"bound": "alu", "kernel": "beam_search_kernel", "achieved": alu_view["achieved"], "peak": alu_view["peak"],
                   "unit": "TOP/s", "frac": alu_view["frac"], "traffic": traffic, "kernel_ms": round(kernel_ms, 3),
                   "note": "the launch is bound by vector-ALU instruction issue, not by bytes: most gathers of the grouped batch "
                           "hit L2 (see hbm for the byte view, drawn_order for the HBM-bound run of the same kernel)"}
        else:
            out = {"bound": "hbm", "kernel": "beam_search_kernel", "achieved": hbm_view["achieved"], "peak": HBM_PEAK_GBPS,
                   "unit": "GB/s", "frac": hbm_view["frac"], "traffic": traffic, "kernel_ms": round(kernel_ms, 3),
                   "note": "the launch is bound by bytes: achieved = measured traffic between L2 and the fabric / kernel time (the "
                           "bytes the kernel gathers, gathered_bytes_per_launch, are more: the rest were L2 hits)"}
        out["alu"] = alu_view
    elif drawn is not None:
        out = dict(drawn, kernel="beam_search_kernel",
                   note="no current instruction counters for the grouped launch: this is the drawn-order launch of the same "
                        "kernel, which is bound by HBM (algorithmic bytes / kernel time)")
    else:
        out = {"bound": "hbm", "kernel": "beam_search_kernel", "achieved": None, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": None,
               "traffic": None, "kernel_ms": round(kernel_ms, 3), "note": "no counters and no oracle run: nothing to hold against a roofline"}
    out["counters"] = counters
    out["hbm"] = hbm_view
    if leg == "grouped":
        out["drawn_order"] = drawn
        out["algorithmic_bytes_per_launch"] = None if algo_bytes is None else round(algo_bytes)
    return out


def prune_roofline(workload: str, sha: str, n: int, d_in: int, degree: int, prune_ms: float) -> dict:
    prof = read_profile("graph_prune_kernel", workload)
    fresh = bool(prof) and prof.get("sources_sha") == sha
    algo = n * (d_in * d_in * 4 + d_in * 4 + degree * 4)  # d_in rows of d_in ids read per node, its own row, the pruned row
    out = {"kernel": "graph_prune_kernel", "kernel_ms": round(prune_ms, 2), "algorithmic_bytes_per_launch": algo,
           "counters": {"file": "profiles/graph_prune_kernel_*_pmc.txt", "fresh": fresh}}
    if fresh:
        valu, traffic = prof["prune.valu_insts"], prof["prune.traffic_bytes"]
        tops = valu * 64 / (prune_ms * 1e-3) / 1e12
        out.update({"bound": "alu", "achieved": round(min(tops, VALU_PEAK_TOPS), 2), "peak": round(VALU_PEAK_TOPS, 2), "unit": "TOP/s",
                    "frac": round(min(1.0, tops / VALU_PEAK_TOPS), 4), "issue_rate_over_nominal": round(tops / VALU_PEAK_TOPS, 4),
                    "traffic": traffic,
                    "hbm": {"traffic": traffic, "achieved": round(traffic / prune_ms / 1e6, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                            "frac": round(traffic / prune_ms / 1e6 / HBM_PEAK_GBPS, 4)},
                    "note": "vector instructions issued x 64 lanes / time against 4 cycles per instruction on every SIMD.  Much of this "
                            "kernel runs with half of a wavefront's lanes switched off, and such instructions leave the SIMD after 2 "
                            "cycles, so the count can exceed the nominal capacity (issue_rate_over_nominal); achieved and frac are "
                            "capped at the peak: the vector ALUs are saturated.  Neighbours' rows are re-read from L2 (XCD-local "
                            "walk), so the algorithmic bytes do not bind (see hbm)"})
    else:
        out.update({"bound": "alu", "achieved": None, "peak": round(VALU_PEAK_TOPS, 2), "unit": "TOP/s", "frac": None, "traffic": None})
    return out


def profile_pass(args, ann, torch, h, h_opt, q, search, sha) -> int:
    """The launches the rocprofv3 commands under profiles/ are for, in a fixed order, then their legend."""
    w = WORKLOADS[args.workload]
    itopk = args.itopk or w["itopk_sweep"][0]
    sequence = []
    for _ in range(1 + max(1, args.steps)):
        search(h, itopk)
        sequence.append("grouped")
    ann.ann_index_set_option(h, ann.ANN_OPT_CLUSTER_ORDER_MIN_QUERIES, -1)
    for _ in range(2):
        search(h, itopk)
        sequence.append("drawn")
    if h_opt is not None:
        for _ in range(1 + max(1, args.steps)):
            search(h_opt, args.opt_itopk or w["opt_itopk_sweep"][0])
            sequence.append("optimized")
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").random_(0, 256)
    dst = torch.empty_like(src)
    for _ in range(3):
        ann.ann_calibration_copy(dst, src)  # 1 GiB read, 1 GiB written: calibrates the byte counters
    torch.cuda.synchronize()
    print(json.dumps({"profile_pass": args.workload, "sources_sha": sha, "queries_per_launch": q.shape[0], "itopk": itopk,
                      "opt_itopk": args.opt_itopk or (w.get("opt_itopk_sweep") or [0])[0],
                      "beam_search_kernel_launches_of_full_batch": sequence,
                      "graph_prune_kernel_launches": ["ann_graph_prune (warm-up)", "ann_graph_prune", "ann_graph_optimize (warm-up)",
                                                      "ann_graph_optimize"] if h_opt is not None else [],
                      "calibration_copy_bytes": 1 << 30}), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

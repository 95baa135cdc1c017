/*
 * CPU oracle for batched greedy beam search over a fixed-degree proximity graph.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU
 * library is checked against.  Nothing in the product path may call it, and it
 * shares no code, header, table or helper with the GPU library.
 *
 * What it follows.  The paper (Fantasy, Sec. 1 and Sec. 3.2 "Stage 3: Parallel Vector
 * Search Latency") describes the per-GPU step only as a greedy traversal of a
 * proximity graph that starts from entry nodes and moves towards more similar
 * vectors, with a beam width w per iteration, a graph out-degree d_g and I
 * iterations, so that about I*w*d_g neighbour vectors are scored per query, each
 * fetched once (Sec. 2, equation for bt_q).  The paper prints no algorithm
 * listing, so the loop below is the fixed-size sorted-list best-first search that
 * those sentences describe, with every choice the paper leaves open written out
 * next to the line that takes it.
 *
 * Order.  Everything is ordered by the pair (key, id), ascending; ids are unique,
 * so this is a strict total order.
 *   key = sum_j (q_j - x_j)^2          for the L2 metric
 *   key = - sum_j q_j * x_j            for the inner-product metric
 * uint8 data: the key is an exact integer.  fp16 / fp32 data: the key is
 * accumulated in double over j = 0..dim-1 and rounded once to float; comparisons
 * then use that float value.
 *
 * Parity pins (tests/test_oracle_pins.py): reachable-set rule against brute force,
 * complete graph, path-graph closed form with counters, output invariants,
 * slot-order independence, monotonicity in max_iters, exact-visited versus
 * forget-each-iteration equivalence, and the paper's worked traffic example
 * (Sec. 3.2: V = 6*6*32 = 1152 rows per query).  Search results themselves have no
 * printed values in the paper to compare with.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { DT_U8 = 0, DT_F16 = 1, DT_F32 = 2 };
enum { METRIC_L2 = 0, METRIC_IP = 1 };

/* One row of the candidate list: key, id, and whether the node's graph row has
 * been read already. */
typedef struct {
    double key; /* exact integer (uint8) or a float value (fp16/fp32 data) */
    int32_t id;
    int32_t expanded;
} item_t;

static int item_cmp(const void* a, const void* b) {
    const item_t* x = (const item_t*)a;
    const item_t* y = (const item_t*)b;
    if (x->key < y->key) return -1;
    if (x->key > y->key) return 1;
    if (x->id < y->id) return -1;
    if (x->id > y->id) return 1;
    return 0;
}

/* IEEE binary16 -> double, by the format's definition. */
static double half_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* subnormal: m * 2^-10 * 2^-14 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return sign ? -v : v;
}

static double elem(const void* row, int32_t dtype, int32_t j) {
    if (dtype == DT_U8) return (double)((const uint8_t*)row)[j];
    if (dtype == DT_F16) return half_to_double(((const uint16_t*)row)[j]);
    return (double)((const float*)row)[j];
}

/* key(q, x): the quantity the search minimises.  uint8 sums are exact in double
 * (at most 128 * 255^2 per 128 dims, far below 2^53). */
static double key_of(const void* q, const void* x, int32_t dim, int32_t dtype, int32_t metric) {
    double acc = 0.0;
    for (int32_t j = 0; j < dim; ++j) {
        double a = elem(q, dtype, j), b = elem(x, dtype, j);
        if (metric == METRIC_L2)
            acc += (a - b) * (a - b);
        else
            acc -= a * b;
    }
    if (dtype != DT_U8) acc = (double)(float)acc; /* rounded once to fp32 */
    return acc;
}

/* Counter-based generator for the entry nodes, so that the GPU side can implement
 * the same rule on its own: the splitmix64 output function applied to
 * seed + (counter + 1) * golden-ratio constant. */
static uint64_t mix64(uint64_t seed, uint64_t counter) {
    uint64_t z = seed + (counter + 1) * 0x9E3779B97F4A7C15ull;
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

typedef struct {
    const void* vectors;
    int64_t n;
    int32_t dim, dtype;
    int64_t row_stride_bytes;
    const int32_t* graph;
    int32_t degree, metric;
    int32_t n_entry, entry_mode;
    uint64_t seed;
    const void* centroids; /* n_clusters x dim, same dtype as the vectors, dense rows */
    const int64_t* cluster_offsets; /* n_clusters + 1; cluster c owns ids [off[c], off[c+1]) */
    int32_t n_clusters, route_c;
    const int32_t* given_routes; /* NULL, or nq x route_c cluster ids that replace the routing step (stage 1
                                    done elsewhere; an id outside [0, n_clusters) names no cluster) */
} index_t;

static size_t elem_size(int32_t dtype) { return dtype == DT_U8 ? 1 : dtype == DT_F16 ? 2 : 4; }

static const void* row_ptr(const index_t* ix, int64_t id) {
    return (const char*)ix->vectors + id * ix->row_stride_bytes;
}

/* The route_c clusters whose centroids are nearest to q under (key, cluster index).
 * This is the single-GPU form of the paper's Stage 1 (K-means as classifier): it
 * decides where a query enters the graph. */
static void nearest_clusters(const index_t* ix, const void* q, int32_t* out /* route_c */) {
    item_t* c = (item_t*)malloc(sizeof(item_t) * (size_t)ix->n_clusters);
    size_t cs = elem_size(ix->dtype) * (size_t)ix->dim;
    for (int32_t i = 0; i < ix->n_clusters; ++i) {
        c[i].key = key_of(q, (const char*)ix->centroids + cs * (size_t)i, ix->dim, ix->dtype, ix->metric);
        c[i].id = i;
        c[i].expanded = 0;
    }
    qsort(c, (size_t)ix->n_clusters, sizeof(item_t), item_cmp);
    for (int32_t t = 0; t < ix->route_c; ++t) out[t] = c[t].id;
    free(c);
}

/* Entry ids of query number qi (its position in the batch).  Returns how many were
 * written (an empty routed cluster yields none for its slots).  Duplicates are
 * not removed here; the search treats the entries as a set.
 *   mode 0: e_j = z_j mod N
 *   mode 1: slot j goes to the (j mod route_c)-th nearest cluster c and
 *           e_j = off[c] + z_j mod |c|                                        */
static int32_t entries_of(const index_t* ix, const void* q, int64_t qi, int32_t* out) {
    int32_t cnt = 0;
    int32_t* near = NULL;
    if (ix->entry_mode == 1) {
        near = (int32_t*)malloc(sizeof(int32_t) * (size_t)ix->route_c);
        if (ix->given_routes)
            memcpy(near, ix->given_routes + qi * ix->route_c, sizeof(int32_t) * (size_t)ix->route_c);
        else
            nearest_clusters(ix, q, near);
    }
    for (int32_t j = 0; j < ix->n_entry; ++j) {
        uint64_t z = mix64(ix->seed, (uint64_t)qi * (uint64_t)ix->n_entry + (uint64_t)j);
        if (ix->entry_mode == 0) {
            out[cnt++] = (int32_t)(z % (uint64_t)ix->n);
        } else {
            int32_t c = near[j % ix->route_c];
            if (c < 0 || c >= ix->n_clusters) continue; /* only a given route can be such: no cluster, no entry */
            int64_t lo = ix->cluster_offsets[c], hi = ix->cluster_offsets[c + 1];
            if (hi > lo) out[cnt++] = (int32_t)(lo + (int64_t)(z % (uint64_t)(hi - lo)));
        }
    }
    free(near);
    return cnt;
}

/* Exact visited set: one bit per node plus the list of set bits, so that clearing
 * costs only what was touched. */
typedef struct {
    uint8_t* bits;
    int32_t* touched;
    int64_t n_touched, cap;
} seen_t;

static int seen_test(const seen_t* s, int32_t id) { return (s->bits[id >> 3] >> (id & 7)) & 1; }
static void seen_add(seen_t* s, int32_t id) {
    s->bits[id >> 3] |= (uint8_t)(1u << (id & 7));
    if (s->n_touched == s->cap) {
        s->cap = s->cap ? s->cap * 2 : 1024;
        s->touched = (int32_t*)realloc(s->touched, sizeof(int32_t) * (size_t)s->cap);
    }
    s->touched[s->n_touched++] = id;
}
static void seen_clear(seen_t* s) {
    for (int64_t i = 0; i < s->n_touched; ++i) s->bits[s->touched[i] >> 3] = 0;
    s->n_touched = 0;
}

/* One query.  L has room for itopk + (largest batch of new candidates). */
static void search_one(const index_t* ix, const void* q, int64_t qi, int32_t k, int32_t itopk, int32_t width,
                       int32_t max_iters, int32_t forget, seen_t* seen, item_t* L, int32_t* scratch,
                       int32_t* out_ids, void* out_dists, int64_t* n_iters, int64_t* n_dist,
                       int64_t* n_parents) {
    int64_t cnt_dist = 0, cnt_parents = 0, cnt_iters = 0;
    int32_t len = 0;

    /* Step 1: entries.  Paper: the traversal starts "from an entry node"; how many
     * and which is left open.  Here: n_entry per query from the counter-based
     * generator, as a set. */
    int32_t ne = entries_of(ix, q, qi, scratch);
    for (int32_t j = 0; j < ne; ++j) {
        int32_t e = scratch[j];
        if (seen_test(seen, e)) continue;
        seen_add(seen, e);
        L[len].key = key_of(q, row_ptr(ix, e), ix->dim, ix->dtype, ix->metric);
        L[len].id = e;
        L[len].expanded = 0;
        ++len;
        ++cnt_dist;
    }
    qsort(L, (size_t)len, sizeof(item_t), item_cmp);
    if (len > itopk) len = itopk;

    /* Step 2: expansion rounds.  max_iters bounds the rounds (the paper's I);
     * the loop also ends once every list entry has been expanded. */
    for (int32_t it = 0; it < max_iters; ++it) {
        /* 2a: parents = the first min(width, #unexpanded) unexpanded entries in
         * list order (best first).  Fewer than width left: take what exists. */
        int32_t np = 0;
        int32_t* parents = scratch;
        for (int32_t i = 0; i < len && np < width; ++i)
            if (!L[i].expanded) {
                L[i].expanded = 1;
                parents[np++] = L[i].id;
            }
        if (np == 0) break;
        ++cnt_iters;
        cnt_parents += np;

        if (forget) {
            /* Test switch: forget every node scored so far except those in the
             * list.  The result must not change (see the pin that uses it). */
            seen_clear(seen);
            for (int32_t i = 0; i < len; ++i) seen_add(seen, L[i].id);
        }

        /* 2b + 2c: every out-neighbour of a parent that is a valid id and has not
         * been scored yet is scored once and appended. */
        int32_t add = 0;
        for (int32_t p = 0; p < np; ++p) {
            const int32_t* nb = ix->graph + (int64_t)parents[p] * ix->degree;
            for (int32_t s = 0; s < ix->degree; ++s) {
                int32_t v = nb[s];
                if (v < 0 || (int64_t)v >= ix->n) continue; /* empty slot */
                if (seen_test(seen, v)) continue;
                seen_add(seen, v);
                item_t* c = &L[len + add];
                c->key = key_of(q, row_ptr(ix, v), ix->dim, ix->dtype, ix->metric);
                c->id = v;
                c->expanded = 0;
                ++add;
                ++cnt_dist;
            }
        }
        /* 2d: keep the itopk smallest of old list + new candidates; carried
         * entries keep their expanded mark. */
        len += add;
        qsort(L, (size_t)len, sizeof(item_t), item_cmp);
        if (len > itopk) len = itopk;
    }

    /* Step 3: the first k list entries; short lists are padded. */
    for (int32_t r = 0; r < k; ++r) {
        int have = r < len;
        out_ids[r] = have ? L[r].id : -1;
        if (ix->dtype == DT_U8)
            ((int32_t*)out_dists)[r] = have ? (int32_t)L[r].key : INT32_MAX;
        else
            ((float*)out_dists)[r] = have ? (float)L[r].key : INFINITY;
    }
    *n_iters = cnt_iters;
    *n_dist = cnt_dist;
    *n_parents = cnt_parents;
    seen_clear(seen);
}

static index_t make_index(const void* vectors, int64_t n, int32_t dim, int32_t dtype, int64_t row_stride_bytes,
                          const int32_t* graph, int32_t degree, int32_t metric, int32_t n_entry,
                          int32_t entry_mode, uint64_t seed, const void* centroids,
                          const int64_t* cluster_offsets, int32_t n_clusters, int32_t route_c) {
    index_t ix;
    ix.vectors = vectors;
    ix.n = n;
    ix.dim = dim;
    ix.dtype = dtype;
    ix.row_stride_bytes = row_stride_bytes;
    ix.graph = graph;
    ix.degree = degree;
    ix.metric = metric;
    ix.n_entry = n_entry;
    ix.entry_mode = entry_mode;
    ix.seed = seed;
    ix.centroids = centroids;
    ix.cluster_offsets = cluster_offsets;
    ix.n_clusters = n_clusters;
    ix.route_c = route_c;
    ix.given_routes = NULL;
    return ix;
}

/*
 * Beam search for nq queries (dense rows of the index dtype).  Host pointers only.
 * out_ids: nq*k int32.  out_dists: nq*k int32 (uint8 data) or float.
 * counters (each nq int64, may be NULL): expansion rounds, keys computed, graph
 * rows read.  forget_visited != 0 selects the forgetful visited set of the test
 * switch above.  routes (routed entry mode only, may be NULL): nq*route_c cluster ids that
 * are used instead of the routing step, as when stage 1 ran elsewhere (paper Sec. 3.1: the
 * classifier and the search are separate stages).  Returns 0, or -1 on arguments it cannot serve.
 */
int oracle_search_routed(const void* vectors, int64_t n, int32_t dim, int32_t dtype, int64_t row_stride_bytes,
                  const int32_t* graph, int32_t degree, int32_t metric, int32_t n_entry, int32_t entry_mode,
                  uint64_t seed, const void* centroids, const int64_t* cluster_offsets, int32_t n_clusters,
                  int32_t route_c, const void* queries, int64_t nq, int32_t k, int32_t itopk, int32_t width,
                  int32_t max_iters, int32_t forget_visited, int32_t* out_ids, void* out_dists,
                  int64_t* out_iters, int64_t* out_n_dist, int64_t* out_n_parents, int32_t n_threads,
                  const int32_t* routes) {
    if (n < 1 || dim < 1 || degree < 1 || n_entry < 1 || k < 1 || itopk < k || width < 1 || max_iters < 0 ||
        nq < 0)
        return -1;
    if (entry_mode == 1 && (n_clusters < 1 || route_c < 1 || route_c > n_clusters)) return -1;
    index_t ix = make_index(vectors, n, dim, dtype, row_stride_bytes, graph, degree, metric, n_entry, entry_mode,
                            seed, centroids, cluster_offsets, n_clusters, route_c);
    ix.given_routes = entry_mode == 1 ? routes : NULL;
    size_t qbytes = elem_size(dtype) * (size_t)dim;
    int64_t batch = (int64_t)width * degree;
    if (batch < n_entry) batch = n_entry;
    int failed = 0;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
#pragma omp parallel
    {
        seen_t seen;
        seen.bits = (uint8_t*)calloc((size_t)(n + 7) / 8, 1);
        seen.touched = NULL;
        seen.n_touched = 0;
        seen.cap = 0;
        item_t* L = (item_t*)malloc(sizeof(item_t) * (size_t)(itopk + batch));
        int32_t* scratch = (int32_t*)malloc(sizeof(int32_t) * (size_t)batch);
        if (!seen.bits || !L || !scratch) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 4)
            for (int64_t i = 0; i < nq; ++i) {
                int64_t it, nd, np;
                search_one(&ix, (const char*)queries + qbytes * (size_t)i, i, k, itopk, width, max_iters,
                           forget_visited, &seen, L, scratch, out_ids + i * k,
                           (char*)out_dists + (size_t)i * (size_t)k * 4, &it, &nd, &np);
                if (out_iters) out_iters[i] = it;
                if (out_n_dist) out_n_dist[i] = nd;
                if (out_n_parents) out_n_parents[i] = np;
            }
        }
        free(seen.bits);
        free(seen.touched);
        free(L);
        free(scratch);
    }
    return failed ? -1 : 0;
}

/* The same with the routing step done by the oracle itself. */
int oracle_search(const void* vectors, int64_t n, int32_t dim, int32_t dtype, int64_t row_stride_bytes,
                  const int32_t* graph, int32_t degree, int32_t metric, int32_t n_entry, int32_t entry_mode,
                  uint64_t seed, const void* centroids, const int64_t* cluster_offsets, int32_t n_clusters,
                  int32_t route_c, const void* queries, int64_t nq, int32_t k, int32_t itopk, int32_t width,
                  int32_t max_iters, int32_t forget_visited, int32_t* out_ids, void* out_dists,
                  int64_t* out_iters, int64_t* out_n_dist, int64_t* out_n_parents, int32_t n_threads) {
    return oracle_search_routed(vectors, n, dim, dtype, row_stride_bytes, graph, degree, metric, n_entry, entry_mode, seed,
                                centroids, cluster_offsets, n_clusters, route_c, queries, nq, k, itopk, width, max_iters,
                                forget_visited, out_ids, out_dists, out_iters, out_n_dist, out_n_parents, n_threads, NULL);
}

/* How many threads oracle_search will use when asked for n_threads (<=0: default). */
int oracle_threads(int32_t n_threads) {
#ifdef _OPENMP
    return n_threads > 0 ? n_threads : omp_get_max_threads();
#else
    (void)n_threads;
    return 1;
#endif
}

/* Exact top-k of all n vectors under (key, id): the plain definition of k-nearest
 * neighbours, used as ground truth.  Same key function as the search. */
int oracle_bruteforce(const void* vectors, int64_t n, int32_t dim, int32_t dtype, int64_t row_stride_bytes,
                      int32_t metric, const void* queries, int64_t nq, int32_t k, int32_t* out_ids,
                      void* out_dists) {
    if (n < 1 || dim < 1 || k < 1 || nq < 0) return -1;
    size_t qbytes = elem_size(dtype) * (size_t)dim;
#pragma omp parallel
    {
        item_t* all = (item_t*)malloc(sizeof(item_t) * (size_t)n);
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < nq; ++i) {
            const void* q = (const char*)queries + qbytes * (size_t)i;
            for (int64_t v = 0; v < n; ++v) {
                all[v].key = key_of(q, (const char*)vectors + v * row_stride_bytes, dim, dtype, metric);
                all[v].id = (int32_t)v;
                all[v].expanded = 0;
            }
            qsort(all, (size_t)n, sizeof(item_t), item_cmp);
            for (int32_t r = 0; r < k; ++r) {
                int have = r < n;
                out_ids[i * k + r] = have ? all[r].id : -1;
                if (dtype == DT_U8)
                    ((int32_t*)out_dists)[i * k + r] = have ? (int32_t)all[r].key : INT32_MAX;
                else
                    ((float*)out_dists)[i * k + r] = have ? (float)all[r].key : INFINITY;
            }
        }
        free(all);
    }
    return 0;
}

/* key(q, x) for explicit (query, id) pairs, as double: lets tests recompute the
 * distances of ids that some other implementation returned. */
void oracle_keys(const void* vectors, int32_t dim, int32_t dtype, int64_t row_stride_bytes, int32_t metric,
                 const void* queries, int64_t nq, int32_t per_query, const int32_t* ids, double* out_keys) {
    size_t qbytes = elem_size(dtype) * (size_t)dim;
    for (int64_t i = 0; i < nq; ++i)
        for (int32_t r = 0; r < per_query; ++r) {
            int32_t id = ids[i * per_query + r];
            out_keys[i * per_query + r] =
                id < 0 ? INFINITY
                       : key_of((const char*)queries + qbytes * (size_t)i,
                                (const char*)vectors + (int64_t)id * row_stride_bytes, dim, dtype, metric);
        }
}

/* Entry ids per query (nq x n_entry, -1 where a slot produced none), for tests. */
int oracle_entries(int64_t n, int32_t dim, int32_t dtype, int32_t metric, int32_t n_entry, int32_t entry_mode,
                   uint64_t seed, const void* centroids, const int64_t* cluster_offsets, int32_t n_clusters,
                   int32_t route_c, const void* queries, int64_t nq, int32_t* out_entries) {
    if (entry_mode == 1 && (n_clusters < 1 || route_c < 1 || route_c > n_clusters)) return -1;
    index_t ix = make_index(NULL, n, dim, dtype, 0, NULL, 1, metric, n_entry, entry_mode, seed, centroids,
                            cluster_offsets, n_clusters, route_c);
    size_t qbytes = elem_size(dtype) * (size_t)dim;
    for (int64_t i = 0; i < nq; ++i) {
        int32_t* row = out_entries + i * n_entry;
        int32_t c = entries_of(&ix, (const char*)queries + qbytes * (size_t)i, i, row);
        for (int32_t j = c; j < n_entry; ++j) row[j] = -1;
    }
    return 0;
}

/* The route_c nearest clusters per query (nq x route_c), for tests. */
int oracle_route(int32_t dim, int32_t dtype, int32_t metric, const void* centroids, int32_t n_clusters,
                 int32_t route_c, const void* queries, int64_t nq, int32_t* out_clusters) {
    if (n_clusters < 1 || route_c < 1 || route_c > n_clusters) return -1;
    index_t ix = make_index(NULL, 1, dim, dtype, 0, NULL, 1, metric, 1, 1, 0, centroids, NULL, n_clusters, route_c);
    size_t qbytes = elem_size(dtype) * (size_t)dim;
    for (int64_t i = 0; i < nq; ++i)
        nearest_clusters(&ix, (const char*)queries + qbytes * (size_t)i, out_clusters + i * route_c);
    return 0;
}

/*
 * Stage 4 of the paper's workflow (Sec. 3.1, "Combine vector candidate results"), local half.
 *
 * oracle_merge_topk: the origin rank reduces the k*c candidates a query got back to the final
 * top-k.  Plain definition: drop padding (id < 0), sort all candidates of the query by
 * (key, id), keep the first k, pad.  keys: int32 (is_float == 0) or float.
 */
int oracle_merge_topk(int32_t is_float, const int32_t* ids, const void* keys, int64_t nq, int32_t per_query, int32_t k,
                      int32_t* out_ids, void* out_keys) {
    if (nq < 0 || per_query < 1 || k < 1 || k > per_query) return -1;
    item_t* all = (item_t*)malloc(sizeof(item_t) * (size_t)per_query);
    for (int64_t q = 0; q < nq; ++q) {
        int32_t cnt = 0;
        for (int32_t e = 0; e < per_query; ++e) {
            int32_t id = ids[q * per_query + e];
            if (id < 0) continue;
            all[cnt].key = is_float ? (double)((const float*)keys)[q * per_query + e]
                                    : (double)((const int32_t*)keys)[q * per_query + e];
            all[cnt].id = id;
            all[cnt].expanded = 0;
            ++cnt;
        }
        qsort(all, (size_t)cnt, sizeof(item_t), item_cmp);
        for (int32_t r = 0; r < k; ++r) {
            int have = r < cnt;
            out_ids[q * k + r] = have ? all[r].id : -1;
            if (is_float)
                ((float*)out_keys)[q * k + r] = have ? (float)all[r].key : INFINITY;
            else
                ((int32_t*)out_keys)[q * k + r] = have ? (int32_t)all[r].key : INT32_MAX;
        }
    }
    free(all);
    return 0;
}

/* oracle_gather: the vectors of the given ids as dense rows (zeros for id outside [0, n)):
 * what a rank sends back besides the ids. */
void oracle_gather(const void* vectors, int64_t n, int32_t dim, int32_t dtype, int64_t row_stride_bytes,
                   const int32_t* ids, int64_t count, void* out) {
    size_t rb = elem_size(dtype) * (size_t)dim;
    for (int64_t i = 0; i < count; ++i) {
        char* dst = (char*)out + rb * (size_t)i;
        if (ids[i] >= 0 && (int64_t)ids[i] < n)
            memcpy(dst, (const char*)vectors + (int64_t)ids[i] * row_stride_bytes, rb);
        else
            memset(dst, 0, rb);
    }
}

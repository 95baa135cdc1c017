/*
 * libann: batched greedy beam search over a fixed-degree proximity graph, on the
 * graph partition and vector partition one MI355X holds in HBM.
 *
 * This is the per-GPU "parallel vector search" step of Fantasy (Sec. 3.1, stage 3;
 * cost model in Sec. 2 and Sec. 3.2 "Stage 3"): every query starts from entry
 * nodes, repeatedly expands the best not-yet-expanded nodes of a fixed-size
 * candidate list (beam width `width`, out-degree `degree`), scores their
 * neighbours against the query and keeps the `itopk` best, and finally returns
 * the first k.  The optional routed entry rule is the single-GPU form of stage 1
 * ("K-means as classifier", Sec. 3.1): entries are drawn inside the clusters whose
 * centroids are nearest to the query.
 *
 * Plain C ABI: pointers and sizes only.  Every pointer marked DEVICE must be
 * memory of the current HIP device; everything else is host memory.  The library
 * never takes ownership of caller memory.
 *
 * Order everywhere: ascending by (key, id) where
 *     key = sum_j (q_j - x_j)^2      for ANN_L2
 *     key = - sum_j q_j * x_j        for ANN_IP
 * uint8 data gives exact int32 keys; fp16 / fp32 data accumulate in fp32.
 */
#ifndef ANN_H_
#define ANN_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ann_index ann_index_t; /* opaque handle */

enum { ANN_U8 = 0, ANN_F16 = 1, ANN_F32 = 2 };  /* element type of vectors, queries, centroids */
enum { ANN_L2 = 0, ANN_IP = 1 };                /* metric */
enum { ANN_ENTRY_UNIFORM = 0, ANN_ENTRY_ROUTED = 1 };
enum {
    ANN_OK = 0,
    ANN_EINVAL = -1,       /* an argument is wrong (null pointer, size out of range, bad alignment) */
    ANN_EUNSUPPORTED = -2, /* valid in principle, but no kernel variant is built for it */
    ANN_ENOMEM = -3,       /* a host or device allocation failed */
    ANN_EHIP = -4          /* a HIP runtime call failed; ann_last_error() has the text */
};

/*
 * Description of one partition (Sec. 1 and Sec. 3.1: each GPU holds its share of the
 * graph and of the vectors in HBM).  Copied by ann_index_load; the arrays it points
 * to are borrowed and must stay alive and unchanged until ann_free.
 */
typedef struct {
    const void* vectors;      /* DEVICE. n rows, row i at byte offset i*row_stride_bytes, 16-byte aligned */
    int64_t n;                /* number of vectors, 1 .. 2^31-1 */
    int32_t dim;              /* elements per vector, at most 1536 (the d of the cost example in Sec. 3.2);
                                 dim*sizeof(element) must be a multiple of 16 */
    int32_t dtype;            /* ANN_U8 / ANN_F16 / ANN_F32 */
    int64_t row_stride_bytes; /* >= dim*sizeof(element), multiple of 16, below 2^31 (128 keeps rows on cache lines) */
    const int32_t* graph;     /* DEVICE. n*degree ids, row-major; a slot outside [0,n) is empty */
    int32_t degree;           /* out-degree of the graph, >= 1 */
    int32_t metric;           /* ANN_L2 / ANN_IP */
    int32_t n_entry;          /* entry nodes drawn per query, >= 1 */
    int32_t entry_mode;       /* ANN_ENTRY_UNIFORM or ANN_ENTRY_ROUTED */
    uint64_t seed;            /* seed of the counter-based entry generator */
    /* ANN_ENTRY_ROUTED only (ignored otherwise): */
    const void* centroids;          /* DEVICE. n_clusters dense rows of `dim` elements, same dtype */
    const int64_t* cluster_offsets; /* DEVICE. n_clusters+1 ascending ids; cluster c = [off[c], off[c+1]) */
    int32_t n_clusters;             /* >= 1 */
    int32_t route_c;                /* clusters a query is routed to, 1 .. min(n_clusters, 8) */
} ann_index_desc_t;

/*
 * Entry rule.  Entry j (0 <= j < n_entry) of the query at position i of a call uses
 *   z = splitmix64 output for state  seed + (i*n_entry + j + 1) * 0x9E3779B97F4A7C15
 *   uniform:  e = z mod n
 *   routed:   c = the (j mod route_c)-th nearest cluster of the query under
 *             (key(query, centroid), cluster index);  e = off[c] + z mod |c|,
 *             no entry if the cluster is empty.
 * Duplicates count once.  Entries depend on the query's position in the call.
 */

/*
 * Validates `desc`, chooses the kernel variant and returns a handle.
 * The borrowed arrays are not copied.  For a routed index whose rows are a multiple of
 * 32 bytes a small device array (4 bytes per cluster) is allocated and filled on the
 * default stream, which is synchronised before returning; nothing else touches the device.
 * Must be called with the device that owns the arrays current.
 * Errors: ANN_EINVAL, ANN_EUNSUPPORTED, ANN_ENOMEM, ANN_EHIP.
 */
int ann_index_load(const ann_index_desc_t* desc, ann_index_t** out_handle);

/*
 * Tuning and test hooks of a handle.  The defaults are what the measurements use; the options exist
 * so that tests can force the rarely taken paths (a visited hash that overflows, a bitmap shorter
 * than a cluster, the plain routing kernel) and so that a benchmark can time the search without
 * the cluster-grouped execution order.  None of them changes a result (Sec. 3.2 "Stage 3" fixes what
 * is computed; these only choose how).  Must not be called while a search on the handle is being
 * enqueued by another thread.  Errors: ANN_EINVAL (unknown option, value out of range),
 * ANN_EUNSUPPORTED (no kernel variant fits).
 */
enum {
    ANN_OPT_CLUSTER_ORDER_MIN_QUERIES = 0, /* routed batches of at least this many queries run grouped by
                                              cluster (default 16384); 0 = always, negative = never */
    ANN_OPT_VISITED_WINDOW_BITS = 1,       /* bits of the exact visited bitmap over the routed clusters' id
                                              ranges, 0 .. 131072 (default 8192; rounded up to 32); 0 = hash only */
    ANN_OPT_VISITED_HASH_BITS_BIAS = 2,    /* -4 .. 4: log2 factor on the size of the visited hash (default 0);
                                              the hash never gets smaller than the rounds need */
    ANN_OPT_MATRIX_CORE_ROUTING = 3,       /* 0: route with the plain one-wavefront-per-query kernel (default 1) */
    ANN_OPT_LANES_PER_ROW = 4,             /* lanes that share one vector row in the gather, among the built
                                              variants (4, 8 or 32); 0 = the default choice */
    ANN_OPT_WAVEFRONTS_PER_QUERY = 5       /* 1, 2 or 4 wavefronts work on one query (the leader keeps the list, all
                                              share a round's gathers); 0 = chosen per call (default) */
};
int ann_index_set_option(ann_index_t* handle, int option, int64_t value);

/*
 * Enqueues the search of `nq` queries on `stream` and returns without waiting.
 *   queries    DEVICE, nq dense rows of `dim` elements of the index dtype, 16-byte aligned
 *   k          results per query, 1 <= k <= itopk
 *   itopk      size of the candidate list, 1 .. 512
 *   width      nodes expanded per round (beam width w), width*degree <= 512
 *   max_iters  upper bound on expansion rounds (the paper's I), >= 0; the search also
 *              stops when every list entry has been expanded
 *   out_ids    DEVICE, nq*k int32; -1 pads a query that reached fewer than k nodes
 *   out_dists  DEVICE, nq*k keys: int32 for ANN_U8 (pad INT32_MAX), float otherwise (pad +inf)
 *   stream     hipStream_t, NULL for the default stream
 * Results are valid once the stream has been synchronised.  nq == 0 succeeds and
 * launches nothing.  In routed mode one block of stream-ordered scratch (nq*route_c int32 for the
 * routes, the routing's own temporaries, and for batches of 16384 queries or more nq + n_clusters
 * int32 for the cluster-grouped execution order) is allocated and released on `stream`; the
 * runtime may hold the calling thread in that allocation until the previous call on the stream has
 * finished (no wrong result follows from it; ann_search_static does not allocate).  On an
 * argument error nothing is launched and the outputs are untouched.  Calls on
 * different streams may share a handle.  A route id outside [0, n_clusters) (only possible
 * through ann_search_routed) names no cluster: it gives no entries, and a query whose routes
 * all do so returns padding.
 */
int ann_search(ann_index_t* handle, const void* queries, int64_t nq, int k, int itopk, int width, int max_iters,
               int32_t* out_ids, void* out_dists, void* stream);

/*
 * ann_search for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same results, same kernels; the
 * temporaries (routes, execution order, routing partials) live in a device array of
 * ANN_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the library runs on
 * holds it until the process ends).  The call allocates and frees nothing.  Its first call on a
 * device looks up that device's address of the array (one runtime query, no allocation): make one
 * call outside any capture first.
 * Limit: the temporaries of one call, each rounded up to 256 bytes -
 *     4*nq*route_c                       routes
 *   + 8*nq*slices*route_c                routing partials of small batches (slices <= 64, nq*slices <= 131072)
 *   + 4*(nq + n_clusters)                execution order, for batches that run grouped by cluster
 * - must fit: e.g. 1M queries at route_c = 1 take 8.1 MB.  A larger batch gives ANN_EUNSUPPORTED
 * and launches nothing; an index with uniform entries needs no temporaries at all.
 * All calls on one GPU share the array: calls that overlap in time on one GPU (different streams or
 * threads) race and give wrong results; calls on one stream are safe.  The array keeps the last
 * call's contents; everything that must start at zero is cleared by the call itself.
 */
#define ANN_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
int ann_search_static(ann_index_t* handle, const void* queries, int64_t nq, int k, int itopk, int width, int max_iters,
                      int32_t* out_ids, void* out_dists, void* stream);

/*
 * Same as ann_search, and additionally writes four int32 per query to
 * out_counters (DEVICE, nq*4, may be NULL): expansion rounds, keys computed
 * (vector rows gathered), graph rows read, visited-table resets.
 */
int ann_search_counters(ann_index_t* handle, const void* queries, int64_t nq, int k, int itopk, int width,
                        int max_iters, int32_t* out_ids, void* out_dists, int32_t* out_counters, void* stream);

/*
 * The routing step alone (routed indices only): for each query the route_c nearest
 * clusters under (key(query, centroid), cluster index), ascending.
 *   out_clusters  DEVICE, nq*route_c int32
 * Small batches split the centroids over more workgroups and use a stream-ordered scratch of
 * at most nq*64*route_c uint64.
 */
int ann_route(ann_index_t* handle, const void* queries, int64_t nq, int32_t* out_clusters, void* stream);

/*
 * The search step alone for a routed index, with the routing already done: `routes`
 * (DEVICE, nq*route_c int32, as written by ann_route for the same queries) replaces
 * the internal routing pass and its scratch.  Stage 1 and stage 3 of the
 * paper's workflow (Sec. 3.1) can so be issued separately, e.g. on different streams
 * for consecutive batches.  out_counters may be NULL.
 */
int ann_search_routed(ann_index_t* handle, const void* queries, int64_t nq, const int32_t* routes, int k, int itopk,
                      int width, int max_iters, int32_t* out_ids, void* out_dists, int32_t* out_counters,
                      void* stream);

/* Releases the handle and what it owns (never the borrowed arrays).  NULL is accepted. */
int ann_free(ann_index_t* handle);

/* Text of the calling thread's last error; never NULL. */
const char* ann_last_error(void);

/* Bytes of LDS one query's wavefront uses for the given search parameters, or a
 * negative error code; lets callers reason about occupancy. */
int64_t ann_lds_bytes(ann_index_t* handle, int itopk, int width);

/*
 * Stage 4, local half (Sec. 3.1, "Combine vector candidate results": a rank returns the
 * vectors of its top-k, not only their ids).  Copies the rows of `count` ids into dense
 * rows of dim elements; an id outside [0, n) gives a row of zeros.
 *   ids          DEVICE, count int32 (e.g. the nq*k out_ids of a search)
 *   out_vectors  DEVICE, count * dim elements of the index dtype, 16-byte aligned
 */
int ann_gather_vectors(ann_index_t* handle, const int32_t* ids, int64_t count, void* out_vectors, void* stream);

/*
 * Stage 4, merge at the origin (Sec. 3.1 / Sec. 3.2 "Stage 4": the top k*c candidates a query
 * gets back from the c partitions it was sent to are reduced to the final top-k).  Needs no
 * index.  For each of nq queries, `per_query` candidates (any order, 1 .. 512; id < 0 =
 * padding, ignored) are reduced to the k smallest under (key, id), k <= per_query; results
 * are padded like ann_search's.  Candidate ids of one query must be distinct.
 *   ids, keys          DEVICE, nq*per_query int32 / (int32 if key_dtype == ANN_U8, else float)
 *   out_ids, out_keys  DEVICE, nq*k
 */
int ann_merge_topk(int key_dtype, const int32_t* ids, const void* keys, int64_t nq, int per_query, int k,
                   int32_t* out_ids, void* out_keys, void* stream);

/*
 * Index construction, second half: turns a k-nearest-neighbour graph into the fixed-degree
 * graph that ann_search walks.  The paper only names the index it searches (Sec. 3.2,
 * "Stage 3": the CAGRA index); the construction is that index's published graph
 * optimisation, with ranks in place of distances.  Needs no index handle.
 *
 *   knn    DEVICE, n rows of d_in int32: entry j of row x is x's neighbour of rank j (0 = nearest,
 *          e.g. an exact or approximate kNN list in ascending distance).  An entry outside
 *          [0, n) or equal to x is "absent" (padding).  The present ids of a row must be
 *          distinct; with a repeated id the result is unspecified (but no access goes astray).
 *   n      1 .. 2^31 - 1;  d_in 1 .. 128;  d_out 1 .. min(d_in, 64).
 *
 * ann_graph_prune.  Detour count of a present edge x -> y of rank j: the number of ranks
 * i < j whose node z = knn[x][i] is present and lists y at a rank below j.  Row x of `pruned`
 * (DEVICE, n*d_out int32) gets the targets of x's present edges in ascending order of
 * (detour count, rank), cut to d_out and padded with -1.
 *
 * ann_graph_optimize.  pruned as above; then node y collects the sources x of the edges
 * pruned[x][k] == y in ascending order of (k, x), at most d_out of them (its reverse list);
 * row x of `out_graph` (DEVICE, n*d_out int32) is the first d_out - d_out/2 entries of
 * pruned[x], then the first d_out/2 entries of x's reverse list that are not among those,
 * then the remaining entries of pruned[x] that are not in the row yet, cut to d_out and padded
 * with -1.  The result is deterministic.
 *   workspace        DEVICE, 256-byte aligned, at least ann_graph_optimize_workspace_bytes(n, d_in,
 *                    d_out) bytes (about n*d_out*12 + n*12); the caller owns it, its contents
 *                    afterwards are unspecified, and calls that share a workspace must not overlap.
 * Both calls only enqueue work on `stream` and never allocate; out-of-range arguments give
 * ANN_EINVAL / ANN_EUNSUPPORTED before anything is launched.
 * ann_graph_optimize_workspace_bytes returns a negative error code for arguments out of range.
 */
int ann_graph_prune(const int32_t* knn, int64_t n, int d_in, int d_out, int32_t* pruned, void* stream);
int64_t ann_graph_optimize_workspace_bytes(int64_t n, int d_in, int d_out);
int ann_graph_optimize(const int32_t* knn, int64_t n, int d_in, int d_out, int32_t* out_graph, void* workspace,
                       int64_t workspace_bytes, void* stream);

/*
 * Measurement aid, not part of the search: copies `bytes` (a multiple of 16, both
 * pointers DEVICE and 16-byte aligned) with a plain grid-stride kernel named
 * ann_calibration_copy_kernel.  A profiler's HBM byte counters can be calibrated
 * against this transfer of known size (bytes read + bytes written).
 */
int ann_calibration_copy(void* dst, const void* src, int64_t bytes, void* stream);

/*
 * Measurement aid, not part of the search: reads the rows of `count` ids (DEVICE, int32, each in
 * [0, n)) of the index's vector table, 16 bytes per lane, several loads in flight, with a kernel named
 * ann_calibration_gather_kernel, and xors everything it read into *sink (DEVICE, 4 bytes, which the
 * caller zeroes).  With uniformly random ids this measures what the memory system delivers for the
 * search's own access pattern (whole rows at random), the practical ceiling below the HBM peak.
 * An id outside [0, n) is skipped (nothing is read for it).
 */
int ann_calibration_gather(ann_index_t* handle, const int32_t* ids, int64_t count, uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ANN_H_ */

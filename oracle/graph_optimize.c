/*
 * CPU oracle for turning a k-nearest-neighbour graph into the fixed-degree search graph.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file, and it
 * shares no code, header, table or helper with the GPU library.
 *
 * What it follows.  The paper (Fantasy, Sec. 3.2 "Stage 3") says only that each rank
 * searches "the CAGRA index" and prints neither the construction nor a worked example.
 * The construction written out here is the graph optimisation published with that index
 * (Ootomo et al., "CAGRA: Highly Parallel Graph Construction and Approximate Nearest
 * Neighbor Search for GPUs", Sec. on graph optimisation): rank-based pruning of edges
 * that a two-hop route makes redundant, then reverse edges.  Every choice that text
 * leaves open (ties, truncation, the order of a row) is fixed below, next to the
 * line that takes it.  Parity is therefore pinned to this reading, not to values the
 * paper prints: it prints none.
 *
 * Input.  knn is n rows of d_in ids; entry j of row x is x's neighbour of rank j (rank 0
 * = nearest).  An entry outside [0, n), or equal to x, is "absent": it is no edge and no
 * intermediate node.  The present ids of a row must be distinct.
 *
 * Step 1, detour counts.  For a present edge x -> y of rank j,
 *     c(x, j) = #{ i < j : z = knn[x][i] is present and y = knn[z][r] for some r < j }
 * i.e. the number of two-hop routes x -> z -> y whose two edges both have a smaller rank
 * than the edge itself.
 *
 * Step 2, pruning.  pruned[x] = the targets of x's present edges in ascending order of
 * (c(x, j), j), cut to d_out, padded with -1.
 *
 * Step 3, reverse edges.  For a node y the candidates are the pairs (k, x) with
 * pruned[x][k] = y; rev[y] = the x of the d_out smallest pairs in ascending order of
 * (k, x), padded with -1.
 *
 * Step 4, merge.  With h = d_out / 2 (rounded down), row x of the result is
 *     the present entries among pruned[x][0 .. d_out - h),
 *     then the first h entries of rev[x] that are not among those,
 *     then the entries of pruned[x][d_out - h ..) not yet in the row, in order,
 * cut to d_out and padded with -1.  The search reads a row as a set, so only the
 * membership of a row matters to it; the order is fixed so that two implementations can
 * be compared entry by entry.
 *
 * Parity pins (tests/test_oracle_graph_pins.py): detour counts against the boolean matrix
 * product that defines two-hop reachability, a graph worked by hand, graphs without
 * two-hop routes, the transitive tournament's closed form, reverse lists against a
 * global lexicographic sort, and the invariants of the merged rows.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static int present(const int32_t* knn, int64_t n, int32_t d_in, int64_t x, int32_t j) {
    const int32_t y = knn[x * d_in + j];
    return y >= 0 && (int64_t)y < n && (int64_t)y != x;
}

/* Step 1.  counts[x * d_in + j] = c(x, j), or -1 where the entry is absent. */
int oracle_graph_detours(const int32_t* knn, int64_t n, int32_t d_in, int32_t* counts) {
    if (!knn || !counts || n <= 0 || d_in <= 0) return 1;
#pragma omp parallel for schedule(dynamic, 64) /* rows are independent */
    for (int64_t x = 0; x < n; ++x) {
        for (int32_t j = 0; j < d_in; ++j) {
            if (!present(knn, n, d_in, x, j)) {
                counts[x * d_in + j] = -1;
                continue;
            }
            const int32_t y = knn[x * d_in + j];
            int32_t c = 0;
            for (int32_t i = 0; i < j; ++i) {
                if (!present(knn, n, d_in, x, i)) continue;
                const int64_t z = knn[x * d_in + i];
                int found = 0;
                for (int32_t r = 0; r < j && !found; ++r)
                    if (present(knn, n, d_in, z, r) && knn[z * d_in + r] == y) found = 1;
                c += found;
            }
            counts[x * d_in + j] = c;
        }
    }
    return 0;
}

/* Step 2.  pruned is n rows of d_out ids. */
int oracle_graph_prune(const int32_t* knn, int64_t n, int32_t d_in, int32_t d_out, int32_t* pruned) {
    if (!knn || !pruned || n <= 0 || d_in <= 0 || d_out <= 0 || d_out > d_in) return 1;
    int32_t* counts = (int32_t*)malloc((size_t)n * d_in * sizeof(int32_t));
    if (!counts) return 2;
    oracle_graph_detours(knn, n, d_in, counts);
    for (int64_t x = 0; x < n; ++x) {
        int32_t filled = 0;
        /* selection in ascending (count, rank): repeatedly take the smallest pair not taken yet */
        int32_t last_c = -1, last_j = -1;
        while (filled < d_out) {
            int32_t best = -1;
            for (int32_t j = 0; j < d_in; ++j) {
                const int32_t c = counts[x * d_in + j];
                if (c < 0) continue;
                const int after_last = c > last_c || (c == last_c && j > last_j);
                if (!after_last) continue;
                if (best < 0 || c < counts[x * d_in + best]) best = j; /* ranks ascend, so ties keep the smaller j */
            }
            if (best < 0) break;
            pruned[x * d_out + filled++] = knn[x * d_in + best];
            last_c = counts[x * d_in + best];
            last_j = best;
        }
        for (; filled < d_out; ++filled) pruned[x * d_out + filled] = -1;
    }
    free(counts);
    return 0;
}

/* Step 3.  rev is n rows of d ids, from a graph of n rows of d ids. */
int oracle_graph_reverse(const int32_t* pruned, int64_t n, int32_t d, int32_t* rev) {
    if (!pruned || !rev || n <= 0 || d <= 0) return 1;
    int32_t* fill = (int32_t*)calloc((size_t)n, sizeof(int32_t));
    if (!fill) return 2;
    for (int64_t i = 0; i < n * d; ++i) rev[i] = -1;
    /* visiting k in the outer loop and x in the inner one meets the pairs in ascending (k, x) */
    for (int32_t k = 0; k < d; ++k)
        for (int64_t x = 0; x < n; ++x) {
            const int32_t y = pruned[x * d + k];
            if (y < 0 || (int64_t)y >= n || (int64_t)y == x) continue;
            if (fill[y] < d) rev[(int64_t)y * d + fill[y]++] = (int32_t)x;
        }
    free(fill);
    return 0;
}

static int in_row(const int32_t* row, int32_t len, int32_t id) {
    for (int32_t i = 0; i < len; ++i)
        if (row[i] == id) return 1;
    return 0;
}

/* Step 4. */
int oracle_graph_merge(const int32_t* pruned, const int32_t* rev, int64_t n, int32_t d, int32_t* out) {
    if (!pruned || !rev || !out || n <= 0 || d <= 0) return 1;
    const int32_t h = d / 2;
    for (int64_t x = 0; x < n; ++x) {
        int32_t* row = out + x * d;
        int32_t len = 0;
        for (int32_t k = 0; k < d - h; ++k) {
            const int32_t y = pruned[x * d + k];
            if (y >= 0 && (int64_t)y < n && (int64_t)y != x) row[len++] = y;
        }
        int32_t taken = 0;
        for (int32_t k = 0; k < d && taken < h; ++k) {
            const int32_t y = rev[x * d + k];
            if (y < 0) continue;
            if (!in_row(row, len, y)) {
                row[len++] = y;
                ++taken;
            }
        }
        for (int32_t k = d - h; k < d && len < d; ++k) {
            const int32_t y = pruned[x * d + k];
            if (y >= 0 && (int64_t)y < n && (int64_t)y != x && !in_row(row, len, y)) row[len++] = y;
        }
        for (; len < d; ++len) row[len] = -1;
    }
    return 0;
}

/* Steps 1 to 4. */
int oracle_graph_optimize(const int32_t* knn, int64_t n, int32_t d_in, int32_t d_out, int32_t* out) {
    if (!knn || !out || n <= 0 || d_in <= 0 || d_out <= 0 || d_out > d_in) return 1;
    int32_t* pruned = (int32_t*)malloc((size_t)n * d_out * sizeof(int32_t));
    int32_t* rev = (int32_t*)malloc((size_t)n * d_out * sizeof(int32_t));
    int rc = (!pruned || !rev) ? 2 : 0;
    if (!rc) rc = oracle_graph_prune(knn, n, d_in, d_out, pruned);
    if (!rc) rc = oracle_graph_reverse(pruned, n, d_out, rev);
    if (!rc) rc = oracle_graph_merge(pruned, rev, n, d_out, out);
    free(pruned);
    free(rev);
    return rc;
}

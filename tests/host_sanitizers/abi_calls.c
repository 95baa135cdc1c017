/* Drives the host side of libann (argument checks, plans, option handling, error texts) through
 * the C ABI without a GPU.  Built and run by tests/test_host_sanitizers.py against a copy of the
 * library whose host code is compiled with -fsanitize=address,undefined: any out-of-bounds
 * access, leak, misaligned access or undefined arithmetic in those paths aborts the run.
 * No call here reaches a kernel launch. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ann.h"

#define FAKE ((void*)0x7F0000000000ull) /* non-null, 16-byte aligned, never dereferenced on these paths */
#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            fprintf(stderr, "line %d: %s (last error: %s)\n", __LINE__, #cond, ann_last_error()); \
            return 1;                                                            \
        }                                                                        \
    } while (0)

static ann_index_desc_t base_desc(void) {
    ann_index_desc_t d;
    memset(&d, 0, sizeof d);
    d.vectors = FAKE;
    d.n = 1000;
    d.dim = 128;
    d.dtype = ANN_U8;
    d.row_stride_bytes = 128;
    d.graph = (const int32_t*)FAKE;
    d.degree = 32;
    d.metric = ANN_L2;
    d.n_entry = 32;
    d.entry_mode = ANN_ENTRY_UNIFORM;
    d.seed = 1;
    return d;
}

int main(void) {
    ann_index_t* h = NULL;
    ann_index_desc_t d = base_desc();
    CHECK(ann_index_load(NULL, &h) == ANN_EINVAL);
    CHECK(ann_index_load(&d, NULL) == ANN_EINVAL);
    CHECK(ann_index_load(&d, &h) == ANN_OK && h);
    /* every list size, width and entry count the planner accepts or refuses */
    for (int itopk = -1; itopk <= 520; ++itopk)
        for (int width = -1; width <= 66; width += (width < 18 ? 1 : 16)) {
            int64_t lds = ann_lds_bytes(h, itopk, width);
            int ok = itopk >= 1 && itopk <= 512 && width >= 1 && width <= 64 && width * 32 <= 512;
            CHECK(ok ? lds > 0 && lds <= 160 * 1024 : lds == ANN_EUNSUPPORTED);
        }
    CHECK(ann_search(h, FAKE, 0, 10, 64, 1, 5, NULL, NULL, NULL) == ANN_OK);
    CHECK(ann_search(h, FAKE, -1, 10, 64, 1, 5, (int32_t*)FAKE, FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_search(h, FAKE, 4, 65, 64, 1, 5, (int32_t*)FAKE, FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_search(h, FAKE, 4, 10, 64, 1, -1, (int32_t*)FAKE, FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_search(h, (char*)FAKE + 4, 4, 10, 64, 1, 5, (int32_t*)FAKE, FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_search(h, NULL, 4, 10, 64, 1, 5, (int32_t*)FAKE, FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_search_counters(h, FAKE, 4, 10, 64, 1, 5, NULL, FAKE, NULL, NULL) == ANN_EINVAL);
    CHECK(ann_search_static(h, FAKE, 0, 10, 64, 1, 5, (int32_t*)FAKE, FAKE, NULL) == ANN_OK);
    CHECK(ann_search_static(h, FAKE, 4, 0, 64, 1, 5, (int32_t*)FAKE, FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_search_routed(h, FAKE, 4, (const int32_t*)FAKE, 10, 64, 1, 5, (int32_t*)FAKE, FAKE, NULL, NULL) == ANN_EINVAL);
    CHECK(ann_route(h, FAKE, 4, (int32_t*)FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_gather_vectors(h, (const int32_t*)FAKE, -1, FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_gather_vectors(h, (const int32_t*)FAKE, 0, FAKE, NULL) == ANN_OK);
    CHECK(ann_calibration_gather(h, NULL, 8, (uint32_t*)FAKE, NULL) == ANN_EINVAL);
    for (int opt = -1; opt <= 6; ++opt)
        for (int64_t v = -5; v <= 5; ++v) (void)ann_index_set_option(h, opt, v);
    CHECK(ann_index_set_option(h, ANN_OPT_VISITED_WINDOW_BITS, 1 << 17) == ANN_OK);
    CHECK(ann_index_set_option(h, ANN_OPT_VISITED_WINDOW_BITS, (1 << 17) + 1) == ANN_EINVAL);
    CHECK(ann_index_set_option(h, ANN_OPT_LANES_PER_ROW, 8) == ANN_OK);
    CHECK(ann_index_set_option(h, ANN_OPT_LANES_PER_ROW, 32) == ANN_OK);
    CHECK(ann_index_set_option(h, ANN_OPT_LANES_PER_ROW, 16) == ANN_EUNSUPPORTED);
    CHECK(strlen(ann_last_error()) > 0);
    CHECK(ann_free(h) == ANN_OK);
    CHECK(ann_free(NULL) == ANN_OK);

    /* a routed index on 400-byte rows: no matrix-core routing, so loading touches no device */
    d = base_desc();
    d.dtype = ANN_F32;
    d.dim = 100;
    d.row_stride_bytes = 400;
    d.entry_mode = ANN_ENTRY_ROUTED;
    d.centroids = FAKE;
    d.cluster_offsets = (const int64_t*)FAKE;
    d.n_clusters = 40;
    d.route_c = 9;
    CHECK(ann_index_load(&d, &h) == ANN_EINVAL && !h);
    d.route_c = 8;
    CHECK(ann_index_load(&d, &h) == ANN_OK && h);
    CHECK(ann_lds_bytes(h, 256, 4) > 0);
    CHECK(ann_index_set_option(h, ANN_OPT_VISITED_WINDOW_BITS, 0) == ANN_OK);
    CHECK(ann_lds_bytes(h, 512, 5) > 0);
    /* beyond the static scratch: refused before anything is looked up or launched */
    CHECK(ann_search_static(h, FAKE, (int64_t)ANN_STATIC_SCRATCH_BYTES, 10, 64, 1, 5, (int32_t*)FAKE, FAKE, NULL) == ANN_EUNSUPPORTED);
    CHECK(strstr(ann_last_error(), "static scratch") != NULL);
    CHECK(ann_search_routed(h, FAKE, 4, NULL, 10, 64, 1, 5, (int32_t*)FAKE, FAKE, NULL, NULL) == ANN_EINVAL);
    CHECK(ann_free(h) == ANN_OK);

    /* descriptors that must be refused */
    d = base_desc();
    d.n = 0;
    CHECK(ann_index_load(&d, &h) == ANN_EINVAL);
    d = base_desc();
    d.row_stride_bytes = (int64_t)1 << 31;
    CHECK(ann_index_load(&d, &h) == ANN_EINVAL);
    d = base_desc();
    d.dim = 1552;
    d.row_stride_bytes = 1552;
    CHECK(ann_index_load(&d, &h) == ANN_EUNSUPPORTED);

    /* entry points without a handle */
    CHECK(ann_merge_topk(ANN_U8, (const int32_t*)FAKE, FAKE, 0, 30, 10, (int32_t*)FAKE, FAKE, NULL) == ANN_OK);
    CHECK(ann_merge_topk(ANN_U8, (const int32_t*)FAKE, FAKE, 4, 513, 10, (int32_t*)FAKE, FAKE, NULL) == ANN_EUNSUPPORTED);
    CHECK(ann_merge_topk(7, (const int32_t*)FAKE, FAKE, 4, 30, 10, (int32_t*)FAKE, FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_graph_prune((const int32_t*)FAKE, 0, 64, 32, (int32_t*)FAKE, NULL) == ANN_EINVAL);
    CHECK(ann_graph_prune((const int32_t*)FAKE, 1000, 129, 32, (int32_t*)FAKE, NULL) == ANN_EUNSUPPORTED);
    CHECK(ann_graph_optimize_workspace_bytes(100000000, 64, 32) > 38000000000ll);
    CHECK(ann_graph_optimize((const int32_t*)FAKE, 1000, 64, 32, (int32_t*)FAKE, FAKE, 16, NULL) == ANN_EINVAL);
    CHECK(ann_calibration_copy(FAKE, FAKE, 24, NULL) == ANN_EINVAL);
    CHECK(ann_calibration_copy(FAKE, FAKE, 0, NULL) == ANN_OK);
    puts("host paths clean");
    return 0;
}

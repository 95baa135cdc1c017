// Host side of libann: argument checks, choice of kernel variant, launches.
// Declarations and the meaning of every argument: include/ann.h.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "ann.h"
#include "combine.h"
#include "graph_build.h"
#include "route_mfma.h"
#include "route_mfma_u8.h"
#include "schedule.h"
#include "variants.h"

namespace ann {

// explicit specialisations live in the inst_*.hip files
#define ANN_DECLARE(DT, METRIC, G, NCH)                                                                           \
    template <>                                                                                                  \
    hipError_t launch_search<DT, METRIC, G, NCH>(const SearchParams&, int, int, unsigned, size_t, hipStream_t);   \
    template <>                                                                                                  \
    hipError_t launch_route<DT, METRIC, G, NCH>(const RouteParams&, hipStream_t);
ANN_ROW_VARIANTS(ANN_DECLARE)
#undef ANN_DECLARE

struct RowVariant {
    int dtype, metric, g, nch;
    hipError_t (*search)(const SearchParams&, int, int, unsigned, size_t, hipStream_t);
    hipError_t (*route)(const RouteParams&, hipStream_t);
};

#define ANN_ENTRY(DT, METRIC, G, NCH) {DT, METRIC, G, NCH, &launch_search<DT, METRIC, G, NCH>, &launch_route<DT, METRIC, G, NCH>},
static const RowVariant kRowVariants[] = {ANN_ROW_VARIANTS(ANN_ENTRY)};
#undef ANN_ENTRY

static thread_local char g_error[512] = "";

static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

static int elem_size(int dtype) { return dtype == ANN_U8 ? 1 : dtype == ANN_F16 ? 2 : 4; }

constexpr uint32_t kMagic = 0x414e4e31u;  // "ANN1"
constexpr int kMaxItopk = 512, kMaxBatch = 512, kMaxWidth = 64;
constexpr int64_t kMaxQueriesPerLaunch = 1 << 22;
// Visited bitmap over the routed clusters: 8192 ids cover a cluster of the 100M / 16384
// partition (about 6100 ids) with room to spare; ids beyond it use the hash.
constexpr int kDefaultWindowBits = 8192, kMaxWindowBits = 1 << 17;
// From this batch size on, a routed batch is executed grouped by cluster (schedule.hip).
constexpr int64_t kMinQueriesForClusterOrder = 16384;

}  // namespace ann

struct ann_index {
    uint32_t magic;
    ann_index_desc_t d;
    int row_bytes;
    const ann::RowVariant* variant;
    // set by ann_index_set_option:
    int hash_bits_bias;       // extra (or fewer) bits for the visited hash
    int window_bits;          // size of the visited bitmap over the routed clusters' ids
    int64_t cluster_order_min;  // batches of at least this many queries run grouped by cluster; < 0: never
    int team;                   // wavefronts per query; 0: chosen per call from the batch size and the row length
    bool matrix_core_routing;
    int32_t* centroid_bias;  // DEVICE, owned: per-centroid term of the uint8 d=128 matrix-core routing, or null
    void* route_bias;        // DEVICE, owned: the same for the general matrix-core routing, or null
};

using namespace ann;

// The smallest variant that covers the row; among equals the one with fewer lanes per row (more rows
// per instruction).  lanes != 0 restricts the choice to variants with that many lanes per row.
static const RowVariant* pick_variant(int dtype, int metric, int64_t row_bytes, int lanes) {
    const RowVariant* best = nullptr;
    for (const RowVariant& v : kRowVariants)
        if (v.dtype == dtype && v.metric == metric && (int64_t)v.g * v.nch * 16 >= row_bytes && (lanes == 0 || v.g == lanes) &&
            (!best || v.g * v.nch < best->g * best->nch || (v.g * v.nch == best->g * best->nch && v.g < best->g)))
            best = &v;
    return best;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" const char* ann_last_error(void) { return g_error; }

extern "C" int ann_index_load(const ann_index_desc_t* desc, ann_index_t** out_handle) {
    if (!desc || !out_handle) return fail(ANN_EINVAL, "ann_index_load: null argument");
    *out_handle = nullptr;
    const ann_index_desc_t& d = *desc;
    if (!d.vectors || !d.graph) return fail(ANN_EINVAL, "ann_index_load: vectors and graph must not be null");
    if (d.n < 1 || d.n > 2147483647ll) return fail(ANN_EINVAL, "ann_index_load: n = %lld outside 1..2^31-1", (long long)d.n);
    if (d.dtype != ANN_U8 && d.dtype != ANN_F16 && d.dtype != ANN_F32)
        return fail(ANN_EINVAL, "ann_index_load: unknown dtype %d", d.dtype);
    if (d.metric != ANN_L2 && d.metric != ANN_IP) return fail(ANN_EINVAL, "ann_index_load: unknown metric %d", d.metric);
    if (d.dim < 1) return fail(ANN_EINVAL, "ann_index_load: dim = %d", d.dim);
    const int64_t row_bytes = (int64_t)d.dim * elem_size(d.dtype);
    if (row_bytes % 16 != 0)
        return fail(ANN_EINVAL, "ann_index_load: a row of %lld bytes is not a multiple of 16", (long long)row_bytes);
    if (d.row_stride_bytes < row_bytes || d.row_stride_bytes % 16 != 0 || d.row_stride_bytes > INT32_MAX)
        return fail(ANN_EINVAL,
                    "ann_index_load: row_stride_bytes = %lld (rows are %lld bytes; must be a multiple of 16 below 2^31)",
                    (long long)d.row_stride_bytes, (long long)row_bytes);
    if (!aligned16(d.vectors)) return fail(ANN_EINVAL, "ann_index_load: vectors not 16-byte aligned");
    if (d.degree < 1 || d.degree > kMaxBatch) return fail(ANN_EINVAL, "ann_index_load: degree = %d outside 1..%d", d.degree, kMaxBatch);
    if (d.n_entry < 1 || d.n_entry > kMaxBatch)
        return fail(ANN_EINVAL, "ann_index_load: n_entry = %d outside 1..%d", d.n_entry, kMaxBatch);
    if (d.entry_mode != ANN_ENTRY_UNIFORM && d.entry_mode != ANN_ENTRY_ROUTED)
        return fail(ANN_EINVAL, "ann_index_load: unknown entry_mode %d", d.entry_mode);
    if (d.entry_mode == ANN_ENTRY_ROUTED) {
        if (!d.centroids || !d.cluster_offsets) return fail(ANN_EINVAL, "ann_index_load: routed entries need centroids and cluster_offsets");
        if (!aligned16(d.centroids)) return fail(ANN_EINVAL, "ann_index_load: centroids not 16-byte aligned");
        if (d.n_clusters < 1) return fail(ANN_EINVAL, "ann_index_load: n_clusters = %d", d.n_clusters);
        if (d.route_c < 1 || d.route_c > d.n_clusters || d.route_c > kMaxRouteC)
            return fail(ANN_EINVAL, "ann_index_load: route_c = %d outside 1..min(n_clusters, %d)", d.route_c, kMaxRouteC);
    }
    const RowVariant* best = pick_variant(d.dtype, d.metric, row_bytes, 0);
    if (!best) return fail(ANN_EUNSUPPORTED, "ann_index_load: no kernel variant for rows of %lld bytes of this dtype", (long long)row_bytes);
    ann_index* h = new (std::nothrow) ann_index;
    if (!h) return fail(ANN_ENOMEM, "ann_index_load: out of host memory");
    h->magic = kMagic;
    h->d = d;
    h->row_bytes = (int)row_bytes;
    h->variant = best;
    h->hash_bits_bias = 0;
    h->window_bits = d.entry_mode == ANN_ENTRY_ROUTED ? kDefaultWindowBits : 0;
    h->cluster_order_min = kMinQueriesForClusterOrder;
    h->team = 0;
    h->matrix_core_routing = true;
    h->centroid_bias = nullptr;
    h->route_bias = nullptr;
    const bool mfma_route = d.entry_mode == ANN_ENTRY_ROUTED;
    if (mfma_route && !(d.dtype == ANN_U8 && d.dim == 128) && row_bytes % 32 == 0) {
        hipError_t e = hipMalloc(&h->route_bias, 4 * (size_t)route_mfma_padded(d.n_clusters));
        if (e == hipSuccess)
            e = launch_route_bias(d.dtype, d.metric, static_cast<const uint8_t*>(d.centroids), d.n_clusters,
                                  (int)row_bytes, h->route_bias, nullptr);
        if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
        if (e != hipSuccess) {
            if (h->route_bias) (void)hipFree(h->route_bias);
            delete h;
            return fail(e == hipErrorOutOfMemory ? ANN_ENOMEM : ANN_EHIP, "ann_index_load: preparing the routing failed: %s",
                        hipGetErrorString(e));
        }
    }
    if (mfma_route && d.dtype == ANN_U8 && d.dim == 128) {
        // routing runs on the matrix cores; its per-centroid term is computed once, here
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&h->centroid_bias),
                                 sizeof(int32_t) * (size_t)route_mfma_u8_padded(d.n_clusters));
        if (e == hipSuccess)
            e = launch_centroid_bias_u8(d.metric, static_cast<const uint8_t*>(d.centroids), d.n_clusters,
                                        h->centroid_bias, nullptr);
        if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
        if (e != hipSuccess) {
            if (h->centroid_bias) (void)hipFree(h->centroid_bias);
            delete h;
            return fail(e == hipErrorOutOfMemory ? ANN_ENOMEM : ANN_EHIP, "ann_index_load: preparing the routing failed: %s",
                        hipGetErrorString(e));
        }
    }
    *out_handle = h;
    return ANN_OK;
}

extern "C" int ann_free(ann_index_t* h) {
    if (!h) return ANN_OK;
    if (h->magic != kMagic) return fail(ANN_EINVAL, "ann_free: not a live handle");
    h->magic = 0;
    if (h->centroid_bias) (void)hipFree(h->centroid_bias);
    if (h->route_bias) (void)hipFree(h->route_bias);
    delete h;
    return ANN_OK;
}

namespace {

struct Plan {
    int list_variant, cap, hash_bits;
    size_t lds_bytes;
};

int make_plan(const ann_index* h, int itopk, int width, Plan* plan, const char* who) {
    if (itopk < 1 || itopk > kMaxItopk) return fail(ANN_EUNSUPPORTED, "%s: itopk = %d outside 1..%d", who, itopk, kMaxItopk);
    if (width < 1 || width > kMaxWidth) return fail(ANN_EUNSUPPORTED, "%s: width = %d outside 1..%d", who, width, kMaxWidth);
    const int64_t batch = (int64_t)width * h->d.degree;
    if (batch > kMaxBatch) return fail(ANN_EUNSUPPORTED, "%s: width*degree = %lld above %d", who, (long long)batch, kMaxBatch);
    const int need = (int)(batch > h->d.n_entry ? batch : h->d.n_entry);
    int lv = -1;
    for (int i = 0; i < kNumListVariants; ++i)
        if (64 * kListVariants[i][0] >= itopk && 64 * kListVariants[i][1] >= need) {
            lv = i;
            break;
        }
    if (lv < 0) return fail(ANN_EUNSUPPORTED, "%s: no list variant for itopk = %d, batch = %d", who, itopk, need);
    plan->list_variant = lv;
    plan->cap = 64 * kListVariants[lv][1];
    // the table is emptied once 3/4 full; right after that it holds <= itopk ids and one
    // round adds <= need, so 3/4 of its size must cover itopk + need
    int bits = 6;
    while (((3 << bits) >> 2) < itopk + need) ++bits;
    bits += (h->window_bits ? 0 : 1) + h->hash_bits_bias;  // without a bitmap: one more bit, so that resets are rarer
    while (((3 << bits) >> 2) < itopk + need) ++bits;
    if (bits > 13) bits = 13;
    plan->hash_bits = bits;
    // words: round scratch (keys + ids, or a copy of the list), parents, window table, bitmap, hash
    const size_t scratch = 3 * (size_t)plan->cap > 128 * (size_t)kListVariants[lv][0] ? 3 * (size_t)plan->cap
                                                                                   : 128 * (size_t)kListVariants[lv][0];
    plan->lds_bytes = sizeof(uint32_t) * (scratch + 64 + 32 + 8 + (size_t)h->window_bits / 32 + (size_t(1) << bits));
    return ANN_OK;
}

}  // namespace

extern "C" int64_t ann_lds_bytes(ann_index_t* h, int itopk, int width) {
    if (!h || h->magic != kMagic) return fail(ANN_EINVAL, "ann_lds_bytes: not a live handle");
    Plan plan;
    const int rc = make_plan(h, itopk, width, &plan, "ann_lds_bytes");
    return rc != ANN_OK ? rc : (int64_t)plan.lds_bytes;
}

extern "C" int ann_index_set_option(ann_index_t* h, int option, int64_t value) {
    if (!h || h->magic != kMagic) return fail(ANN_EINVAL, "ann_index_set_option: not a live handle");
    switch (option) {
        case ANN_OPT_CLUSTER_ORDER_MIN_QUERIES:
            h->cluster_order_min = value;
            return ANN_OK;
        case ANN_OPT_VISITED_WINDOW_BITS:
            if (value < 0 || value > kMaxWindowBits)
                return fail(ANN_EINVAL, "ann_index_set_option: visited window of %lld bits outside 0..%d", (long long)value, kMaxWindowBits);
            h->window_bits = h->d.entry_mode == ANN_ENTRY_ROUTED ? (int)((value + 31) / 32 * 32) : 0;
            return ANN_OK;
        case ANN_OPT_VISITED_HASH_BITS_BIAS:
            if (value < -4 || value > 4) return fail(ANN_EINVAL, "ann_index_set_option: hash bits bias %lld outside -4..4", (long long)value);
            h->hash_bits_bias = (int)value;
            return ANN_OK;
        case ANN_OPT_MATRIX_CORE_ROUTING:
            h->matrix_core_routing = value != 0;
            return ANN_OK;
        case ANN_OPT_WAVEFRONTS_PER_QUERY:
            if (value != 0 && value != 1 && value != 2 && value != 4)
                return fail(ANN_EUNSUPPORTED, "ann_index_set_option: %lld wavefronts per query (0, 1, 2 or 4)", (long long)value);
            h->team = (int)value;
            return ANN_OK;
        case ANN_OPT_LANES_PER_ROW: {
            const RowVariant* v = value < 0 || value > 64 ? nullptr : pick_variant(h->d.dtype, h->d.metric, h->row_bytes, (int)value);
            if (!v)
                return fail(ANN_EUNSUPPORTED, "ann_index_set_option: no kernel variant with %lld lanes per row for this index", (long long)value);
            h->variant = v;
            return ANN_OK;
        }
        default:
            return fail(ANN_EINVAL, "ann_index_set_option: unknown option %d", option);
    }
}

namespace {

// Where a call's temporaries come from: consecutive 256-byte aligned pieces of one block, which is either
// given (the static scratch) or one stream-ordered allocation of `reserve` bytes, made when the first piece
// is asked for and released on the same stream once the call has enqueued its work.  One allocation per
// call, not one per temporary: on the host an allocate/release pair costs as much as several kernel launches
// (with two pairs per call, small batches in flight on four streams reached 11.9 M queries/s, with one 14.8 M).
struct Workspace {
    hipStream_t stream;
    char* base = nullptr;
    size_t bytes = 0, used = 0;
    size_t reserve = 0;  // > 0: the block is this call's own allocation (made on first use)
    bool owned = false;

    Workspace(hipStream_t s, size_t reserve_bytes) : stream(s), reserve(reserve_bytes) {}
    Workspace(hipStream_t s, void* buffer, size_t buffer_bytes) : stream(s), base(static_cast<char*>(buffer)), bytes(buffer_bytes) {}
    Workspace(const Workspace&) = delete;

    // DEVICE memory of `n` bytes, 256-byte aligned, or null (the reason in *err).
    void* take(size_t n, hipError_t* err) {
        *err = hipSuccess;
        if (!base && reserve > 0) {
            void* p = nullptr;
            *err = hipMallocAsync(&p, reserve, stream);
            if (*err != hipSuccess) return nullptr;
            base = static_cast<char*>(p);
            bytes = reserve;
            owned = true;
        }
        const size_t at = (used + 255) / 256 * 256;
        if (!base || at + n > bytes) {
            *err = hipErrorOutOfMemory;
            return nullptr;
        }
        used = at + n;
        return base + at;
    }
    ~Workspace() {
        if (owned) (void)hipFreeAsync(base, stream);
    }
};

size_t padded256(size_t n) { return (n + 255) / 256 * 256; }

// Bytes of temporaries the routing of nq queries takes.
size_t route_scratch_bytes(const ann_index_t* h, int64_t nq) {
    if (nq <= 0 || !(h->matrix_core_routing && (h->centroid_bias || h->route_bias))) return 0;
    const int slices = h->centroid_bias ? route_mfma_u8_slices(h->d.n_clusters, nq) : route_mfma_slices(h->d.n_clusters, nq);
    return slices > 1 ? padded256(sizeof(uint64_t) * (size_t)nq * slices * h->d.route_c) : 0;
}

// Bytes of temporaries a whole search call of nq queries takes (what Workspace::take hands out): the routes and
// the routing's own temporaries unless the caller brings the routes, and the execution order of a large batch.
size_t search_scratch_bytes(const ann_index_t* h, int64_t nq, bool routes_given) {
    if (h->d.entry_mode != ANN_ENTRY_ROUTED || nq <= 0) return 0;
    size_t need = 0;
    if (!routes_given) need += padded256(sizeof(int32_t) * (size_t)nq * h->d.route_c) + route_scratch_bytes(h, nq);
    if (h->cluster_order_min >= 0 && nq >= h->cluster_order_min) need += padded256(sizeof(int32_t) * ((size_t)nq + h->d.n_clusters));
    return need;
}

int route_impl(ann_index_t* h, const void* queries, int64_t nq, int32_t* out_clusters, Workspace& ws) {
    hipStream_t st = ws.stream;
    if (h->matrix_core_routing && (h->centroid_bias || h->route_bias)) {
        // matrix-core routing; small batches cut the centroid range into slices and merge them
        const int slices = h->centroid_bias ? route_mfma_u8_slices(h->d.n_clusters, nq) : route_mfma_slices(h->d.n_clusters, nq);
        uint64_t* partial = nullptr;
        if (slices > 1) {
            hipError_t e;
            partial = static_cast<uint64_t*>(ws.take(sizeof(uint64_t) * (size_t)nq * slices * h->d.route_c, &e));
            if (!partial) return fail(ANN_ENOMEM, "ann_route: no scratch memory for %d centroid slices: %s", slices, hipGetErrorString(e));
        }
        const uint8_t* cen = static_cast<const uint8_t*>(h->d.centroids);
        const uint8_t* qs = static_cast<const uint8_t*>(queries);
        const hipError_t e =
            h->centroid_bias ? launch_route_mfma_u8(h->d.metric, h->d.route_c, cen, h->centroid_bias, h->d.n_clusters, qs, nq,
                                                    out_clusters, partial, slices, st)
                             : launch_route_mfma(h->d.dtype, h->d.metric, h->d.route_c, cen, h->route_bias, h->d.n_clusters,
                                                 h->row_bytes, qs, nq, out_clusters, partial, slices, st);
        if (e != hipSuccess) return fail(ANN_EHIP, "ann_route: launch failed: %s", hipGetErrorString(e));
        return ANN_OK;
    }
    for (int64_t q0 = 0; q0 < nq; q0 += kMaxQueriesPerLaunch) {
        RouteParams rp;
        rp.centroids = static_cast<const uint8_t*>(h->d.centroids);
        rp.n_clusters = h->d.n_clusters;
        rp.row_bytes = h->row_bytes;
        rp.queries = static_cast<const uint8_t*>(queries) + q0 * h->row_bytes;
        rp.nq = nq - q0 < kMaxQueriesPerLaunch ? nq - q0 : kMaxQueriesPerLaunch;
        rp.route_c = h->d.route_c;
        rp.out = out_clusters + q0 * h->d.route_c;
        const hipError_t e = h->variant->route(rp, st);
        if (e != hipSuccess) return fail(ANN_EHIP, "ann_route: launch failed: %s", hipGetErrorString(e));
    }
    return ANN_OK;
}

}  // namespace

extern "C" int ann_route(ann_index_t* h, const void* queries, int64_t nq, int32_t* out_clusters, void* stream) {
    if (!h || h->magic != kMagic) return fail(ANN_EINVAL, "ann_route: not a live handle");
    if (h->d.entry_mode != ANN_ENTRY_ROUTED) return fail(ANN_EINVAL, "ann_route: the index has no centroids");
    if (nq < 0) return fail(ANN_EINVAL, "ann_route: nq = %lld", (long long)nq);
    if (nq == 0) return ANN_OK;
    if (!queries || !out_clusters) return fail(ANN_EINVAL, "ann_route: null argument");
    if (!aligned16(queries)) return fail(ANN_EINVAL, "ann_route: queries not 16-byte aligned");
    Workspace ws(static_cast<hipStream_t>(stream), route_scratch_bytes(h, nq));
    return route_impl(h, queries, nq, out_clusters, ws);
}

namespace {

// Wavefronts per query when the caller has not fixed them.  A team pays where a round's gathers are the
// long pole and the chip is not full anyway: long rows (a wavefront covers few of them per instruction and
// has a bounded number of loads in flight) and a batch that leaves most wavefront slots empty.
int default_team(const ann_index_t* h, int64_t nq) {
    if (h->row_bytes >= 1024) return 4;               // 1536-byte rows: +15 % even at 50 000 queries per launch
    if (h->row_bytes >= 256 && nq <= 2048) return 4;  // 384-byte rows: a few percent, small batches only
    return 1;                                         // 128-byte rows: a round's gathers are one instruction group
}

// Checks the arguments of a search and launches it; `route` is null for uniform entries.
int search_impl(ann_index_t* h, const void* queries, int64_t nq, const int32_t* route, bool route_given, int k,
                int itopk, int width, int max_iters, int32_t* out_ids, void* out_dists, int32_t* out_counters,
                Workspace& ws) {
    hipStream_t stream = ws.stream;
    if (nq < 0) return fail(ANN_EINVAL, "ann_search: nq = %lld", (long long)nq);
    if (k < 1 || k > itopk) return fail(ANN_EINVAL, "ann_search: k = %d outside 1..itopk (%d)", k, itopk);
    if (max_iters < 0) return fail(ANN_EINVAL, "ann_search: max_iters = %d", max_iters);
    if (route_given && h->d.entry_mode != ANN_ENTRY_ROUTED)
        return fail(ANN_EINVAL, "ann_search_routed: the index does not use routed entries");
    Plan plan;
    const int rc = make_plan(h, itopk, width, &plan, "ann_search");
    if (rc != ANN_OK) return rc;
    if (nq == 0) return ANN_OK;
    if (!queries || !out_ids || !out_dists || (route_given && !route)) return fail(ANN_EINVAL, "ann_search: null argument");
    if (!aligned16(queries)) return fail(ANN_EINVAL, "ann_search: queries not 16-byte aligned");

    if (h->d.entry_mode == ANN_ENTRY_ROUTED && !route_given) {
        hipError_t e;
        int32_t* routes = static_cast<int32_t*>(ws.take(sizeof(int32_t) * (size_t)nq * h->d.route_c, &e));
        if (!routes) return fail(ANN_ENOMEM, "ann_search: no scratch memory for the routes: %s", hipGetErrorString(e));
        const int r = route_impl(h, queries, nq, routes, ws);
        if (r != ANN_OK) return r;
        route = routes;
    }
    // routed batches that are large enough run grouped by cluster, for cache reuse
    int32_t* order = nullptr;
    if (h->d.entry_mode == ANN_ENTRY_ROUTED && h->cluster_order_min >= 0 && nq >= h->cluster_order_min && nq <= 2147483647ll) {
        hipError_t e;
        order = static_cast<int32_t*>(ws.take(sizeof(int32_t) * ((size_t)nq + h->d.n_clusters), &e));
        if (!order) return fail(ANN_ENOMEM, "ann_search: no scratch memory for the execution order: %s", hipGetErrorString(e));
        e = launch_cluster_order(route, h->d.route_c, nq, h->d.n_clusters, order + nq, order, stream);
        if (e != hipSuccess) return fail(ANN_EHIP, "ann_search: launching the execution-order kernels failed: %s", hipGetErrorString(e));
    }

    const int team = h->team ? h->team : default_team(h, nq);
    for (int64_t q0 = 0; q0 < nq; q0 += kMaxQueriesPerLaunch) {
        const int64_t cnt = nq - q0 < kMaxQueriesPerLaunch ? nq - q0 : kMaxQueriesPerLaunch;
        SearchParams p;
        p.vectors = static_cast<const uint8_t*>(h->d.vectors);
        p.n = h->d.n;
        p.row_stride = h->d.row_stride_bytes;
        p.row_bytes = h->row_bytes;
        p.graph = h->d.graph;
        p.degree = h->d.degree;
        p.degree_inv = ((1u << 20) + (uint32_t)h->d.degree - 1) / (uint32_t)h->d.degree;
        p.queries = static_cast<const uint8_t*>(queries);
        p.nq = nq;
        p.q_base = q0;
        p.q_count = cnt;
        p.q_per_xcd = (cnt + 7) / 8;
        p.k = k;
        p.itopk = itopk;
        p.width = width;
        p.max_iters = max_iters;
        p.n_entry = h->d.n_entry;
        p.entry_mode = h->d.entry_mode;
        p.seed = h->d.seed;
        p.route = route;
        p.cluster_offsets = h->d.cluster_offsets;
        p.route_c = h->d.route_c;
        p.n_clusters = h->d.n_clusters;
        p.hash_bits = plan.hash_bits;
        p.window_bits = h->window_bits;
        p.cap = plan.cap;
        p.out_ids = out_ids;
        p.out_dists = static_cast<uint32_t*>(out_dists);
        p.out_counters = out_counters;
        p.order = order;
        const hipError_t e = h->variant->search(p, plan.list_variant, team, (unsigned)(8 * p.q_per_xcd), plan.lds_bytes, stream);
        if (e != hipSuccess) return fail(ANN_EHIP, "ann_search: launch failed: %s", hipGetErrorString(e));
    }
    return ANN_OK;
}

}  // namespace

extern "C" int ann_search_counters(ann_index_t* h, const void* queries, int64_t nq, int k, int itopk, int width,
                                   int max_iters, int32_t* out_ids, void* out_dists, int32_t* out_counters,
                                   void* stream) {
    if (!h || h->magic != kMagic) return fail(ANN_EINVAL, "ann_search: not a live handle");
    Workspace ws(static_cast<hipStream_t>(stream), search_scratch_bytes(h, nq, false));
    return search_impl(h, queries, nq, nullptr, false, k, itopk, width, max_iters, out_ids, out_dists, out_counters, ws);
}

extern "C" int ann_search_routed(ann_index_t* h, const void* queries, int64_t nq, const int32_t* routes, int k,
                                 int itopk, int width, int max_iters, int32_t* out_ids, void* out_dists,
                                 int32_t* out_counters, void* stream) {
    if (!h || h->magic != kMagic) return fail(ANN_EINVAL, "ann_search_routed: not a live handle");
    Workspace ws(static_cast<hipStream_t>(stream), search_scratch_bytes(h, nq, true));
    return search_impl(h, queries, nq, routes, true, k, itopk, width, max_iters, out_ids, out_dists, out_counters, ws);
}

extern "C" int ann_search(ann_index_t* h, const void* queries, int64_t nq, int k, int itopk, int width, int max_iters,
                          int32_t* out_ids, void* out_dists, void* stream) {
    return ann_search_counters(h, queries, nq, k, itopk, width, max_iters, out_ids, out_dists, nullptr, stream);
}

// ---------------------------------------------------------------------------------------------
// ann_search_static: the same search with its temporaries in a device array that is part of the
// library's code object, for callers that cannot allocate.
namespace {

constexpr size_t kStaticScratchBytes = (size_t)ANN_STATIC_SCRATCH_BYTES;
// Host code must not use this name as an address: it is a host-side stand-in.  The device address is
// asked for once per device (static_scratch_of_current_device) and that pointer is what kernels get.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices];  // per device: where that device holds its copy of `scratch`

int static_scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(ANN_EHIP, "ann_search_static: hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(ANN_EUNSUPPORTED, "ann_search_static: device %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(ANN_EHIP, "ann_search_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return ANN_OK;
}

}  // namespace

extern "C" int ann_search_static(ann_index_t* h, const void* queries, int64_t nq, int k, int itopk, int width, int max_iters,
                                 int32_t* out_ids, void* out_dists, void* stream) {
    if (!h || h->magic != kMagic) return fail(ANN_EINVAL, "ann_search_static: not a live handle");
    const size_t need = search_scratch_bytes(h, nq, false);
    if (need > kStaticScratchBytes)
        return fail(ANN_EUNSUPPORTED,
                    "ann_search_static: %lld queries need %zu bytes of temporaries, the static scratch holds %zu; split the batch",
                    (long long)nq, need, kStaticScratchBytes);
    void* base = nullptr;
    if (need > 0) {
        const int rc = static_scratch_of_current_device(&base);
        if (rc != ANN_OK) return rc;
    }
    Workspace ws(static_cast<hipStream_t>(stream), base, need > 0 ? kStaticScratchBytes : 0);
    return search_impl(h, queries, nq, nullptr, false, k, itopk, width, max_iters, out_ids, out_dists, nullptr, ws);
}

extern "C" int ann_gather_vectors(ann_index_t* h, const int32_t* ids, int64_t count, void* out_vectors, void* stream) {
    if (!h || h->magic != kMagic) return fail(ANN_EINVAL, "ann_gather_vectors: not a live handle");
    if (count < 0) return fail(ANN_EINVAL, "ann_gather_vectors: count = %lld", (long long)count);
    if (count == 0) return ANN_OK;
    if (!ids || !out_vectors) return fail(ANN_EINVAL, "ann_gather_vectors: null argument");
    if (!aligned16(out_vectors)) return fail(ANN_EINVAL, "ann_gather_vectors: out_vectors not 16-byte aligned");
    const hipError_t e = launch_gather_rows(static_cast<const uint8_t*>(h->d.vectors), h->d.n, h->d.row_stride_bytes,
                                            h->row_bytes, ids, count, static_cast<uint8_t*>(out_vectors),
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ANN_OK : fail(ANN_EHIP, "ann_gather_vectors: launch failed: %s", hipGetErrorString(e));
}

extern "C" int ann_merge_topk(int key_dtype, const int32_t* ids, const void* keys, int64_t nq, int per_query, int k,
                              int32_t* out_ids, void* out_keys, void* stream) {
    if (key_dtype != ANN_U8 && key_dtype != ANN_F16 && key_dtype != ANN_F32)
        return fail(ANN_EINVAL, "ann_merge_topk: unknown key_dtype %d", key_dtype);
    if (nq < 0) return fail(ANN_EINVAL, "ann_merge_topk: nq = %lld", (long long)nq);
    if (per_query < 1 || per_query > kMaxItopk) return fail(ANN_EUNSUPPORTED, "ann_merge_topk: per_query = %d outside 1..%d", per_query, kMaxItopk);
    if (k < 1 || k > per_query) return fail(ANN_EINVAL, "ann_merge_topk: k = %d outside 1..per_query (%d)", k, per_query);
    if (nq == 0) return ANN_OK;
    if (!ids || !keys || !out_ids || !out_keys) return fail(ANN_EINVAL, "ann_merge_topk: null argument");
    for (int64_t q0 = 0; q0 < nq; q0 += kMaxQueriesPerLaunch) {
        const int64_t cnt = nq - q0 < kMaxQueriesPerLaunch ? nq - q0 : kMaxQueriesPerLaunch;
        const hipError_t e = launch_merge_topk(key_dtype != ANN_U8, ids + q0 * per_query,
                                               static_cast<const uint32_t*>(keys) + q0 * per_query, cnt, per_query, k,
                                               out_ids + q0 * k, static_cast<uint32_t*>(out_keys) + q0 * k,
                                               static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return fail(ANN_EHIP, "ann_merge_topk: launch failed: %s", hipGetErrorString(e));
    }
    return ANN_OK;
}

namespace {

int check_graph_shape(const char* who, int64_t n, int d_in, int d_out) {
    if (n < 1 || n > 0x7fffffffLL) return fail(ANN_EINVAL, "%s: n = %lld outside 1..2^31-1", who, (long long)n);
    if (d_in < 1 || d_out < 1 || d_out > d_in) return fail(ANN_EINVAL, "%s: need 1 <= d_out <= d_in (got %d, %d)", who, d_out, d_in);
    if (d_in > kMaxKnnDegree || d_out > kMaxGraphDegree)
        return fail(ANN_EUNSUPPORTED, "%s: d_in = %d above %d or d_out = %d above %d", who, d_in, kMaxKnnDegree, d_out, kMaxGraphDegree);
    return ANN_OK;
}

}  // namespace

extern "C" int ann_graph_prune(const int32_t* knn, int64_t n, int d_in, int d_out, int32_t* pruned, void* stream) {
    if (const int rc = check_graph_shape("ann_graph_prune", n, d_in, d_out)) return rc;
    if (!knn || !pruned) return fail(ANN_EINVAL, "ann_graph_prune: null argument");
    const hipError_t e = launch_graph_prune(knn, n, d_in, d_out, pruned, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ANN_OK : fail(ANN_EHIP, "ann_graph_prune: launch failed: %s", hipGetErrorString(e));
}

extern "C" int64_t ann_graph_optimize_workspace_bytes(int64_t n, int d_in, int d_out) {
    if (const int rc = check_graph_shape("ann_graph_optimize_workspace_bytes", n, d_in, d_out)) return rc;
    return graph_optimize_scratch_bytes(n, d_out);
}

extern "C" int ann_graph_optimize(const int32_t* knn, int64_t n, int d_in, int d_out, int32_t* out_graph, void* workspace,
                                  int64_t workspace_bytes, void* stream) {
    if (const int rc = check_graph_shape("ann_graph_optimize", n, d_in, d_out)) return rc;
    if (!knn || !out_graph || !workspace) return fail(ANN_EINVAL, "ann_graph_optimize: null argument");
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(ANN_EINVAL, "ann_graph_optimize: workspace not 256-byte aligned");
    const int64_t need = ann_graph_optimize_workspace_bytes(n, d_in, d_out);
    if (workspace_bytes < need)
        return fail(ANN_EINVAL, "ann_graph_optimize: workspace of %lld bytes, %lld needed", (long long)workspace_bytes, (long long)need);
    const hipError_t e = launch_graph_optimize(knn, n, d_in, d_out, out_graph, workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ANN_OK : fail(ANN_EHIP, "ann_graph_optimize: launch failed: %s", hipGetErrorString(e));
}

namespace ann {
__global__ void __launch_bounds__(256) ann_calibration_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                                   int64_t n16) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}
}  // namespace ann

namespace ann {
// Piece p (16 bytes) is piece p % pieces of row p / pieces.  A workgroup takes 8 * 256 consecutive pieces at a
// time (256 whole rows of 128 bytes) and every thread has its eight loads in flight before it uses one.
__global__ void __launch_bounds__(256) ann_calibration_gather_kernel(const uint8_t* __restrict__ vectors, int64_t n,
                                                                     int64_t row_stride, int pieces, uint64_t pieces_inv,
                                                                     const int32_t* __restrict__ ids, int64_t count,
                                                                     uint32_t* sink) {
    __shared__ uint32_t part[256];
    const int64_t total = count * pieces;
    uint32_t acc = 0;
    // the ids of the next chunk are fetched while the rows of the current one are in flight
    // p / pieces as the high half of p * ceil(2^64 / pieces): exact for p < 2^41, pieces <= 128
    auto row_of = [&](int64_t p) -> int64_t { return pieces == 1 ? p : (int64_t)__umul64hi((uint64_t)p, pieces_inv); };
    auto id_of = [&](int64_t p) -> int32_t { return p < total ? ids[row_of(p)] : -1; };
    const int64_t step = (int64_t)gridDim.x * 2048;
    int64_t base = (int64_t)blockIdx.x * 2048;
    int32_t id[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) id[u] = id_of(base + u * 256 + threadIdx.x);
    for (; base < total; base += step) {
        typedef uint32_t word4 __attribute__((ext_vector_type(4)));
        word4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t p = base + u * 256 + threadIdx.x;
            x[u] = word4{0u, 0u, 0u, 0u};
            if (id[u] >= 0 && (int64_t)id[u] < n) {
                const int64_t r = row_of(p);
                // no row is read twice: non-temporal loads keep them from displacing each other in L2
                x[u] = __builtin_nontemporal_load(
                    reinterpret_cast<const word4*>(vectors + (int64_t)id[u] * row_stride + (p - r * pieces) * 16));
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) id[u] = id_of(base + step + u * 256 + threadIdx.x);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] ^= part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) atomicXor(sink, part[0]);
}
}  // namespace ann

extern "C" int ann_calibration_gather(ann_index_t* h, const int32_t* ids, int64_t count, uint32_t* sink, void* stream) {
    if (!h || h->magic != kMagic) return fail(ANN_EINVAL, "ann_calibration_gather: not a live handle");
    if (count < 0) return fail(ANN_EINVAL, "ann_calibration_gather: count = %lld", (long long)count);
    if (count == 0) return ANN_OK;
    if (!ids || !sink) return fail(ANN_EINVAL, "ann_calibration_gather: null argument");
    const int pieces = h->row_bytes / 16;  // at most 128 (2048-byte rows)
    if (count > (int64_t)1 << 33) return fail(ANN_EUNSUPPORTED, "ann_calibration_gather: count above 2^33");
    const uint64_t pieces_inv = pieces == 1 ? 0 : (~0ull) / (uint64_t)pieces + 1;  // ceil(2^64 / pieces)
    const int64_t want = (count * pieces + 2047) / 2048;  // eight pieces per thread
    const unsigned blocks = (unsigned)(want < 1 ? 1 : want > 2048 ? 2048 : want);  // 8 workgroups of 4 wavefronts per compute unit
    hipLaunchKernelGGL(ann::ann_calibration_gather_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint8_t*>(h->d.vectors), h->d.n, h->d.row_stride_bytes, pieces, pieces_inv, ids, count,
                       sink);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? ANN_OK : fail(ANN_EHIP, "ann_calibration_gather: launch failed: %s", hipGetErrorString(e));
}

extern "C" int ann_calibration_copy(void* dst, const void* src, int64_t bytes, void* stream) {
    if (!dst || !src || bytes < 0 || bytes % 16 != 0 || !aligned16(dst) || !aligned16(src))
        return fail(ANN_EINVAL, "ann_calibration_copy: pointers must be non-null and 16-byte aligned, bytes a multiple of 16");
    if (bytes == 0) return ANN_OK;
    hipLaunchKernelGGL(ann::ann_calibration_copy_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint4*>(dst), static_cast<const uint4*>(src), bytes / 16);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? ANN_OK : fail(ANN_EHIP, "ann_calibration_copy: launch failed: %s", hipGetErrorString(e));
}

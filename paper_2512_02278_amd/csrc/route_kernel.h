// Routing: for each query the route_c nearest centroids under (key, cluster index).
// Single-GPU form of Fantasy's stage 1 ("K-means as classifier", Sec. 3.1): it only
// decides in which clusters a query's entry nodes are drawn.
//
// One wavefront per query.  Centroid rows are scored exactly like vector rows
// (same RowOps), each lane group walking its own stride of centroids and keeping
// its route_c best in registers; the groups' lists are then sorted together.
#pragma once

#include "row_ops.h"

namespace ann {

constexpr int kMaxRouteC = 8;

struct RouteParams {
    const uint8_t* centroids;  // n_clusters dense rows of row_bytes
    int32_t n_clusters;
    int32_t row_bytes;
    const uint8_t* queries;
    int64_t nq;
    int32_t route_c;
    int32_t* out;  // nq * route_c
};

template <class Row>
__global__ void __launch_bounds__(64) route_kernel(const RouteParams p) {
    constexpr int PR = (64 / Row::G * kMaxRouteC + 63) / 64;  // registers per lane of the final sort
    __shared__ uint64_t pool[64 * PR];
    const int lane = lane_id();
    const int64_t qi = blockIdx.x;
    if (qi >= p.nq) return;
    Row row;
    row.load_query(p.queries + qi * (int64_t)p.row_bytes, p.row_bytes, lane);
    constexpr int G = Row::G, NCH = Row::NCH, RPS = 64 / G;
    const int grp = lane / G;

    uint64_t best[kMaxRouteC];
#pragma unroll
    for (int i = 0; i < kMaxRouteC; ++i) best[i] = kInfKey;

    for (int c0 = 0; c0 < p.n_clusters; c0 += RPS) {
        const int c = c0 + grp;
        const bool live = c < p.n_clusters;
        u32x4 x[NCH];
        row.load_row(x, row.lane_piece(p.centroids + (int64_t)(live ? c : 0) * p.row_bytes), live);
        const uint32_t okey = row.key(x, lane);
        uint64_t cand = live ? (((uint64_t)okey << 32) | (uint32_t)c) : kInfKey;
        if (__any(cand < best[kMaxRouteC - 1])) {
#pragma unroll
            for (int i = 0; i < kMaxRouteC; ++i) {  // insertion into the ascending list
                const uint64_t lo = cand < best[i] ? cand : best[i];
                cand = cand < best[i] ? best[i] : cand;
                best[i] = lo;
            }
        }
    }
    // RPS groups x kMaxRouteC entries: sort them in one go
#pragma unroll
    for (int r = 0; r < PR; ++r) pool[r * 64 + lane] = kInfKey;
    __syncthreads();
    if (row.lg == 0) {
#pragma unroll
        for (int i = 0; i < kMaxRouteC; ++i) pool[grp * kMaxRouteC + i] = best[i];
    }
    __syncthreads();
    uint64_t v[PR];
#pragma unroll
    for (int r = 0; r < PR; ++r) v[r] = pool[lane * PR + r];
    bitonic_sort<PR>(v, lane);
#pragma unroll
    for (int r = 0; r < PR; ++r)
        if (lane * PR + r < p.route_c) p.out[qi * p.route_c + lane * PR + r] = (int32_t)(uint32_t)v[r];
}

}  // namespace ann

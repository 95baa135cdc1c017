// Cluster-grouped execution order of a batch (schedule.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ann {

// order[0..nq): the query positions sorted by route[q * route_c] (the nearest cluster of q).
// counts: scratch of n_clusters int32.  Both DEVICE; everything is enqueued on `stream`.
hipError_t launch_cluster_order(const int32_t* route, int route_c, int64_t nq, int n_clusters, int32_t* counts,
                                int32_t* order, hipStream_t stream);

}  // namespace ann

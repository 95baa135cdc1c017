// Matrix-core routing for any element type, rows a multiple of 32 bytes (route_mfma.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ann {

// Entries of the per-centroid bias array: n_clusters rounded up to whole pairs of 32-row tiles.
inline int route_mfma_padded(int n_clusters) { return (n_clusters + 63) / 64 * 64; }

// bias (4 bytes per entry: int32 for uint8 data, float otherwise): the per-centroid term of the
// score; padding entries get a value that never wins.
hipError_t launch_route_bias(int dtype, int metric, const uint8_t* centroids, int n_clusters, int row_bytes, void* bias,
                             hipStream_t stream);

// out[q][0..route_c): the nearest clusters of query q under (score, cluster index), ascending.
hipError_t launch_route_mfma(int dtype, int metric, int route_c, const uint8_t* centroids, const void* bias,
                             int n_clusters, int row_bytes, const uint8_t* queries, int64_t nq, int32_t* out,
                             hipStream_t stream);

}  // namespace ann

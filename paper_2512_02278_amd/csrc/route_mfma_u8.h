// Matrix-core routing for uint8 vectors of 128 dimensions (route_mfma_u8.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ann {

// Length of the per-centroid bias array: n_clusters rounded up to whole tiles of 32.
inline int route_mfma_u8_padded(int n_clusters) { return (n_clusters + 31) / 32 * 32; }

// bias[c] = sum (c-128)^2 for L2, -128 * sum (c-128) for the inner product; padding rows get a
// value that never wins.  `bias` has route_mfma_u8_padded(n_clusters) entries.
hipError_t launch_centroid_bias_u8(int metric, const uint8_t* centroids, int n_clusters, int32_t* bias,
                                   hipStream_t stream);

// Slices to cut the centroid range into for a batch of nq queries (1 for large batches).
int route_mfma_u8_slices(int n_clusters, int64_t nq);

// out[q][0..route_c): the nearest clusters of query q under (key, cluster index), ascending.
// slices > 1 needs `partial`: DEVICE scratch of nq * slices * route_c uint64.
hipError_t launch_route_mfma_u8(int metric, int route_c, const uint8_t* centroids, const int32_t* bias, int n_clusters,
                                const uint8_t* queries, int64_t nq, int32_t* out, uint64_t* partial, int slices,
                                hipStream_t stream);

}  // namespace ann

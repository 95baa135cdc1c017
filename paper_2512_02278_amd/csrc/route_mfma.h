// Matrix-core routing for any element type, rows a multiple of 32 bytes (route_mfma.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ann {

// Entries of the per-centroid bias array: n_clusters rounded up to whole tiles of 128 rows.
inline int route_mfma_padded(int n_clusters) { return (n_clusters + 127) / 128 * 128; }

// bias (4 bytes per entry: int32 for uint8 data, float otherwise): the per-centroid term of the
// score; padding entries get a value that never wins.
hipError_t launch_route_bias(int dtype, int metric, const uint8_t* centroids, int n_clusters, int row_bytes, void* bias,
                             hipStream_t stream);

// Small batches leave most CUs idle when every workgroup walks all centroids, so the centroid
// range is cut into slices (grid.y): about 512 workgroups, each slice at least `min_steps`
// steps long, at most 64 slices.  `steps` = steps of the centroid loop (tiles or tile pairs).
inline int route_slices(int steps, int min_steps, int64_t nq) {
    const int64_t groups = (nq + 255) / 256;
    int64_t s = 512 / groups;
    if (s > steps / min_steps) s = steps / min_steps;
    if (s > 64) s = 64;
    return s < 1 ? 1 : (int)s;
}
int route_mfma_slices(int n_clusters, int64_t nq);

// Each slice leaves its best (ordered score << 32 | cluster) words in partial[q][slice][route_c],
// ascending; this picks the route_c smallest per query.
hipError_t launch_route_merge(int route_c, const uint64_t* partial, int slices, int64_t nq, int32_t* out,
                              hipStream_t stream);

// out[q][0..route_c): the nearest clusters of query q under (score, cluster index), ascending.
// slices > 1 needs `partial`: DEVICE scratch of nq * slices * route_c uint64.
hipError_t launch_route_mfma(int dtype, int metric, int route_c, const uint8_t* centroids, const void* bias,
                             int n_clusters, int row_bytes, const uint8_t* queries, int64_t nq, int32_t* out,
                             uint64_t* partial, int slices, hipStream_t stream);

}  // namespace ann

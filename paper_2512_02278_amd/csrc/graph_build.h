// kNN graph -> fixed-degree search graph: detour-count pruning, reverse edges, merge (graph_build.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ann {

constexpr int kMaxKnnDegree = 128;   // d_in
constexpr int kMaxGraphDegree = 64;  // d_out

// pruned[n * d_out] <- for every row of knn[n * d_in], its present ids by ascending (detour count, rank).
hipError_t launch_graph_prune(const int32_t* knn, int64_t n, int d_in, int d_out, int32_t* pruned, hipStream_t stream);

// Bytes of device scratch launch_graph_optimize needs (a multiple of 256).
int64_t graph_optimize_scratch_bytes(int64_t n, int d_out);

// out[n * d_out] <- the pruned rows of knn[n * d_in] with up to d_out/2 reverse edges per row;
// scratch: DEVICE, 256-byte aligned.
hipError_t launch_graph_optimize(const int32_t* knn, int64_t n, int d_in, int d_out, int32_t* out, void* scratch,
                                 hipStream_t stream);

}  // namespace ann

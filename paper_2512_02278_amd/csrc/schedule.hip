// Execution order of a batch: queries grouped by the cluster they were routed to first.
//
// Queries of one cluster walk the same few thousand vector and graph rows.  Run next to each
// other (in time and on one XCD) they find most rows in the L2 / memory-side cache instead of
// HBM - what the paper's dispatch stage does across GPUs by sending a query to the owners of
// its clusters (Sec. 3.1, stage 2), done here inside one GPU.  Only the order of execution
// changes: a query's entries and results depend on its position in the batch, which it keeps.
//
// Counting sort by cluster id: histogram, exclusive scan, scatter.  The order inside a cluster
// is whatever the atomics give; results do not depend on it.
#include <hip/hip_runtime.h>

#include "schedule.h"

namespace ann {

__global__ void __launch_bounds__(256) fill_zero_kernel(int32_t* p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0;
}

// A route id outside [0, n_clusters) names no cluster; such a query is filed under cluster 0, so
// that it still gets a place in the order (it runs, finds no entries and returns padding).
__device__ __forceinline__ int32_t bucket_of(int32_t c, int n_clusters) {
    return (uint32_t)c < (uint32_t)n_clusters ? c : 0;
}

__global__ void __launch_bounds__(256) cluster_histogram_kernel(const int32_t* route, int route_c, int64_t nq,
                                                                int n_clusters, int32_t* counts) {
    for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < nq; q += (int64_t)gridDim.x * 256)
        atomicAdd(&counts[bucket_of(route[q * route_c], n_clusters)], 1);
}

// counts[c] <- number of queries routed to clusters below c (one workgroup, any n).
__global__ void __launch_bounds__(1024) exclusive_scan_kernel(int32_t* counts, int n) {
    __shared__ int32_t part[1024];
    const int t = threadIdx.x;
    const int per = (n + 1023) / 1024;
    const int lo = t * per, hi = min(n, lo + per);
    int32_t sum = 0;
    for (int i = lo; i < hi; ++i) sum += counts[i];
    part[t] = sum;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {  // Hillis-Steele inclusive scan of the per-thread sums
        const int32_t v = t >= d ? part[t - d] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    int32_t run = part[t] - sum;
    for (int i = lo; i < hi; ++i) {
        const int32_t c = counts[i];
        counts[i] = run;
        run += c;
    }
}

__global__ void __launch_bounds__(256) cluster_scatter_kernel(const int32_t* route, int route_c, int64_t nq,
                                                              int n_clusters, int32_t* offsets, int32_t* order) {
    for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < nq; q += (int64_t)gridDim.x * 256)
        order[atomicAdd(&offsets[bucket_of(route[q * route_c], n_clusters)], 1)] = (int32_t)q;
}

hipError_t launch_cluster_order(const int32_t* route, int route_c, int64_t nq, int n_clusters, int32_t* counts,
                                int32_t* order, hipStream_t stream) {
    const unsigned blocks = (unsigned)((nq + 255) / 256 < 4096 ? (nq + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n_clusters + 255) / 256)), dim3(256), 0, stream, counts,
                       (int64_t)n_clusters);
    hipLaunchKernelGGL(cluster_histogram_kernel, dim3(blocks), dim3(256), 0, stream, route, route_c, nq, n_clusters, counts);
    hipLaunchKernelGGL(exclusive_scan_kernel, dim3(1), dim3(1024), 0, stream, counts, n_clusters);
    hipLaunchKernelGGL(cluster_scatter_kernel, dim3(blocks), dim3(256), 0, stream, route, route_c, nq, n_clusters, counts, order);
    return hipGetLastError();
}

}  // namespace ann

// The local half of Fantasy's stage 4 ("Combine vector candidate results", Sec. 3.1): a rank
// returns the vectors of its top-k, not only their ids, and the origin merges the k*c
// candidates it receives for a query into the final top-k.
//
//   gather_rows_kernel   out[i] = vectors[ids[i]] (zeros for id < 0); G lanes move one row in
//                        16-byte pieces, so a 128-byte row is one full-line load and store.
//   merge_topk_kernel    one wavefront per query: the c sorted lists of k (key, id) pairs are
//                        loaded as packed 64-bit words, sorted by the register bitonic network
//                        and the first k written back.  Order: (key, id) ascending, padding
//                        (id < 0) last.
#include <hip/hip_runtime.h>

#include "combine.h"
#include "row_ops.h"

namespace ann {

__global__ void __launch_bounds__(256) gather_rows_kernel(const uint8_t* __restrict__ vectors, int64_t n,
                                                          int64_t row_stride, int row_bytes,
                                                          const int32_t* __restrict__ ids, int64_t count,
                                                          uint8_t* __restrict__ out) {
    const int pieces = row_bytes >> 4;
    const int64_t total = count * pieces;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / pieces;
        const int p = (int)(i - r * pieces);
        const int32_t id = ids[r];
        u32x4 v = {0, 0, 0, 0};
        if (id >= 0 && (int64_t)id < n)
            v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vectors + (int64_t)id * row_stride + p * 16));
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out + r * row_bytes + p * 16));
    }
}

// keys are int32 (uint8 data) or float; both are turned into order-preserving uint32
template <bool FLOAT_KEYS, int R>
__global__ void __launch_bounds__(64) merge_topk_kernel(const int32_t* __restrict__ ids, const uint32_t* __restrict__ keys,
                                                        int64_t nq, int per_query, int k,
                                                        int32_t* __restrict__ out_ids, uint32_t* __restrict__ out_keys) {
    const int lane = lane_id();
    const int64_t q = blockIdx.x;
    if (q >= nq) return;
    uint64_t v[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane * R + r;
        v[r] = kInfKey;
        if (e < per_query) {
            const int32_t id = ids[q * per_query + e];
            const uint32_t raw = keys[q * per_query + e];
            const uint32_t okey = FLOAT_KEYS ? float_to_ordered(__builtin_bit_cast(float, raw)) : (raw ^ 0x80000000u);
            if (id >= 0) v[r] = ((uint64_t)okey << 32) | (uint32_t)id;
        }
    }
    bitonic_sort<R>(v, lane);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane * R + r;
        if (e < k) {
            const bool have = v[r] != kInfKey;
            const uint32_t okey = (uint32_t)(v[r] >> 32);
            out_ids[q * k + e] = have ? (int32_t)(uint32_t)v[r] : -1;
            out_keys[q * k + e] = !have ? (FLOAT_KEYS ? 0x7f800000u : 0x7fffffffu)
                                        : (FLOAT_KEYS ? __builtin_bit_cast(uint32_t, ordered_to_float(okey))
                                                      : (okey ^ 0x80000000u));
        }
    }
}

hipError_t launch_gather_rows(const uint8_t* vectors, int64_t n, int64_t row_stride, int row_bytes, const int32_t* ids,
                              int64_t count, uint8_t* out, hipStream_t stream) {
    const int64_t total = count * (row_bytes >> 4);
    const unsigned blocks = (unsigned)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks), dim3(256), 0, stream, vectors, n, row_stride, row_bytes, ids,
                       count, out);
    return hipGetLastError();
}

template <bool F>
static hipError_t launch_merge_r(int regs, const int32_t* ids, const uint32_t* keys, int64_t nq, int per_query, int k,
                                 int32_t* out_ids, uint32_t* out_keys, hipStream_t stream) {
    const dim3 grid((unsigned)nq), block(64);
    switch (regs) {
        case 1: hipLaunchKernelGGL((merge_topk_kernel<F, 1>), grid, block, 0, stream, ids, keys, nq, per_query, k, out_ids, out_keys); break;
        case 2: hipLaunchKernelGGL((merge_topk_kernel<F, 2>), grid, block, 0, stream, ids, keys, nq, per_query, k, out_ids, out_keys); break;
        case 4: hipLaunchKernelGGL((merge_topk_kernel<F, 4>), grid, block, 0, stream, ids, keys, nq, per_query, k, out_ids, out_keys); break;
        case 8: hipLaunchKernelGGL((merge_topk_kernel<F, 8>), grid, block, 0, stream, ids, keys, nq, per_query, k, out_ids, out_keys); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_merge_topk(bool float_keys, const int32_t* ids, const void* keys, int64_t nq, int per_query, int k,
                             int32_t* out_ids, void* out_keys, hipStream_t stream) {
    int regs = 1;
    while (64 * regs < per_query) regs *= 2;
    return float_keys ? launch_merge_r<true>(regs, ids, static_cast<const uint32_t*>(keys), nq, per_query, k, out_ids,
                                             static_cast<uint32_t*>(out_keys), stream)
                      : launch_merge_r<false>(regs, ids, static_cast<const uint32_t*>(keys), nq, per_query, k, out_ids,
                                              static_cast<uint32_t*>(out_keys), stream);
}

}  // namespace ann

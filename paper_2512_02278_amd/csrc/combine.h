// Result-vector gather and k*c-way merge (combine.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ann {

hipError_t launch_gather_rows(const uint8_t* vectors, int64_t n, int64_t row_stride, int row_bytes, const int32_t* ids,
                              int64_t count, uint8_t* out, hipStream_t stream);

// per query `per_query` (<= 512) candidates; keys int32 or float (4 bytes each)
hipError_t launch_merge_topk(bool float_keys, const int32_t* ids, const void* keys, int64_t nq, int per_query, int k,
                             int32_t* out_ids, void* out_keys, hipStream_t stream);

}  // namespace ann

// Which kernel variants are built, and how the host reaches them.
//
// A row variant fixes element type, metric, lanes per row (G) and 16-byte pieces per
// lane (NCH); it serves every row of at most G*NCH*16 bytes.  A list variant fixes
// the registers per lane of the candidate list (LPL: itopk <= 64*LPL) and of one
// round's neighbour ids (CPL: width*degree and n_entry <= 64*CPL).
#pragma once

#include <hip/hip_runtime.h>

#include "beam_search_kernel.h"
#include "route_kernel.h"

namespace ann {

// X(dtype, metric, G, NCH)
#define ANN_ROW_VARIANTS(X)                                                  \
    X(kU8, kL2, 8, 1) X(kU8, kIP, 8, 1) X(kU8, kL2, 8, 2) X(kU8, kIP, 8, 2) X(kU8, kL2, 4, 2) X(kU8, kIP, 4, 2) \
    X(kF16, kL2, 8, 2) X(kF16, kIP, 8, 2) X(kF16, kL2, 32, 3) X(kF16, kIP, 32, 3) \
    X(kF32, kL2, 8, 3) X(kF32, kIP, 8, 3) X(kF32, kL2, 32, 4) X(kF32, kIP, 32, 4)

// List variants (LPL, CPL); a request is served by the first one that is large enough.
constexpr int kListVariants[][2] = {{1, 1}, {2, 2}, {3, 2}, {4, 2}, {4, 4}, {4, 8}, {8, 8}};
constexpr int kNumListVariants = 7;

template <int DT, int METRIC, int G, int NCH>
hipError_t launch_search(const SearchParams& p, int list_variant, unsigned grid, size_t lds_bytes, hipStream_t stream);

template <int DT, int METRIC, int G, int NCH>
hipError_t launch_route(const RouteParams& p, hipStream_t stream);

#define ANN_DEFINE_ROW_VARIANT(DT, METRIC, G, NCH)                                                              \
    template <>                                                                                                 \
    hipError_t launch_search<DT, METRIC, G, NCH>(const SearchParams& p, int list_variant, unsigned grid,        \
                                                 size_t lds_bytes, hipStream_t stream) {                        \
        using Row = RowOps<DT, METRIC, G, NCH>;                                                                 \
        switch (list_variant) {                                                                                 \
            case 0: hipLaunchKernelGGL((beam_search_kernel<Row, 1, 1>), dim3(grid), dim3(64), lds_bytes, stream, p); break; \
            case 1: hipLaunchKernelGGL((beam_search_kernel<Row, 2, 2>), dim3(grid), dim3(64), lds_bytes, stream, p); break; \
            case 2: hipLaunchKernelGGL((beam_search_kernel<Row, 3, 2>), dim3(grid), dim3(64), lds_bytes, stream, p); break; \
            case 3: hipLaunchKernelGGL((beam_search_kernel<Row, 4, 2>), dim3(grid), dim3(64), lds_bytes, stream, p); break; \
            case 4: hipLaunchKernelGGL((beam_search_kernel<Row, 4, 4>), dim3(grid), dim3(64), lds_bytes, stream, p); break; \
            case 5: hipLaunchKernelGGL((beam_search_kernel<Row, 4, 8>), dim3(grid), dim3(64), lds_bytes, stream, p); break; \
            case 6: hipLaunchKernelGGL((beam_search_kernel<Row, 8, 8>), dim3(grid), dim3(64), lds_bytes, stream, p); break; \
            default: return hipErrorInvalidValue;                                                               \
        }                                                                                                       \
        return hipGetLastError();                                                                               \
    }                                                                                                           \
    template <>                                                                                                 \
    hipError_t launch_route<DT, METRIC, G, NCH>(const RouteParams& p, hipStream_t stream) {                     \
        using Row = RowOps<DT, METRIC, G, NCH>;                                                                 \
        hipLaunchKernelGGL((route_kernel<Row>), dim3((unsigned)p.nq), dim3(64), 0, stream, p);                  \
        return hipGetLastError();                                                                               \
    }

}  // namespace ann

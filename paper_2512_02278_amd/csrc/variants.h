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
    X(kF32, kL2, 8, 3) X(kF32, kIP, 8, 3) X(kF32, kL2, 32, 4) X(kF32, kIP, 32, 4)                               \
    X(kU8, kL2, 32, 3) X(kU8, kIP, 32, 3) X(kF16, kL2, 32, 6) X(kF16, kIP, 32, 6) X(kF32, kL2, 32, 12) X(kF32, kIP, 32, 12)

// List variants (LPL, CPL); a request is served by the first one that is large enough.
constexpr int kListVariants[][2] = {{1, 1}, {2, 2}, {3, 2}, {4, 2}, {4, 4}, {4, 8}, {8, 8}};
constexpr int kNumListVariants = 7;

// Wavefronts per query a launch may use (see BeamSearch).
constexpr int kTeamSizes[] = {1, 2, 4};
constexpr int kNumTeamSizes = 3;

template <int DT, int METRIC, int G, int NCH>
hipError_t launch_search(const SearchParams& p, int list_variant, int team, unsigned grid, size_t lds_bytes, hipStream_t stream);

template <int DT, int METRIC, int G, int NCH>
hipError_t launch_route(const RouteParams& p, hipStream_t stream);

#define ANN_LAUNCH_LIST(LPL, CPL)                                                                                         \
    switch (team) {                                                                                                       \
        case 1: hipLaunchKernelGGL((beam_search_kernel<Row, LPL, CPL, 1>), dim3(grid), dim3(64), lds_bytes, stream, p); break;  \
        case 2: hipLaunchKernelGGL((beam_search_kernel<Row, LPL, CPL, 2>), dim3(grid), dim3(128), lds_bytes, stream, p); break; \
        case 4: hipLaunchKernelGGL((beam_search_kernel<Row, LPL, CPL, 4>), dim3(grid), dim3(256), lds_bytes, stream, p); break; \
        default: return hipErrorInvalidValue;                                                                             \
    }                                                                                                                     \
    break;

#define ANN_DEFINE_ROW_VARIANT(DT, METRIC, G, NCH)                                                              \
    template <>                                                                                                 \
    hipError_t launch_search<DT, METRIC, G, NCH>(const SearchParams& p, int list_variant, int team, unsigned grid, \
                                                 size_t lds_bytes, hipStream_t stream) {                        \
        using Row = RowOps<DT, METRIC, G, NCH>;                                                                 \
        switch (list_variant) {                                                                                 \
            case 0: ANN_LAUNCH_LIST(1, 1)                                                                       \
            case 1: ANN_LAUNCH_LIST(2, 2)                                                                       \
            case 2: ANN_LAUNCH_LIST(3, 2)                                                                       \
            case 3: ANN_LAUNCH_LIST(4, 2)                                                                       \
            case 4: ANN_LAUNCH_LIST(4, 4)                                                                       \
            case 5: ANN_LAUNCH_LIST(4, 8)                                                                       \
            case 6: ANN_LAUNCH_LIST(8, 8)                                                                       \
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

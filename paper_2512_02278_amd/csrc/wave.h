// Wavefront-level building blocks for gfx950 (wave64): lane exchange, group
// reductions and bitonic networks over 64-bit keys held in registers.
//
// Element layout ("blocked"): a wavefront holds 64*R keys, key number e lives in
// lane e / R, register e % R.  Small exchange distances (the most frequent ones in
// a bitonic network) then stay inside a lane and cost no cross-lane traffic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ann {

constexpr uint64_t kInfKey = ~0ull;  // sorts last; its low bit marks it "expanded"

__device__ __forceinline__ int lane_id() {
    return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Number of set bits of `mask` below the calling lane.
__device__ __forceinline__ int rank_below(uint64_t mask) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Value of `v` held by lane (lane ^ mask).
__device__ __forceinline__ uint32_t xor_lane(uint32_t v, int lane, int mask) {
    return (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, (int)v);
}
__device__ __forceinline__ uint64_t xor_lane64(uint64_t v, int lane, int mask) {
    uint32_t lo = xor_lane((uint32_t)v, lane, mask);
    uint32_t hi = xor_lane((uint32_t)(v >> 32), lane, mask);
    return ((uint64_t)hi << 32) | lo;
}

// Butterfly sum over groups of G consecutive lanes; every lane of a group ends up
// with the same value, and the order of additions is the same for every group.
template <int G, class T>
__device__ __forceinline__ T group_sum(T v, int lane) {
#pragma unroll
    for (int m = 1; m < G; m <<= 1) {
        uint32_t o = xor_lane(__builtin_bit_cast(uint32_t, v), lane, m);
        v = v + __builtin_bit_cast(T, o);
    }
    return v;
}

__device__ __forceinline__ void order2(uint64_t& lo, uint64_t& hi) {
    uint64_t a = lo, b = hi;
    lo = a < b ? a : b;
    hi = a < b ? b : a;
}

// Keep the smaller key if `keep_min`, else the larger.
__device__ __forceinline__ uint64_t pick(uint64_t mine, uint64_t other, bool keep_min) {
    return ((other < mine) == keep_min) ? other : mine;
}

// Half-cleaner stages at distances J, J/2, ..., 1 over 64*R blocked keys: sorts
// every 2*J-aligned bitonic run of length 2*J.
template <int R, int J>
__device__ __forceinline__ void bitonic_clean(uint64_t (&v)[R], int lane) {
    if constexpr (J >= 1) {
        if constexpr (J >= R) {
            constexpr int lm = J / R;
            const bool low = (lane & lm) == 0;
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = pick(v[r], xor_lane64(v[r], lane, lm), low);
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r)
                if ((r & J) == 0) order2(v[r], v[r | J]);
        }
        bitonic_clean<R, J / 2>(v, lane);
    }
}

// Merge step for runs of length K/2 into runs of length K: one mirror stage
// (e against e ^ (K-1)), then half-cleaners; recurses up to the full width.
template <int R, int K>
__device__ __forceinline__ void bitonic_sort_from(uint64_t (&v)[R], int lane) {
    if constexpr (K <= 64 * R) {
        if constexpr (K <= R) {
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (r < (r ^ (K - 1))) order2(v[r], v[r ^ (K - 1)]);
        } else {
            constexpr int lm = K / R - 1;  // lane mirror inside the K-run
            const bool low = (lane & (K / (2 * R))) == 0;
            uint64_t o[R];
#pragma unroll
            for (int r = 0; r < R; ++r) o[r] = xor_lane64(v[R - 1 - r], lane, lm);
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = pick(v[r], o[r], low);
        }
        bitonic_clean<R, K / 4>(v, lane);
        bitonic_sort_from<R, K * 2>(v, lane);
    }
}

// Full ascending sort of 64*R blocked keys.
template <int R>
__device__ __forceinline__ void bitonic_sort(uint64_t (&v)[R], int lane) {
    bitonic_sort_from<R, 2>(v, lane);
}

// Sorts 64*R blocked keys that form one bitonic run.
template <int R>
__device__ __forceinline__ void bitonic_merge(uint64_t (&v)[R], int lane) {
    bitonic_clean<R, 32 * R>(v, lane);
}

}  // namespace ann

// Wavefront-level building blocks for gfx950 (wave64): lane exchange, group
// reductions and bitonic networks over 64-bit keys held in registers.
//
// Two element layouts for 64*R keys held by a wavefront:
//   "blocked": key number e lives in lane e / R, register e % R.  The small exchange distances
//              of a full sort (the most frequent ones) stay inside a lane.  R a power of two.
//   "striped": key number e lives in register e / 64, lane e % 64.  Any R; a register is a
//              contiguous run of 64 keys, so consecutive lanes hold consecutive keys (LDS
//              accesses by key number are conflict-free, the first k keys are the first lanes).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ann {

constexpr uint64_t kInfKey = ~0ull;  // sorts last; its low bit marks it "expanded"

__device__ __forceinline__ int lane_id() {
    return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// base + number of set bits of `mask` below the calling lane (the count instructions add to an operand).
__device__ __forceinline__ int rank_below(uint64_t mask, int base = 0) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, (uint32_t)base));
}

// Value of `v` held by lane (lane ^ MASK), MASK a compile-time constant: DPP moves inside a
// row of 16 lanes (quad permutes, half-row and row mirrors, rotate by 8), ds_bpermute across
// rows.  The search loop is bound by vector-ALU issue, and the LDS crossbar takes the
// cross-row moves off the vector ALU.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v) {
    // every lane has a source inside its row for the controls used here, so the "old" value is dead
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
template <int MASK>
__device__ __forceinline__ uint32_t xor_lane(uint32_t v, int lane) {
    static_assert(MASK >= 0 && MASK < 64, "lane mask");
    if constexpr ((MASK & 48) != 0) {
        return (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ MASK) << 2, (int)v);
    } else {
        constexpr int low = MASK & 15;
        if constexpr (low == 1) v = dpp_move<0xB1>(v);        // quad_perm [1,0,3,2]
        else if constexpr (low == 2) v = dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
        else if constexpr (low == 3) v = dpp_move<0x1B>(v);   // quad_perm [3,2,1,0]
        else if constexpr (low == 4) v = dpp_move<0x1B>(dpp_move<0x141>(v));  // (i ^ 7) ^ 3
        else if constexpr (low == 7) v = dpp_move<0x141>(v);  // row_half_mirror
        else if constexpr (low == 8) v = dpp_move<0x128>(v);  // row_ror:8
        else if constexpr (low == 15) v = dpp_move<0x140>(v); // row_mirror
        else static_assert(low == 0, "unsupported lane mask");
        return v;
    }
}
template <int MASK>
__device__ __forceinline__ uint64_t xor_lane64(uint64_t v, int lane) {
    uint32_t lo = xor_lane<MASK>((uint32_t)v, lane);
    uint32_t hi = xor_lane<MASK>((uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

// Butterfly sum over groups of G consecutive lanes; every lane of a group ends up
// with the same value, and the order of additions is the same for every group.
template <int MASK>
__device__ __forceinline__ uint32_t xor_lane_dpp(uint32_t v, int lane) {
    constexpr int low = MASK & 15;
    if constexpr (low == 1) v = dpp_move<0xB1>(v);
    else if constexpr (low == 2) v = dpp_move<0x4E>(v);
    else if constexpr (low == 4) v = dpp_move<0x1B>(dpp_move<0x141>(v));
    else if constexpr (low == 8) v = dpp_move<0x128>(v);
    else static_assert(low == 0, "unsupported lane mask");
    if constexpr ((MASK & 48) != 0) v = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ (MASK & 48)) << 2, (int)v);
    return v;
}
template <int G, int M = 1, class T>
__device__ __forceinline__ T group_sum(T v, int lane) {
    if constexpr (M < G) {
        const uint32_t o = xor_lane_dpp<M>(__builtin_bit_cast(uint32_t, v), lane);
        return group_sum<G, M * 2>(v + __builtin_bit_cast(T, o), lane);
    } else {
        return v;
    }
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
            for (int r = 0; r < R; ++r) v[r] = pick(v[r], xor_lane64<lm>(v[r], lane), low);
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
template <int R, int K, int KMAX>
__device__ __forceinline__ void bitonic_sort_from(uint64_t (&v)[R], int lane) {
    if constexpr (K <= KMAX) {
        if constexpr (K <= R) {
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (r < (r ^ (K - 1))) order2(v[r], v[r ^ (K - 1)]);
        } else {
            constexpr int lm = K / R - 1;  // lane mirror inside the K-run
            const bool low = (lane & (K / (2 * R))) == 0;
            uint64_t o[R];
#pragma unroll
            for (int r = 0; r < R; ++r) o[r] = xor_lane64<lm>(v[R - 1 - r], lane);
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = pick(v[r], o[r], low);
        }
        bitonic_clean<R, K / 4>(v, lane);
        bitonic_sort_from<R, K * 2, KMAX>(v, lane);
    }
}

// Full ascending sort of 64*R blocked keys.
template <int R>
__device__ __forceinline__ void bitonic_sort(uint64_t (&v)[R], int lane) {
    bitonic_sort_from<R, 2, 64 * R>(v, lane);
}

// Sorts every aligned run of KMAX keys on its own.  With real keys only among the first
// KMAX and the empty key everywhere else, that already sorts all 64*R.
template <int R, int KMAX>
__device__ __forceinline__ void bitonic_sort_runs(uint64_t (&v)[R], int lane) {
    bitonic_sort_from<R, 2, KMAX>(v, lane);
}

// Sorts 64*R blocked keys that form one bitonic run.
template <int R>
__device__ __forceinline__ void bitonic_merge(uint64_t (&v)[R], int lane) {
    bitonic_clean<R, 32 * R>(v, lane);
}

// Striped layout: sorts 64*R keys that form one bitonic run that first rises and then falls (what
// "element e of an ascending run against element 64*R-1-e of another" leaves behind).  R need not be
// a power of two: the run is thought of as the upper part of P >= R registers (P a power of two) whose
// lower P - R registers hold keys below everything - still one rising-then-falling run, and a
// compare-exchange with such a register changes nothing, so it is left out.  First the stages between
// registers (distances P/2 .. 1 registers), then the six lane stages inside every register.
template <int R, int P, int D>
__device__ __forceinline__ void striped_register_stages(uint64_t (&v)[R]) {
    if constexpr (D >= 1) {
        constexpr int pad = P - R;
#pragma unroll
        for (int i = 0; i < P; ++i)
            if ((i & D) == 0 && i >= pad) order2(v[i - pad], v[i + D - pad]);
        striped_register_stages<R, P, D / 2>(v);
    }
}
template <int R>
__device__ __forceinline__ void striped_merge(uint64_t (&v)[R], int lane) {
    constexpr int P = R <= 1 ? 1 : R <= 2 ? 2 : R <= 4 ? 4 : 8;
    static_assert(R >= 1 && R <= 8, "registers per lane");
    striped_register_stages<R, P, P / 2>(v);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        uint64_t one[1] = {v[r]};
        bitonic_clean<1, 32>(one, lane);
        v[r] = one[0];
    }
}

}  // namespace ann

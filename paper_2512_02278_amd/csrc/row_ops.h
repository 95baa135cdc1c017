// Distance of one query to gathered vector rows, for each element type and metric.
//
// A row is read by a group of G consecutive lanes; lane lg of the group reads the
// 16-byte pieces number c*G + lg (c = 0..NCH-1), so one load instruction of a group
// covers G*16 contiguous bytes (a whole 128-byte line for G = 8).  The query is held
// in registers in the same arrangement.  Pieces beyond the row's length are neither
// loaded nor counted.  Partial sums are combined by a fixed butterfly over the
// group, so a (query, row) pair always gives the same bits.
//
// Keys are returned as uint32 that compare like the key itself: the int32 value
// for uint8 data (never negative for L2; offset by 2^31 for inner product), and the
// usual order-preserving transform of the IEEE bits for float keys.
#pragma once

#include "wave.h"

// Row and graph loads are ordinary cached loads: queries of one cluster run next to each other and
// re-read each other's rows from L2 / the memory-side cache (a non-temporal hint costs a quarter of
// the throughput with the cluster-grouped order and a tenth even without it).

namespace ann {

enum { kU8 = 0, kF16 = 1, kF32 = 2 };
enum { kL2 = 0, kIP = 1 };

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t float_to_ordered(float f) {
    f = f + 0.0f;  // -0 becomes +0, so equal keys have equal bits
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_float(uint32_t u) {
    u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
    return __builtin_bit_cast(float, u);
}

template <int DT, int METRIC, int G_, int NCH_>
struct RowOps {
    static constexpr int G = G_;
    static constexpr int NCH = NCH_;
    static constexpr int kDtype = DT;
    static constexpr int kMetric = METRIC;
    static constexpr int kRowsPerStep = 64 / G;

    u32x4 q[NCH];        // this lane's pieces of the query
    uint32_t piece_ok;   // bit c set: piece c of this lane lies inside the row
    bool full;           // the row fills every piece of every lane (uniform)
    int minus_two;       // -2 in a scalar register (uint8 L2 keys)
    int32_t qq;          // uint8 L2 only: sum of squares of the query
    int lg;              // lane index inside its group

    __device__ __forceinline__ void load_query(const uint8_t* qrow, int row_bytes, int lane) {
        lg = lane & (G - 1);
        piece_ok = 0;
        full = row_bytes >= G * NCH * 16;
        minus_two = -2;
        asm volatile("" : "+s"(minus_two));
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int off = (c * G + lg) * 16;
            const bool ok = off < row_bytes;
            q[c] = ok ? *reinterpret_cast<const u32x4*>(qrow + off) : u32x4{0, 0, 0, 0};
            piece_ok |= ok ? (1u << c) : 0u;
        }
        qq = 0;
        if constexpr (DT == kU8 && METRIC == kL2) {
            uint32_t s = 0;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                s = __builtin_amdgcn_udot4(q[c].x, q[c].x, s, false);
                s = __builtin_amdgcn_udot4(q[c].y, q[c].y, s, false);
                s = __builtin_amdgcn_udot4(q[c].z, q[c].z, s, false);
                s = __builtin_amdgcn_udot4(q[c].w, q[c].w, s, false);
            }
            qq = group_sum<G>((int32_t)s, lane);
        }
    }

    // This lane's first piece of the row that starts at `row`.
    __device__ __forceinline__ const uint8_t* lane_piece(const uint8_t* row) const { return row + lg * 16; }

    // Issues this lane's loads of the row whose lane_piece() is `piece` (rows the caller does
    // not want pass live = false and read nothing).
    __device__ __forceinline__ void load_row(u32x4 (&x)[NCH], const uint8_t* piece, bool live) const {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const bool ok = live && ((piece_ok >> c) & 1u);
            x[c] = ok ? *reinterpret_cast<const u32x4*>(piece + c * G * 16) : u32x4{0, 0, 0, 0};
        }
    }

    // For rows that fill every piece of every lane (`full`): a row buffer whose registers hold nothing yet, and the
    // load of a wanted row into it.  No instruction is spent on clearing: every piece of a wanted row is loaded
    // before it is used, and the key of a row passed with live = false is ignored, whatever it is computed from.
    __device__ __forceinline__ void blank_row(u32x4 (&x)[NCH]) const {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            uint32_t a, b, d, e;
            asm volatile("" : "=v"(a), "=v"(b), "=v"(d), "=v"(e));  // defines the registers, emits nothing
            x[c] = u32x4{a, b, d, e};
        }
    }
    __device__ __forceinline__ void load_full_row(u32x4 (&x)[NCH], const uint8_t* piece, bool live) const {
        if (live) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) x[c] = *reinterpret_cast<const u32x4*>(piece + c * G * 16);
        }
    }

    // The same for a buffer that is reused from row to row: a piece this lane does not load keeps what
    // x held.  The caller zeroes x once (pieces beyond the row's end then stay zero for good) and
    // ignores the key of a row it passed with live = false.
    __device__ __forceinline__ void reload_row(u32x4 (&x)[NCH], const uint8_t* piece, bool live) const {
#pragma unroll
        for (int c = 0; c < NCH; ++c)
            if (live && ((piece_ok >> c) & 1u)) x[c] = *reinterpret_cast<const u32x4*>(piece + c * G * 16);
    }

    // Ordered key of the row whose pieces are in x; valid in every lane of the group.
    __device__ __forceinline__ uint32_t key(const u32x4 (&x)[NCH], int lane) const {
        if constexpr (DT == kU8) {
            uint32_t qx = 0, xx = 0;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const uint32_t xs[4] = {x[c].x, x[c].y, x[c].z, x[c].w};
                const uint32_t qs[4] = {q[c].x, q[c].y, q[c].z, q[c].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    qx = __builtin_amdgcn_udot4(qs[i], xs[i], qx, false);
                    if constexpr (METRIC == kL2) xx = __builtin_amdgcn_udot4(xs[i], xs[i], xx, false);
                }
            }
            if constexpr (METRIC == kL2) {
                // sum (q-x)^2 = qq + xx - 2 qx, exact in int32; a lane's q.x is below 2^23 (at most 48 bytes of
                // 255 * 255 each), so the 24-bit multiply-add does it in one instruction
                static_assert(NCH <= 8, "a lane's share of q.x must fit 24 bits");
                // (the factor comes from a register the optimiser cannot see through: with the literal it turns the
                // 24-bit multiply into two shifts and a subtraction)
                int32_t part = (int32_t)xx + __mul24((int)qx, minus_two);
                return (uint32_t)(qq + group_sum<G>(part, lane));
            } else {
                int32_t s = group_sum<G>((int32_t)qx, lane);
                return (uint32_t)(-s) ^ 0x80000000u;  // signed order -> unsigned order
            }
        } else if constexpr (DT == kF32) {
            float acc = 0.0f;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const uint32_t xs[4] = {x[c].x, x[c].y, x[c].z, x[c].w};
                const uint32_t qs[4] = {q[c].x, q[c].y, q[c].z, q[c].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a = __builtin_bit_cast(float, qs[i]), b = __builtin_bit_cast(float, xs[i]);
                    if constexpr (METRIC == kL2) {
                        const float d = a - b;
                        acc = __builtin_fmaf(d, d, acc);
                    } else {
                        acc = __builtin_fmaf(a, b, acc);
                    }
                }
            }
            acc = group_sum<G>(acc, lane);
            return float_to_ordered(METRIC == kL2 ? acc : -acc);
        } else {
            float acc = 0.0f;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const uint32_t xs[4] = {x[c].x, x[c].y, x[c].z, x[c].w};
                const uint32_t qs[4] = {q[c].x, q[c].y, q[c].z, q[c].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const half2_t a = __builtin_bit_cast(half2_t, qs[i]), b = __builtin_bit_cast(half2_t, xs[i]);
                    if constexpr (METRIC == kL2) {
                        const float d0 = (float)a.x - (float)b.x, d1 = (float)a.y - (float)b.y;
                        acc = __builtin_fmaf(d0, d0, acc);
                        acc = __builtin_fmaf(d1, d1, acc);
                    } else {
                        acc = __builtin_amdgcn_fdot2(a, b, acc, false);  // fp16 products, fp32 accumulate
                    }
                }
            }
            acc = group_sum<G>(acc, lane);
            return float_to_ordered(METRIC == kL2 ? acc : -acc);
        }
    }

    // Ordered key -> the value written to out_dists (bit pattern of int32 or float).
    static __device__ __forceinline__ uint32_t key_to_output(uint32_t okey) {
        if constexpr (DT == kU8) {
            return METRIC == kL2 ? okey : (okey ^ 0x80000000u);
        } else {
            return __builtin_bit_cast(uint32_t, ordered_to_float(okey));
        }
    }
    static __device__ __forceinline__ uint32_t pad_output() {
        if constexpr (DT == kU8) return 0x7fffffffu;  // INT32_MAX
        return 0x7f800000u;                            // +inf
    }
};

}  // namespace ann

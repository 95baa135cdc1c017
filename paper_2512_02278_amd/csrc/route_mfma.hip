// Routing on the matrix cores for any element type and any row length that is a multiple of
// 32 bytes: nearest route_c centroids per query under (score, cluster index).
//
// Stage 1 of Fantasy (Sec. 3.2, "Local K-means Assignment") is a dense contraction,
// Q (b x d) against C (d x C), followed by a per-query selection.  The score that is ranked is
// the key without its per-query constant:
//     L2:  |c|^2 - 2 q.c          IP:  -q.c
// uint8 operands are shifted by -128 into int8 (exact int32 sums; for the inner product the shift
// adds -128*sum(c') per centroid, which goes into the bias); fp16 / fp32 operands accumulate in
// fp32 on v_mfma_f32_32x32x16_f16 / v_mfma_f32_32x32x2_f32.
//
// A wavefront owns 64 queries (two operand sets of 32) and walks the centroids 64 at a time
// (two sets of 32): four 32x32 accumulator tiles, and per 16-byte piece of the rows two loads
// of each operand feed four matrix instructions.  Operands stream from L1/L2; nothing is staged
// in LDS, and the rows can be of any length.  In a 32x32 result a lane holds 16 centroids of one
// query, so a query's best list lives in two lanes and is merged once at the end.  Rows are
// visited in ascending cluster order, so a strict "<" keeps the lower index among equal scores.
#include <hip/hip_runtime.h>

#include "route_mfma.h"

namespace ann {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

template <int DT>
struct Mma;

template <>
struct Mma<0> {  // uint8 -> int8, int32 sums
    typedef v16i acc_t;
    typedef int32_t score_t;
    static __device__ __forceinline__ v4i prep(v4i x) { return x ^ (int)0x80808080; }
    static __device__ __forceinline__ void mma(acc_t& c, v4i a, v4i b) {
        c = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ score_t score(score_t bias, int32_t dot, bool l2) {
        return bias - (l2 ? 2 : 1) * dot;
    }
    static __device__ __forceinline__ uint32_t ordered(score_t s) { return (uint32_t)s ^ 0x80000000u; }
    static constexpr score_t kWorst = 0x7fffffff;
};
template <>
struct Mma<1> {  // fp16, fp32 sums
    typedef v16f acc_t;
    typedef float score_t;
    static __device__ __forceinline__ v4i prep(v4i x) { return x; }
    static __device__ __forceinline__ void mma(acc_t& c, v4i a, v4i b) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ score_t score(score_t bias, float dot, bool l2) {
        return l2 ? __builtin_fmaf(-2.0f, dot, bias) : bias - dot;  // bias is 0 for real rows of an IP index
    }
    static __device__ __forceinline__ uint32_t ordered(score_t s) {
        s = s + 0.0f;
        const uint32_t u = __builtin_bit_cast(uint32_t, s);
        return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    }
    static constexpr score_t kWorst = __builtin_inff();
};
template <>
struct Mma<2> : Mma<1> {  // fp32: four K=2 instructions per 16-byte piece
    static __device__ __forceinline__ void mma(acc_t& c, v4i a, v4i b) {
        const v4f x = __builtin_bit_cast(v4f, a), y = __builtin_bit_cast(v4f, b);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.x, y.x, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.y, y.y, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.z, y.z, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.w, y.w, c, 0, 0, 0);
    }
};

// bias[c]: the per-centroid term of the score; rows beyond n_clusters (padding up to a multiple
// of 64) get a value that never wins.
template <int DT, int METRIC>
__global__ void __launch_bounds__(256) route_bias_kernel(const uint8_t* centroids, int n_clusters, int padded,
                                                         int row_bytes, void* bias_out) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= padded) return;
    const uint8_t* row = centroids + (int64_t)c * row_bytes;
    if constexpr (DT == 0) {
        int32_t* bias = static_cast<int32_t*>(bias_out);
        if (c >= n_clusters) {
            bias[c] = 0x3fffffff;
            return;
        }
        int32_t acc = 0;
        for (int i = 0; i < row_bytes / 4; ++i) {
            const uint32_t w = reinterpret_cast<const uint32_t*>(row)[i] ^ 0x80808080u;
            acc = METRIC == 0 ? __builtin_amdgcn_sdot4((int)w, (int)w, acc, false)
                              : __builtin_amdgcn_sdot4((int)w, 0x01010101, acc, false);
        }
        bias[c] = METRIC == 0 ? acc : -128 * acc;
    } else {
        float* bias = static_cast<float*>(bias_out);
        if (c >= n_clusters) {
            bias[c] = 1.0e38f;
            return;
        }
        float acc = 0.0f;
        if (METRIC == 0) {
            const int n = row_bytes / (DT == 1 ? 2 : 4);
            for (int i = 0; i < n; ++i) {
                const float v = DT == 1 ? (float)reinterpret_cast<const _Float16*>(row)[i]
                                        : reinterpret_cast<const float*>(row)[i];
                acc = __builtin_fmaf(v, v, acc);
            }
        }
        bias[c] = acc;
    }
}

template <int DT, int METRIC, int RC>
__global__ void __launch_bounds__(256) route_mfma_kernel(const uint8_t* __restrict__ centroids,
                                                         const void* __restrict__ bias_in, int n_clusters,
                                                         int row_bytes, const uint8_t* __restrict__ queries,
                                                         int64_t nq, int32_t* __restrict__ out,
                                                         uint64_t* __restrict__ partial, int pairs_per_slice) {
    // blockIdx.y = slice of the centroid tile pairs this workgroup walks; with several slices the
    // best words of a slice go to partial[q][slice][RC] and route_merge_kernel finishes the job
    typedef Mma<DT> M;
    typedef typename M::acc_t acc_t;
    typedef typename M::score_t score_t;
    __shared__ uint64_t pool[4][64][2][RC];
    const score_t* bias = static_cast<const score_t*>(bias_in);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int64_t q0 = ((int64_t)blockIdx.x * 4 + wave) * 64;
    if (q0 >= nq) return;  // whole wavefront; no block-wide barrier is used below

    const uint8_t* qrow[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        int64_t q = q0 + s * 32 + col;
        if (q >= nq) q = nq - 1;
        qrow[s] = queries + q * row_bytes + half * 16;
    }
    score_t best_s[2][RC];
    int32_t best_i[2][RC];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            best_s[s][r] = M::kWorst;
            best_i[s][r] = 0x7fffffff;
        }

    const int pieces = row_bytes / 32;  // 16-byte pieces per lane and row
    const int all_pairs = (n_clusters + 63) / 64;
    const int n_pairs = min(all_pairs, (int)(blockIdx.y + 1) * pairs_per_slice);
    for (int cp = blockIdx.y * pairs_per_slice; cp < n_pairs; ++cp) {
        const uint8_t* arow[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int r = cp * 64 + i * 32 + col;
            if (r >= n_clusters) r = n_clusters - 1;
            arow[i] = centroids + (int64_t)r * row_bytes + half * 16;
        }
        acc_t acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][s][v] = 0;
        for (int t = 0; t < pieces; ++t) {
            v4i a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = M::prep(*reinterpret_cast<const v4i*>(arow[i] + t * 32));
#pragma unroll
            for (int s = 0; s < 2; ++s) b[s] = M::prep(*reinterpret_cast<const v4i*>(qrow[s] + t * 32));
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int s = 0; s < 2; ++s) M::mma(acc[i][s], a[i], b[s]);
        }
        // result element v of a lane is row 8 (v / 4) + 4 half + v % 4 of its 32-row tile
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int base = cp * 64 + i * 32;
            score_t bs[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) bs[v] = bias[base + 8 * (v / 4) + 4 * half + (v % 4)];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const score_t score = M::score(bs[v], acc[i][s][v], METRIC == 0);
                    const int32_t idx = base + 8 * (v / 4) + 4 * half + (v % 4);
                    if (score < best_s[s][RC - 1]) {
                        // insertion; equal scores stay behind the earlier (smaller) index
                        score_t cs = score;
                        int32_t ci = idx;
#pragma unroll
                        for (int r = 0; r < RC; ++r) {
                            const bool first = cs < best_s[s][r];
                            const score_t ts = best_s[s][r];
                            const int32_t ti = best_i[s][r];
                            best_s[s][r] = first ? cs : ts;
                            best_i[s][r] = first ? ci : ti;
                            cs = first ? ts : cs;
                            ci = first ? ti : ci;
                        }
                    }
                }
            }
        }
    }

    // the two lanes of a query merge their ascending lists through LDS
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < RC; ++r)
            pool[wave][s * 32 + col][half][r] = ((uint64_t)M::ordered(best_s[s][r]) << 32) | (uint32_t)best_i[s][r];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int64_t q = q0 + lane;  // every lane merges one query
    if (q < nq) {
        int ia = 0, ib = 0;
        for (int r = 0; r < RC; ++r) {
            const uint64_t x = ia < RC ? pool[wave][lane][0][ia] : ~0ull;
            const uint64_t y = ib < RC ? pool[wave][lane][1][ib] : ~0ull;
            const bool take_x = x < y;
            if (gridDim.y == 1)
                out[q * RC + r] = (int32_t)(uint32_t)(take_x ? x : y);
            else
                partial[(q * gridDim.y + blockIdx.y) * RC + r] = take_x ? x : y;
            ia += take_x ? 1 : 0;
            ib += take_x ? 0 : 1;
        }
    }
}

// One thread per query: the RC smallest of its slices' words.
template <int RC>
__global__ void __launch_bounds__(256) route_merge_kernel(const uint64_t* __restrict__ partial, int slices, int64_t nq,
                                                          int32_t* __restrict__ out) {
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= nq) return;
    uint64_t best[RC];
#pragma unroll
    for (int r = 0; r < RC; ++r) best[r] = ~0ull;
    for (int i = 0; i < slices * RC; ++i) {
        uint64_t c = partial[q * slices * RC + i];
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            const uint64_t lo = c < best[r] ? c : best[r];
            c = c < best[r] ? best[r] : c;
            best[r] = lo;
        }
    }
#pragma unroll
    for (int r = 0; r < RC; ++r) out[q * RC + r] = (int32_t)(uint32_t)best[r];
}

hipError_t launch_route_merge(int route_c, const uint64_t* partial, int slices, int64_t nq, int32_t* out,
                              hipStream_t stream) {
    const dim3 grid((unsigned)((nq + 255) / 256)), block(256);
#define ANN_RC(N) \
    case N: hipLaunchKernelGGL((route_merge_kernel<N>), grid, block, 0, stream, partial, slices, nq, out); break;
    switch (route_c) {
        ANN_RC(1) ANN_RC(2) ANN_RC(3) ANN_RC(4) ANN_RC(5) ANN_RC(6) ANN_RC(7) ANN_RC(8)
        default: return hipErrorInvalidValue;
    }
#undef ANN_RC
    return hipGetLastError();
}

int route_mfma_slices(int n_clusters, int64_t nq) { return route_slices((n_clusters + 63) / 64, 4, nq); }

template <int DT, int METRIC>
static hipError_t launch_rc(int rc, const uint8_t* centroids, const void* bias, int n_clusters, int row_bytes,
                            const uint8_t* queries, int64_t nq, int32_t* out, uint64_t* partial, int slices,
                            hipStream_t stream) {
    const int all_pairs = (n_clusters + 63) / 64;
    const int pairs_per_slice = (all_pairs + slices - 1) / slices;
    slices = (all_pairs + pairs_per_slice - 1) / pairs_per_slice;  // no slice may start beyond the last pair
    const dim3 grid((unsigned)((nq + 255) / 256), (unsigned)slices), block(256);
#define ANN_RC(N)                                                                                                 \
    case N:                                                                                                       \
        hipLaunchKernelGGL((route_mfma_kernel<DT, METRIC, N>), grid, block, 0, stream, centroids, bias, n_clusters, \
                           row_bytes, queries, nq, out, partial, pairs_per_slice);                                \
        break;
    switch (rc) {
        ANN_RC(1) ANN_RC(2) ANN_RC(3) ANN_RC(4) ANN_RC(5) ANN_RC(6) ANN_RC(7) ANN_RC(8)
        default: return hipErrorInvalidValue;
    }
#undef ANN_RC
    if (slices > 1) return launch_route_merge(rc, partial, slices, nq, out, stream);
    return hipGetLastError();
}

template <int DT, int METRIC>
static hipError_t launch_bias(const uint8_t* centroids, int n_clusters, int row_bytes, void* bias, hipStream_t stream) {
    const int padded = route_mfma_padded(n_clusters);
    hipLaunchKernelGGL((route_bias_kernel<DT, METRIC>), dim3((unsigned)((padded + 255) / 256)), dim3(256), 0, stream,
                       centroids, n_clusters, padded, row_bytes, bias);
    return hipGetLastError();
}

#define ANN_DISPATCH(CALL)                                     \
    switch (dtype * 2 + metric) {                              \
        case 0: return CALL(0, 0);                             \
        case 1: return CALL(0, 1);                             \
        case 2: return CALL(1, 0);                             \
        case 3: return CALL(1, 1);                             \
        case 4: return CALL(2, 0);                             \
        case 5: return CALL(2, 1);                             \
        default: return hipErrorInvalidValue;                  \
    }

hipError_t launch_route_bias(int dtype, int metric, const uint8_t* centroids, int n_clusters, int row_bytes, void* bias,
                             hipStream_t stream) {
#define ANN_CALL(D, M) launch_bias<D, M>(centroids, n_clusters, row_bytes, bias, stream)
    ANN_DISPATCH(ANN_CALL)
#undef ANN_CALL
}

hipError_t launch_route_mfma(int dtype, int metric, int route_c, const uint8_t* centroids, const void* bias,
                             int n_clusters, int row_bytes, const uint8_t* queries, int64_t nq, int32_t* out,
                             uint64_t* partial, int slices, hipStream_t stream) {
#define ANN_CALL(D, M) launch_rc<D, M>(route_c, centroids, bias, n_clusters, row_bytes, queries, nq, out, partial, slices, stream)
    ANN_DISPATCH(ANN_CALL)
#undef ANN_CALL
}

}  // namespace ann

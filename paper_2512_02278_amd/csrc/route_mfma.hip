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
// A wavefront owns a 64 x 64 block of scores (two operand sets of 32 rows on either side): four 32x32
// accumulator tiles, and per 16-byte piece of the rows two reads of each operand feed four matrix
// instructions.  Operand chunks are staged in LDS by the workgroup (see the kernel); the rows can be of any
// length.  In a 32x32 result a lane holds 16 centroids of one query, so a query's best candidates live in a few
// lanes' registers and are merged once at the end.  A lane visits its rows in ascending cluster order, so a
// strict "<" keeps the lower index among equal scores, and the final merge compares (score, index) words.
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

// One workgroup: 128 queries against 128 centroids at a time, four wavefronts in a 2 x 2 arrangement, each
// owning a 64 x 64 block of scores (2 x 2 result tiles of 32 x 32).  The rows are walked in chunks of 64 bytes;
// a chunk of both operands (128 rows x 64 bytes each) is staged in LDS once per workgroup, piece-major
// ([16-byte piece][row], one unit of padding per piece so that the staging writes spread over the banks),
// which is the order the matrix instruction consumes: lane (row % 32, half) reads consecutive 16-byte units.
// The next chunk travels from L2 to registers while the current one is multiplied; two LDS buffers, one
// barrier per chunk.  (Streaming the operands straight from L1/L2 in the instruction's layout - 32 rows x 32
// bytes per load - left this kernel at a twelfth of the fp16 matrix rate.)
template <int DT, int METRIC, int RC>
__global__ void __launch_bounds__(256) route_mfma_kernel(const uint8_t* __restrict__ centroids,
                                                         const void* __restrict__ bias_in, int n_clusters,
                                                         int row_bytes, const uint8_t* __restrict__ queries,
                                                         int64_t nq, int32_t* __restrict__ out,
                                                         uint64_t* __restrict__ partial, int tiles_per_slice) {
    // blockIdx.y = slice of the 128-centroid tiles this workgroup walks; with several slices the best words
    // of a slice go to partial[q][slice][RC] and route_merge_kernel finishes the job
    typedef Mma<DT> M;
    typedef typename M::acc_t acc_t;
    typedef typename M::score_t score_t;
    constexpr int kRows = 128, kPieces = 4, kPieceStride = kRows + 1;
    constexpr int kOperand = kPieces * kPieceStride;  // 16-byte units of one operand chunk
    __shared__ v4i smem[4 * kOperand];                // [buffer 0 / 1][centroids, queries]; afterwards the pool of best lists
    static_assert(sizeof(v4i) * 4 * kOperand >= sizeof(uint64_t) * kRows * 4 * RC, "the pool reuses the staging buffers");
    const score_t* bias = static_cast<const score_t*>(bias_in);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wq = wave >> 1, wc = wave & 1;  // which 64 queries / which 64 centroids of the tile
    const int col = lane & 31, half = lane >> 5;
    const int64_t q0 = (int64_t)blockIdx.x * kRows;

    // staging: thread x moves piece x % 4 of rows x / 4 and x / 4 + 64 (four threads read 64 contiguous bytes)
    const int st_piece = threadIdx.x & 3, st_row = threadIdx.x >> 2;
    const uint8_t* qsrc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int64_t q = q0 + st_row + 64 * i;
        if (q >= nq) q = nq - 1;
        qsrc[i] = queries + q * row_bytes + st_piece * 16;
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

    const int chunks = (row_bytes + 63) / 64;
    const int all_tiles = (n_clusters + kRows - 1) / kRows;
    const int tile_end = min(all_tiles, (int)(blockIdx.y + 1) * tiles_per_slice);
    const v4i zero = v4i{0, 0, 0, 0};
    for (int ct = blockIdx.y * tiles_per_slice; ct < tile_end; ++ct) {
        const uint8_t* csrc[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int r = ct * kRows + st_row + 64 * i;
            if (r >= n_clusters) r = n_clusters - 1;  // its bias never wins
            csrc[i] = centroids + (int64_t)r * row_bytes + st_piece * 16;
        }
        v4i ra[2], rb[2];
        auto fetch = [&](int ch) {
            const int off = ch * 64;
            const bool ok = off + st_piece * 16 < row_bytes;  // rows are multiples of 32 bytes: the last chunk may be half empty
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                ra[i] = ok ? M::prep(*reinterpret_cast<const v4i*>(csrc[i] + off)) : zero;
                rb[i] = ok ? M::prep(*reinterpret_cast<const v4i*>(qsrc[i] + off)) : zero;
            }
        };
        auto stage = [&](int buf) {
            v4i* a = smem + buf * 2 * kOperand;
            v4i* b = a + kOperand;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[st_piece * kPieceStride + st_row + 64 * i] = ra[i];
                b[st_piece * kPieceStride + st_row + 64 * i] = rb[i];
            }
        };
        acc_t acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][s][v] = 0;
        fetch(0);
        stage(0);
        __syncthreads();
        for (int ch = 0; ch < chunks; ++ch) {
            if (ch + 1 < chunks) fetch(ch + 1);
            const v4i* a_chunk = smem + (ch & 1) * 2 * kOperand;
            const v4i* b_chunk = a_chunk + kOperand;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                v4i a[2], b[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) a[i] = a_chunk[(2 * t + half) * kPieceStride + wc * 64 + i * 32 + col];
#pragma unroll
                for (int s = 0; s < 2; ++s) b[s] = b_chunk[(2 * t + half) * kPieceStride + wq * 64 + s * 32 + col];
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int s = 0; s < 2; ++s) M::mma(acc[i][s], a[i], b[s]);
            }
            if (ch + 1 < chunks) stage((ch + 1) & 1);
            __syncthreads();
        }
        // result element v of a lane is row 8 (v / 4) + 4 half + v % 4 of its 32-row tile
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int base = ct * kRows + wc * 64 + i * 32;
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

    // A query's candidates sit in four ascending lists: two lanes (halves) in each of the two wavefronts that
    // hold its row of the tile.  They meet in LDS (the staging buffers are free now) and one thread per
    // query merges them.
    uint64_t* pool = reinterpret_cast<uint64_t*>(smem);  // [query 0..127][list 0..3][RC]
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < RC; ++r)
            pool[((wq * 64 + s * 32 + col) * 4 + wc * 2 + half) * RC + r] =
                ((uint64_t)M::ordered(best_s[s][r]) << 32) | (uint32_t)best_i[s][r];
    __syncthreads();
    const int64_t q = q0 + threadIdx.x;
    if (threadIdx.x < kRows && q < nq) {
        const uint64_t* mine = pool + threadIdx.x * 4 * RC;
        int at[4] = {0, 0, 0, 0};
        for (int r = 0; r < RC; ++r) {
            uint64_t best = ~0ull;
            int from = 0;
#pragma unroll
            for (int l = 0; l < 4; ++l) {
                const uint64_t x = at[l] < RC ? mine[l * RC + at[l]] : ~0ull;
                if (x < best) {
                    best = x;
                    from = l;
                }
            }
#pragma unroll
            for (int l = 0; l < 4; ++l) at[l] += from == l ? 1 : 0;
            if (gridDim.y == 1)
                out[q * RC + r] = (int32_t)(uint32_t)best;
            else
                partial[(q * gridDim.y + blockIdx.y) * RC + r] = best;
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

// Small batches leave most CUs idle when every workgroup walks all centroids, so the centroid range is cut into
// slices (grid.y): about 512 workgroups of 128 queries, each slice at least two tiles of 128 centroids, at most 64.
int route_mfma_slices(int n_clusters, int64_t nq) {
    const int64_t groups = (nq + 127) / 128;
    const int tiles = (n_clusters + 127) / 128;
    int64_t s = 512 / groups;
    if (s > tiles / 2) s = tiles / 2;
    if (s > 64) s = 64;
    return s < 1 ? 1 : (int)s;
}

template <int DT, int METRIC>
static hipError_t launch_rc(int rc, const uint8_t* centroids, const void* bias, int n_clusters, int row_bytes,
                            const uint8_t* queries, int64_t nq, int32_t* out, uint64_t* partial, int slices,
                            hipStream_t stream) {
    const int all_tiles = (n_clusters + 127) / 128;
    const int tiles_per_slice = (all_tiles + slices - 1) / slices;
    slices = (all_tiles + tiles_per_slice - 1) / tiles_per_slice;  // no slice may start beyond the last tile
    const dim3 grid((unsigned)((nq + 127) / 128), (unsigned)slices), block(256);
#define ANN_RC(N)                                                                                                 \
    case N:                                                                                                       \
        hipLaunchKernelGGL((route_mfma_kernel<DT, METRIC, N>), grid, block, 0, stream, centroids, bias, n_clusters, \
                           row_bytes, queries, nq, out, partial, tiles_per_slice);                                \
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

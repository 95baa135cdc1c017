// Routing for uint8 vectors of 128 dimensions on the matrix cores.
//
// Stage 1 of Fantasy (Sec. 3.2, "Local K-means Assignment") is the one dense
// contraction on the path: Q (b x d) against the centroids C (d x C), then the
// nearest clusters per query.  Here both operands are shifted into int8 and the query
// is negated on the way, u = 127 - q (byte-wise q ^ 0x7f) and w = c - 128 (c ^ 0x80),
// multiplied on v_mfma_i32_32x32x32_i8 with exact int32 accumulation (dot = u.w), and
// ranked by the key without its per-query terms:
//     L2:  sum (q - c)^2 = sum ((w + 1) + u)^2   ->   bias_c + 2 dot,  bias_c = sum (c - 127)^2
//     IP:  -q.c = -(127 - u).(w + 128)           ->   bias_c +   dot,  bias_c = -127 sum w
// which orders a query's centroids exactly as (key, cluster index) does.  Negating the
// query makes the score a sum, so one shift-add per result forms the packed word below.
//
// Tiling.  A = 32 centroids x 32 bytes, B = 32 queries x 32 bytes per instruction;
// a wavefront keeps 64 queries (two B sets) in registers for the whole kernel and
// walks all centroids, 32 at a time.  The four wavefronts of a workgroup (256 queries)
// share each centroid tile: it is fetched from L2 once (one 16-byte piece per thread,
// shifted to int8 on the way), double-buffered in LDS in the order the matrix
// instruction consumes it, and read back conflict-free.  Without the sharing the kernel
// is bound by L2 bandwidth.  In the 32x32 result a lane holds 16 centroids
// of ONE query (column = lane % 32), so the running best list of a query lives in
// two lanes' registers and needs no exchange until the end.  Rows are visited in
// ascending cluster order, so a strict "<" keeps the lower index among equal keys.
//
// Selection is the expensive part (16 results per lane and tile against 4 matrix
// instructions), so it works on packed words: the bias array holds bias*16 + v, v being
// the result slot of that row inside a lane, and one multiply-add gives score*16 + v.  A
// tree of v_min3 finds a tile's best (score, row) in a lane, and only a tile whose best
// beats the worst kept score is looked at value by value.
#include <hip/hip_runtime.h>

#include "route_mfma.h"
#include "route_mfma_u8.h"

namespace ann {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kPadScore = 0x03ffffff;  // score of the padding rows: above every real one, and score*16 fits

template <int METRIC>
__global__ void __launch_bounds__(256) centroid_bias_kernel(const uint8_t* centroids, int n_clusters, int padded,
                                                            int32_t* bias) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= padded) return;
    // result slot of a row inside a lane: tile row 8 (v / 4) + 4 half + v % 4  <->  v
    const int slot = 4 * ((c & 31) >> 3) + (c & 3);
    if (c >= n_clusters) {
        bias[c] = kPadScore * 16 + slot;
        return;
    }
    const uint32_t* row = reinterpret_cast<const uint32_t*>(centroids + (int64_t)c * 128);
    int32_t acc = 0;
    for (int i = 0; i < 32; ++i) {
        if (METRIC == 0) {
            // (c - 127) as int8 is c ^ 0x7f with the sign flipped: its square is the same
            const uint32_t w1 = row[i] ^ 0x7f7f7f7fu;
            acc = __builtin_amdgcn_sdot4((int)w1, (int)w1, acc, false);
        } else {
            const uint32_t w = row[i] ^ 0x80808080u;
            acc = __builtin_amdgcn_sdot4((int)w, 0x01010101, acc, false);
        }
    }
    bias[c] = (METRIC == 0 ? acc : -127 * acc) * 16 + slot;
}

template <int METRIC, int RC>
__global__ void __launch_bounds__(256) route_mfma_u8_kernel(const uint8_t* __restrict__ centroids,
                                                            const int32_t* __restrict__ bias, int n_clusters,
                                                            const uint8_t* __restrict__ queries, int64_t nq,
                                                            int32_t* __restrict__ out, uint64_t* __restrict__ partial,
                                                            int tiles_per_slice) {
    // blockIdx.y = slice of the centroid tiles this workgroup walks.  With one slice the final
    // clusters go to `out`; with several, each slice writes its best (score, cluster) words to
    // partial[q][slice][RC] and route_merge_kernel picks the overall best.
    constexpr int NQS = 2;  // query sets of 32 per wavefront
    __shared__ uint64_t pool[4][NQS * 32][2][RC];
    __shared__ v4i atile[2][8 * 32];  // [piece 0..7][row 0..31] 16-byte units of one centroid tile
    __shared__ v4i btile[2][8];       // the tile's 32 bias words
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int64_t q0 = ((int64_t)blockIdx.x * 4 + wave) * (NQS * 32);  // may lie beyond nq: such wavefronts only help loading

    // B: lane holds, for query (q0 + 32 s + col), the 16 bytes number 2 t + half of the row
    v4i b[NQS][4];
#pragma unroll
    for (int s = 0; s < NQS; ++s) {
        int64_t q = q0 + s * 32 + col;
        if (q >= nq) q = nq - 1;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            b[s][t] = *reinterpret_cast<const v4i*>(queries + q * 128 + (2 * t + half) * 16);
            b[s][t] ^= (int)0x7f7f7f7f;  // u = 127 - q
        }
    }
    int32_t best_s[NQS][RC], best_i[NQS][RC];
#pragma unroll
    for (int s = 0; s < NQS; ++s)
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            best_s[s][r] = 0x7fffffff;
            best_i[s][r] = 0x7fffffff;
        }

    // thread x fetches piece x % 8 of tile row x / 8 (eight threads read one 128-byte row)
    const int ld_row = threadIdx.x >> 3, ld_piece = threadIdx.x & 7;
    const int all_tiles = (n_clusters + 31) / 32;
    const int tile0 = blockIdx.y * tiles_per_slice;
    const int n_tiles = min(all_tiles, tile0 + tiles_per_slice);
    auto fetch = [&](int ct) {
        int r = ct * 32 + ld_row;
        if (r >= n_clusters) r = n_clusters - 1;
        return *reinterpret_cast<const v4i*>(centroids + (int64_t)r * 128 + ld_piece * 16) ^ (int)0x80808080;
    };
    const v4i* bias4 = reinterpret_cast<const v4i*>(bias);
    atile[tile0 & 1][ld_piece * 32 + ld_row] = fetch(tile0);
    if (threadIdx.x < 8) btile[tile0 & 1][threadIdx.x] = bias4[tile0 * 8 + threadIdx.x];
    __syncthreads();
    for (int ct = tile0; ct < n_tiles; ++ct) {
        v4i next, next_bias;
        if (ct + 1 < n_tiles) {
            next = fetch(ct + 1);
            if (threadIdx.x < 8) next_bias = bias4[(ct + 1) * 8 + threadIdx.x];
        }
        v4i a[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) a[t] = atile[ct & 1][(2 * t + half) * 32 + col];
        // result element v of a lane is row 8 (v / 4) + 4 half + v % 4 of the tile
        v4i bs[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) bs[g] = btile[ct & 1][2 * g + half];
        // both query sets are multiplied before either is looked at: the matrix core works on
        // the second while the vector ALU selects from the first
        v16i accs[NQS];
#pragma unroll
        for (int s = 0; s < NQS; ++s) {
            accs[s] = v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int t = 0; t < 4; ++t) accs[s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t], b[s][t], accs[s], 0, 0, 0);
        }
#pragma unroll
        for (int s = 0; s < NQS; ++s) {
            const v16i acc = accs[s];
            // packed[v] = score * 16 + v
            int32_t packed[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) packed[v] = bs[v / 4][v % 4] + (acc[v] << (METRIC == 0 ? 5 : 4));
            int32_t m01 = min(min(packed[0], packed[1]), packed[2]);
            int32_t m02 = min(min(packed[3], packed[4]), packed[5]);
            int32_t m03 = min(min(packed[6], packed[7]), packed[8]);
            int32_t m04 = min(min(packed[9], packed[10]), packed[11]);
            int32_t m05 = min(min(packed[12], packed[13]), packed[14]);
            const int32_t tile_best = min(min(min(m01, m02), min(m03, m04)), min(m05, packed[15]));
            const int32_t tile_score = tile_best >> 4;
            if constexpr (RC == 1) {
                // strict "<" on the score alone: among equal scores the earlier tile stays
                const bool better = tile_score < best_s[s][0];
                best_s[s][0] = better ? tile_score : best_s[s][0];
                best_i[s][0] = better ? ct * 32 + 8 * ((tile_best & 15) >> 2) + 4 * half + (tile_best & 3) : best_i[s][0];
            } else if (__any(tile_score < best_s[s][RC - 1])) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int32_t score = packed[v] >> 4;
                    const int32_t idx = ct * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    if (score < best_s[s][RC - 1]) {
                        // insertion; equal scores stay behind the earlier (smaller) index
                        int32_t cs = score, ci = idx;
#pragma unroll
                        for (int r = 0; r < RC; ++r) {
                            const bool first = cs < best_s[s][r];
                            const int32_t ts = best_s[s][r], ti = best_i[s][r];
                            best_s[s][r] = first ? cs : ts;
                            best_i[s][r] = first ? ci : ti;
                            cs = first ? ts : cs;
                            ci = first ? ti : ci;
                        }
                    }
                }
            }
        }
        if (ct + 1 < n_tiles) {
            atile[(ct + 1) & 1][ld_piece * 32 + ld_row] = next;
            if (threadIdx.x < 8) btile[(ct + 1) & 1][threadIdx.x] = next_bias;
        }
        __syncthreads();
    }

    // the two lanes of a query merge their ascending lists through LDS
#pragma unroll
    for (int s = 0; s < NQS; ++s)
#pragma unroll
        for (int r = 0; r < RC; ++r)
            pool[wave][s * 32 + col][half][r] =
                ((uint64_t)((uint32_t)best_s[s][r] ^ 0x80000000u) << 32) | (uint32_t)best_i[s][r];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // lane -> query (q0 + lane): every lane merges one query
    const int64_t q = q0 + lane;
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

template <int METRIC>
static hipError_t launch_rc(int rc, const uint8_t* centroids, const int32_t* bias, int n_clusters,
                            const uint8_t* queries, int64_t nq, int32_t* out, uint64_t* partial, int slices,
                            hipStream_t stream) {
    const int all_tiles = (n_clusters + 31) / 32;
    const int tiles_per_slice = (all_tiles + slices - 1) / slices;
    slices = (all_tiles + tiles_per_slice - 1) / tiles_per_slice;  // no slice may start beyond the last tile
    const dim3 grid((unsigned)((nq + 255) / 256), (unsigned)slices), block(256);
    switch (rc) {
        case 1:
            hipLaunchKernelGGL((route_mfma_u8_kernel<METRIC, 1>), grid, block, 0, stream, centroids, bias, n_clusters, queries, nq, out, partial, tiles_per_slice);
            break;
        case 2:
            hipLaunchKernelGGL((route_mfma_u8_kernel<METRIC, 2>), grid, block, 0, stream, centroids, bias, n_clusters, queries, nq, out, partial, tiles_per_slice);
            break;
        case 3:
            hipLaunchKernelGGL((route_mfma_u8_kernel<METRIC, 3>), grid, block, 0, stream, centroids, bias, n_clusters, queries, nq, out, partial, tiles_per_slice);
            break;
        case 4:
            hipLaunchKernelGGL((route_mfma_u8_kernel<METRIC, 4>), grid, block, 0, stream, centroids, bias, n_clusters, queries, nq, out, partial, tiles_per_slice);
            break;
        case 5:
            hipLaunchKernelGGL((route_mfma_u8_kernel<METRIC, 5>), grid, block, 0, stream, centroids, bias, n_clusters, queries, nq, out, partial, tiles_per_slice);
            break;
        case 6:
            hipLaunchKernelGGL((route_mfma_u8_kernel<METRIC, 6>), grid, block, 0, stream, centroids, bias, n_clusters, queries, nq, out, partial, tiles_per_slice);
            break;
        case 7:
            hipLaunchKernelGGL((route_mfma_u8_kernel<METRIC, 7>), grid, block, 0, stream, centroids, bias, n_clusters, queries, nq, out, partial, tiles_per_slice);
            break;
        case 8:
            hipLaunchKernelGGL((route_mfma_u8_kernel<METRIC, 8>), grid, block, 0, stream, centroids, bias, n_clusters, queries, nq, out, partial, tiles_per_slice);
            break;
        default: return hipErrorInvalidValue;
    }
    if (slices > 1) return launch_route_merge(rc, partial, slices, nq, out, stream);
    return hipGetLastError();
}

hipError_t launch_centroid_bias_u8(int metric, const uint8_t* centroids, int n_clusters, int32_t* bias,
                                   hipStream_t stream) {
    const int padded = route_mfma_u8_padded(n_clusters);
    const dim3 grid((unsigned)((padded + 255) / 256)), block(256);
    if (metric == 0)
        hipLaunchKernelGGL((centroid_bias_kernel<0>), grid, block, 0, stream, centroids, n_clusters, padded, bias);
    else
        hipLaunchKernelGGL((centroid_bias_kernel<1>), grid, block, 0, stream, centroids, n_clusters, padded, bias);
    return hipGetLastError();
}

int route_mfma_u8_slices(int n_clusters, int64_t nq) { return route_slices((n_clusters + 31) / 32, 8, nq); }

hipError_t launch_route_mfma_u8(int metric, int route_c, const uint8_t* centroids, const int32_t* bias, int n_clusters,
                                const uint8_t* queries, int64_t nq, int32_t* out, uint64_t* partial, int slices,
                                hipStream_t stream) {
    return metric == 0 ? launch_rc<0>(route_c, centroids, bias, n_clusters, queries, nq, out, partial, slices, stream)
                       : launch_rc<1>(route_c, centroids, bias, n_clusters, queries, nq, out, partial, slices, stream);
}

}  // namespace ann

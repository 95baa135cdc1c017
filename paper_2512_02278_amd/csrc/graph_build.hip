// kNN graph -> fixed-degree search graph.
//
// The paper searches "the CAGRA index" (Fantasy Sec. 3.2, stage 3) and leaves its construction
// to that index's own publication; the steps here are that publication's graph optimisation,
// with ranks standing in for distances:
//   1. detour count of an edge x -> y of rank j: the number of earlier neighbours z of x (rank
//      below j) that list y at a rank below j;
//   2. a row keeps its d_out edges of smallest (count, rank);
//   3. reverse edges: node y collects the sources x of its in-edges, ordered by (position of y
//      in x's pruned row, x), at most d_out of them;
//   4. merged row: the first d_out - d_out/2 forward edges, then up to d_out/2 reverse edges not
//      among those, then the remaining forward edges that are not in the row yet.
// An id outside [0, n) or equal to the row's own node is absent everywhere.
//
// One wavefront works on a run of consecutive nodes.  Step 1 is the expensive one: d_in graph
// rows of d_in ids are read per node (16 KB at d_in = 64), a random gather like the search's
// own, but with rows that mostly sit in the node's own cluster: runs of consecutive nodes stay
// on one XCD so that its L2 serves the re-reads.  The ids of x's row go into a small LDS table
// (id -> rank); the ids of every neighbour's row pass a Bloom filter of x's row, and those that
// survive are looked up in the table and bump an LDS counter.
// Step 3 is a counting sort by target (histogram - counted by the pruning kernel itself -, scan,
// scatter of (position, source) words) followed by a selection per node, so that the result does not
// depend on the order in which the atomics land.
#include <hip/hip_runtime.h>

#include "graph_build.h"
#include "wave.h"

namespace ann {
namespace {

constexpr int kNodesPerWave = 32;
// Nodes per workgroup of in_edges_kernel (at most 256).  Small on purpose: the fewer nodes an XCD has in
// flight, the fewer target lists are half-written in its L2 at a time, and the more of their 8-byte words
// merge into whole lines before they are written back (22.5 ms per 25M nodes with 256, 9.5 ms with 8).
constexpr int kChunkNodes = 8;
constexpr int kScanChunk = 4096;  // elements per workgroup of the scan kernels: 256 threads x 16

__device__ __forceinline__ void wave_lds_sync() { __syncthreads(); }  // one wavefront per workgroup

__device__ __forceinline__ bool is_present(int32_t y, int64_t n, int64_t x) { return y >= 0 && (int64_t)y < n && (int64_t)y != x; }

// Node run of workgroup b: runs are dealt to the 8 XCDs (workgroup b runs on XCD b % 8) so that
// each XCD walks one contiguous eighth of the ids.
__device__ __forceinline__ int64_t first_node_of(int64_t b, int64_t runs_per_xcd) {
    return ((b & 7) * runs_per_xcd + (b >> 3)) * kNodesPerWave;
}

// ------------------------------------------------------------------------------------- steps 1 + 2
// id -> rank table of one row: B buckets of four 32-bit ids (one 16-byte LDS read fetches a bucket)
// plus one byte of rank per slot.  A bucket fills from slot 0 upwards; an id that finds its bucket
// full goes to the next one.  With 64*R ids in 128*R buckets a full bucket is met by about one
// lookup in six hundred, so the lookup is a straight line: one bucket, four compares, and a
// wave-uniform branch to the rare walk over further buckets.  (A per-lane probing loop would
// run as long as its slowest lane and cost mostly scalar branch and mask instructions, and the
// scalar unit is shared by the four SIMDs of a compute unit.)
constexpr uint32_t kEmptyId = 0xffffffffu;

template <int B>
__device__ __forceinline__ uint32_t bucket_of(uint32_t id) {
    return (id * 0x9E3779B1u) >> (32 - __builtin_ctz(B));
}

// Slot index of `id` in bucket `b`, or -1.
__device__ __forceinline__ int match_in(const uint4 t, uint32_t id) {
    return t.x == id ? 0 : t.y == id ? 1 : t.z == id ? 2 : t.w == id ? 3 : -1;
}

template <int B>
__device__ __forceinline__ void rank_table_insert(uint32_t* tid, uint8_t* trk, uint32_t id, int rank) {
    uint32_t b = bucket_of<B>(id);
    for (;;) {  // ends: the row's ids fill at most an eighth of the slots
        for (int s = 0; s < 4; ++s) {
            const uint32_t old = atomicCAS(&tid[4 * b + s], kEmptyId, id);
            if (old == kEmptyId) {
                trk[4 * b + s] = (uint8_t)rank;
                return;
            }
            if (old == id) return;  // a repeated id (not allowed in a row) keeps one of its ranks
        }
        b = (b + 1) & (B - 1);
    }
}

// Slot of `id` (4 * bucket + position) or -1.  Called by all lanes; lanes with live == false get -1.
template <int B>
__device__ __forceinline__ int rank_table_find(const uint32_t* tid, uint32_t id, bool live) {
    uint32_t b = bucket_of<B>(id);
    uint4 t = reinterpret_cast<const uint4*>(tid)[b];
    int s = match_in(t, id);
    bool more = live && s < 0 && t.w != kEmptyId;  // bucket full and no match: the id may have moved on
    while (__ballot(more)) {
        if (more) {
            b = (b + 1) & (B - 1);
            t = reinterpret_cast<const uint4*>(tid)[b];
            s = match_in(t, id);
            more = s < 0 && t.w != kEmptyId;
        }
    }
    return (live && s >= 0) ? (int)(4 * b) + s : -1;
}

// R registers per lane: rank j of a row lives in lane j % 64, register j / 64 (d_in <= 64 * R).
//
// Only about one id in ten of a neighbour's row is also in x's row (clustered 128-d data), so the
// ids first pass a one-hash Bloom filter of x's row (2048 * R bits in LDS, one 4-byte read each);
// the survivors are queued in LDS with the later of their two ranks and looked up 64 at a time.
//
// COUNT: the kernel also counts the in-edges of the pruned graph (step 3's histogram) - one returning
// atomic per pruned edge, whose result is the edge's slot in its target's list.  The atomics are
// memory-side work that overlaps this kernel's instruction-bound lookups, instead of a pass of its own.
template <int R, bool COUNT, bool VEC>
__global__ void __launch_bounds__(64) graph_prune_kernel(const int32_t* __restrict__ knn, int64_t n, int d_in, int d_out,
                                                         int32_t* __restrict__ pruned, int64_t runs_per_xcd,
                                                         uint32_t* indeg, uint32_t* __restrict__ slot) {
    constexpr int B = 128 * R, U = 8, kBloomBits = 11 + (R > 1), kQueue = 128;
    __shared__ __align__(16) uint32_t tid[4 * B];   // ids of x's row, by bucket
    __shared__ uint8_t trk[4 * B];                  // their ranks
    __shared__ uint32_t bloom[(1 << kBloomBits) / 32];
    __shared__ uint64_t queue[kQueue];              // ring of (later rank << 32) | id waiting for a lookup
    __shared__ uint32_t cnt[64 * R];                // detour count per rank
    __shared__ __align__(16) uint32_t key[64 * R];  // (count << 8) | rank, all ones where absent
    __shared__ int32_t nbr[64 * R];                 // x's row, -1 where absent
    __shared__ int32_t orow[64];
    const int lane = lane_id();
    const int64_t x0 = first_node_of(blockIdx.x, runs_per_xcd);
    const int64_t x1 = x0 + kNodesPerWave < n ? x0 + kNodesPerWave : n;

    // looks up queue[head .. head + 64) (the first `live` of them are real) and counts the detours
    auto drain = [&](int head, int live) {
        const uint64_t e = queue[(head + lane) & (kQueue - 1)];
        const int slot = rank_table_find<B>(tid, (uint32_t)e, lane < live);
        if (slot >= 0) {
            const int j = trk[slot];
            if ((int)(e >> 32) < j) atomicAdd(&cnt[j], 1u);  // both hops rank below the edge itself
        }
    };

    for (int64_t x = x0; x < x1; ++x) {
        int32_t mine[R];
        bool have[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int j = lane + 64 * r;
            mine[r] = j < d_in ? knn[x * d_in + j] : -1;
            have[r] = is_present(mine[r], n, x);
            nbr[j] = have[r] ? mine[r] : -1;
            cnt[j] = 0u;
        }
        for (int i = lane; i < B; i += 64) reinterpret_cast<uint4*>(tid)[i] = make_uint4(kEmptyId, kEmptyId, kEmptyId, kEmptyId);
        for (int i = lane; i < (1 << kBloomBits) / 32; i += 64) bloom[i] = 0u;
        wave_lds_sync();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (have[r]) {
                rank_table_insert<B>(tid, trk, (uint32_t)mine[r], lane + 64 * r);
                const uint32_t hb = ((uint32_t)mine[r] * 0x9E3779B1u) >> (32 - kBloomBits);
                atomicOr(&bloom[hb >> 5], 1u << (hb & 31));
            }
        }
        wave_lds_sync();

        // rows of the neighbours at ranks 0 .. d_in-2 (the last one has no edge after it); every id that passes
        // the Bloom filter is queued with the later of its two ranks
        int head = 0, queued = 0;  // wave-uniform
        auto push = [&](int32_t ys, int later) {
            const uint32_t y = (uint32_t)ys;
            const uint32_t hb = (y * 0x9E3779B1u) >> (32 - kBloomBits);
            const bool pass = ys >= 0 && ((bloom[hb >> 5] >> (hb & 31)) & 1u);
            const uint64_t m = __ballot(pass);
            if (pass) queue[(head + queued + rank_below(m)) & (kQueue - 1)] = ((uint64_t)(uint32_t)later << 32) | y;
            queued += __builtin_popcountll(m);
            if (queued >= 64) {
                wave_lds_sync();
                drain(head, 64);
                head = (head + 64) & (kQueue - 1);
                queued -= 64;
            }
        };
        if constexpr (VEC) {
            // rows of d_in % 4 == 0 ids, 16-byte aligned: a lane reads four consecutive ranks, 16 * R lanes
            // cover a row, so one load instruction fetches 4 / R rows; four of them in flight
            constexpr int kLanesPerRow = 16 * R, kRowsPerLoad = 64 / kLanesPerRow, UV = 4;
            const int quad = lane % kLanesPerRow, sub = lane / kLanesPerRow;
            for (int i0 = 0; i0 < d_in - 1; i0 += UV * kRowsPerLoad) {
                int4 v[UV];
#pragma unroll
                for (int u = 0; u < UV; ++u) {
                    const int i = i0 + u * kRowsPerLoad + sub;
                    const int32_t z = i < d_in - 1 ? nbr[i] : -1;
                    v[u] = make_int4(-1, -1, -1, -1);
                    if (z >= 0 && 4 * quad < d_in - 1) v[u] = *reinterpret_cast<const int4*>(knn + (int64_t)z * d_in + 4 * quad);
                }
#pragma unroll
                for (int u = 0; u < UV; ++u) {
                    const int i = i0 + u * kRowsPerLoad + sub;
                    const int32_t c4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int rr = 4 * quad + c;
                        push(rr < d_in - 1 ? c4[c] : -1, max(i, rr));
                    }
                }
            }
        } else {
            // any d_in: a lane reads rank lane (+ 64) of one row per load, U rows in flight
            for (int i0 = 0; i0 < d_in - 1; i0 += U) {
                int32_t v[U][R];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = i0 + u;
                    const int32_t z = i < d_in - 1 ? __builtin_amdgcn_readfirstlane(nbr[i]) : -1;
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const int rr = lane + 64 * r;
                        v[u][r] = (z >= 0 && rr < d_in - 1) ? knn[(int64_t)z * d_in + rr] : -1;
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int r = 0; r < R; ++r) push(v[u][r], max(i0 + u, lane + 64 * r));
                }
            }
        }
        wave_lds_sync();
        if (queued > 0) drain(head, queued);
        wave_lds_sync();

        // position of every present edge in ascending (count, rank)
        uint32_t mykey[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int j = lane + 64 * r;
            mykey[r] = have[r] ? ((cnt[j] << 8) | (uint32_t)j) : 0xffffffffu;
            key[j] = mykey[r];
        }
        wave_lds_sync();
        int pos[R];
#pragma unroll
        for (int r = 0; r < R; ++r) pos[r] = 0;
        // fully unrolled, the 32 reads of two registers per lane would all be in flight and take 128 VGPRs
        constexpr int kRankUnroll = R == 1 ? 16 : 4;
#pragma unroll kRankUnroll
        for (int t = 0; t < 16 * R; ++t) {
            const uint4 k4 = reinterpret_cast<const uint4*>(key)[t];
#pragma unroll
            for (int r = 0; r < R; ++r)
                pos[r] += (k4.x < mykey[r]) + (k4.y < mykey[r]) + (k4.z < mykey[r]) + (k4.w < mykey[r]);
        }
        orow[lane] = -1;
        wave_lds_sync();
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (have[r] && pos[r] < d_out) orow[pos[r]] = mine[r];
        wave_lds_sync();
        if (lane < d_out) {
            const int32_t y = orow[lane];  // a present id or -1
            pruned[x * d_out + lane] = y;
            if (COUNT && y >= 0) slot[x * d_out + lane] = atomicAdd(&indeg[y], 1u);
        }
        wave_lds_sync();
    }
}

// ------------------------------------------------------------------------------------- step 3
__global__ void __launch_bounds__(256) fill_zero_u32_kernel(uint32_t* p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0u;
}

// Chunk of kChunkNodes nodes a workgroup of the edge kernel works on: like the node runs above, the chunks
// are dealt so that an XCD walks a contiguous eighth of the ids; the edges of neighbouring nodes point
// into the same few clusters, and their 8-byte words then meet in one L2 before they are written back.
__device__ __forceinline__ int64_t chunk_of(int64_t b, int64_t chunks_per_xcd) { return (b & 7) * chunks_per_xcd + (b >> 3); }

// Chunk c covers the kChunkNodes nodes from kChunkNodes * c on: element t of their rows is node
// kChunkNodes * c + t / d, position t % d, with t / d == (t * d_inv) >> 22 for t < 256 * d, d <= 64
// (d_inv = ceil(2^22 / d)).
// Exclusive scan of indeg[0..n) into off[0..n] (64-bit), in three launches: per-chunk sums, a scan of
// those by one workgroup, then every chunk scans itself on top of its prefix.
__global__ void __launch_bounds__(256) chunk_sums_kernel(const uint32_t* __restrict__ deg, int64_t n, int64_t* sums) {
    __shared__ int64_t part[256];
    const int t = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + t * 16;
    int64_t s = 0;
    for (int i = 0; i < 16; ++i)
        if (base + i < n) s += deg[base + i];
    part[t] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (t < w) part[t] += part[t + w];
        __syncthreads();
    }
    if (t == 0) sums[blockIdx.x] = part[0];
}

__global__ void __launch_bounds__(1024) scan_sums_kernel(int64_t* sums, int64_t count) {
    __shared__ int64_t part[1024];
    const int t = threadIdx.x;
    const int64_t per = (count + 1023) / 1024;
    const int64_t lo = t * per, hi = lo + per < count ? lo + per : count;
    int64_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += sums[i];
    part[t] = s;
    __syncthreads();
    for (int w = 1; w < 1024; w <<= 1) {  // Hillis-Steele inclusive scan of the per-thread sums
        const int64_t v = t >= w ? part[t - w] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    int64_t run = part[t] - s;
    for (int64_t i = lo; i < hi; ++i) {
        const int64_t c = sums[i];
        sums[i] = run;
        run += c;
    }
}

__global__ void __launch_bounds__(256) offsets_kernel(const uint32_t* __restrict__ deg, int64_t n,
                                                      const int64_t* __restrict__ sums, int64_t* off) {
    __shared__ int64_t part[256];
    const int t = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + t * 16;
    int64_t s = 0;
    for (int i = 0; i < 16; ++i)
        if (base + i < n) s += deg[base + i];
    part[t] = s;
    __syncthreads();
    for (int w = 1; w < 256; w <<= 1) {
        const int64_t v = t >= w ? part[t - w] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    int64_t run = sums[blockIdx.x] + part[t] - s;
    for (int i = 0; i < 16; ++i) {
        if (base + i < n) {
            off[base + i] = run;
            run += deg[base + i];
            if (base + i == n - 1) off[n] = run;
        }
    }
}

// pairs[off[y] + slot[e]] <- (position << 32) | source of every edge e into y
__global__ void __launch_bounds__(256) in_edges_kernel(const int32_t* __restrict__ g, int64_t n, int d, uint32_t d_inv,
                                                       const int64_t* __restrict__ off, const uint32_t* __restrict__ slot,
                                                       uint64_t* __restrict__ pairs, int64_t chunks_per_xcd) {
    const int64_t xb = chunk_of(blockIdx.x, chunks_per_xcd) * kChunkNodes;
    const int rows = n - xb < kChunkNodes ? (n > xb ? (int)(n - xb) : 0) : kChunkNodes;
    for (int t = threadIdx.x; t < rows * d; t += 256) {
        const int xl = (int)(((uint32_t)t * d_inv) >> 22);
        const int64_t x = xb + xl;
        const int32_t y = g[xb * d + t];
        if (is_present(y, n, x)) pairs[off[y] + slot[xb * d + t]] = ((uint64_t)(uint32_t)(t - xl * d) << 32) | (uint32_t)x;
    }
}

// ------------------------------------------------------------------------------------- steps 3 (selection) + 4
__global__ void __launch_bounds__(64) graph_merge_kernel(const int32_t* __restrict__ pruned, int64_t n, int d,
                                                         const int64_t* __restrict__ off,
                                                         const uint64_t* __restrict__ pairs, int32_t* __restrict__ out,
                                                         int64_t runs_per_xcd) {
    __shared__ int32_t fwd[64];
    __shared__ int32_t row[64];
    const int lane = lane_id();
    const int h = d / 2, nh = d - h;
    const int64_t x0 = first_node_of(blockIdx.x, runs_per_xcd);
    const int64_t x1 = x0 + kNodesPerWave < n ? x0 + kNodesPerWave : n;
    for (int64_t x = x0; x < x1; ++x) {
        // the 64 smallest (position, source) words of x's in-edges, ascending: one word per lane
        uint64_t best[1] = {kInfKey};
        const int64_t lo = off[x], hi = off[x + 1];
        for (int64_t c0 = lo; c0 < hi; c0 += 64) {
            uint64_t v[1] = {c0 + lane < hi ? pairs[c0 + lane] : kInfKey};
            bitonic_sort<1>(v, lane);
            if (c0 == lo) {  // the first chunk (the only one for most nodes) is the best so far as it is
                best[0] = v[0];
                continue;
            }
            // element e of the best so far against element 63 - e of the sorted chunk keeps the 64
            // smallest of both, as one bitonic run
            const uint64_t o = xor_lane64<63>(v[0], lane);
            best[0] = o < best[0] ? o : best[0];
            bitonic_merge<1>(best, lane);
        }
        const int32_t rv = (lane < d && best[0] != kInfKey) ? (int32_t)(uint32_t)best[0] : -1;
        const int32_t f = lane < d ? pruned[x * d + lane] : -1;
        const bool fok = is_present(f, n, x);
        fwd[lane] = fok ? f : -1;
        const bool head = fok && lane < nh;
        const uint64_t bh = __ballot(head);
        const int n_head = __builtin_popcountll(bh);
        if (head) row[rank_below(bh)] = f;
        wave_lds_sync();
        bool member = false;
        for (int t = 0; t < nh; ++t) member |= fwd[t] == rv;
        const bool fresh = rv >= 0 && !member;
        const uint64_t bf = __ballot(fresh);
        const int rk = rank_below(bf);
        const int n_fresh = __builtin_popcountll(bf);
        const int n_take = n_fresh < h ? n_fresh : h;
        if (fresh && rk < h) row[n_head + rk] = rv;
        wave_lds_sync();
        bool dup = false;
        for (int t = 0; t < n_take; ++t) dup |= row[n_head + t] == f;
        const bool tail = fok && lane >= nh && !dup;
        const uint64_t bt = __ballot(tail);
        const int pos = n_head + n_take + rank_below(bt);
        if (tail && pos < d) row[pos] = f;
        const int all = n_head + n_take + __builtin_popcountll(bt);
        const int len = all < d ? all : d;
        wave_lds_sync();
        if (lane < d) out[x * d + lane] = lane < len ? row[lane] : -1;
        wave_lds_sync();
    }
}

unsigned blocks_for(int64_t items) {
    const int64_t b = (items + 255) / 256;
    return (unsigned)(b < 65536 ? (b > 0 ? b : 1) : 65536);
}

int64_t align256(int64_t b) { return (b + 255) & ~(int64_t)255; }

int64_t runs_per_xcd_of(int64_t n) {
    const int64_t runs = (n + kNodesPerWave - 1) / kNodesPerWave;
    return (runs + 7) / 8;
}

}  // namespace

namespace {

template <int R, bool COUNT>
void launch_prune_rc(bool vec, dim3 grid, hipStream_t stream, const int32_t* knn, int64_t n, int d_in, int d_out,
                     int32_t* pruned, int64_t rpx, uint32_t* indeg, uint32_t* slot) {
    if (vec)
        hipLaunchKernelGGL((graph_prune_kernel<R, COUNT, true>), grid, dim3(64), 0, stream, knn, n, d_in, d_out, pruned, rpx, indeg, slot);
    else
        hipLaunchKernelGGL((graph_prune_kernel<R, COUNT, false>), grid, dim3(64), 0, stream, knn, n, d_in, d_out, pruned, rpx, indeg, slot);
}

hipError_t launch_prune(const int32_t* knn, int64_t n, int d_in, int d_out, int32_t* pruned, uint32_t* indeg,
                        uint32_t* slot, hipStream_t stream) {
    const int64_t rpx = runs_per_xcd_of(n);
    const dim3 grid((unsigned)(8 * rpx));
    // rows that start on 16-byte boundaries are read four ids per lane
    const bool vec = d_in % 4 == 0 && (reinterpret_cast<uintptr_t>(knn) & 15u) == 0;
    if (d_in <= 64 && indeg) launch_prune_rc<1, true>(vec, grid, stream, knn, n, d_in, d_out, pruned, rpx, indeg, slot);
    else if (d_in <= 64) launch_prune_rc<1, false>(vec, grid, stream, knn, n, d_in, d_out, pruned, rpx, indeg, slot);
    else if (indeg) launch_prune_rc<2, true>(vec, grid, stream, knn, n, d_in, d_out, pruned, rpx, indeg, slot);
    else launch_prune_rc<2, false>(vec, grid, stream, knn, n, d_in, d_out, pruned, rpx, indeg, slot);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_graph_prune(const int32_t* knn, int64_t n, int d_in, int d_out, int32_t* pruned, hipStream_t stream) {
    return launch_prune(knn, n, d_in, d_out, pruned, nullptr, nullptr, stream);
}

// scratch layout: pruned (n * d i32) | indeg (n u32) | off (n + 1 i64) | chunk sums (i64) | pairs (n * d u64)
int64_t graph_optimize_scratch_bytes(int64_t n, int d) {
    const int64_t chunks = (n + kScanChunk - 1) / kScanChunk;
    return align256(n * d * 4) + align256(n * 4) + align256((n + 1) * 8) + align256(chunks * 8) + align256(n * d * 8);
}

hipError_t launch_graph_optimize(const int32_t* knn, int64_t n, int d_in, int d, int32_t* out, void* scratch,
                                 hipStream_t stream) {
    const int64_t chunks = (n + kScanChunk - 1) / kScanChunk;
    char* base = static_cast<char*>(scratch);
    int32_t* pruned = reinterpret_cast<int32_t*>(base);
    base += align256(n * d * 4);
    uint32_t* indeg = reinterpret_cast<uint32_t*>(base);
    base += align256(n * 4);
    int64_t* off = reinterpret_cast<int64_t*>(base);
    base += align256((n + 1) * 8);
    int64_t* sums = reinterpret_cast<int64_t*>(base);
    base += align256(chunks * 8);
    uint64_t* pairs = reinterpret_cast<uint64_t*>(base);
    // until the last kernel writes it, `out` holds the slot of every edge within its target's list
    uint32_t* slot = reinterpret_cast<uint32_t*>(out);
    const uint32_t d_inv = (uint32_t)(((1u << 22) + d - 1) / d);
    const int64_t chunks_per_xcd = ((n + kChunkNodes - 1) / kChunkNodes + 7) / 8;
    const unsigned node_blocks = (unsigned)(8 * chunks_per_xcd);
    hipLaunchKernelGGL(fill_zero_u32_kernel, dim3(blocks_for(n)), dim3(256), 0, stream, indeg, n);
    const hipError_t e = launch_prune(knn, n, d_in, d, pruned, indeg, slot, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(chunk_sums_kernel, dim3((unsigned)chunks), dim3(256), 0, stream, indeg, n, sums);
    hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(1024), 0, stream, sums, chunks);
    hipLaunchKernelGGL(offsets_kernel, dim3((unsigned)chunks), dim3(256), 0, stream, indeg, n, sums, off);
    hipLaunchKernelGGL(in_edges_kernel, dim3(node_blocks), dim3(256), 0, stream, pruned, n, d, d_inv, off, slot, pairs, chunks_per_xcd);
    const int64_t rpx = runs_per_xcd_of(n);
    hipLaunchKernelGGL(graph_merge_kernel, dim3((unsigned)(8 * rpx)), dim3(64), 0, stream, pruned, n, d, off, pairs, out, rpx);
    return hipGetLastError();
}

}  // namespace ann

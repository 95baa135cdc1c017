// Beam search kernel: one wavefront (64 lanes) per query, or a team of two or four (see BeamSearch).
//
// State of a query:
//   * candidate list: 64*LPL packed keys in registers, ascending, striped layout
//     (wave.h: entry e in register e / 64, lane e % 64; LPL is any of 1..8, so a list
//     of 129..192 entries costs three registers per lane, not four).  A packed key is
//     (ordered key << 32) | (id << 1) | expanded, so one unsigned 64-bit compare
//     orders by (key, id) and the expanded mark rides along.
//   * visited set in LDS, two parts.  (a) An exact bitmap over the id ranges of
//     the clusters the query was routed to ("windows"): a K-means partition is
//     stored as contiguous ids, and nearly every node a query scores lies in its
//     routed clusters, so one bit per id of those ranges remembers them all.
//     (b) An open-addressing hash of ids for everything outside the windows.  It
//     is emptied when it fills up and the list's ids are put back.  Forgetting
//     other nodes cannot change the result: the list always holds the itopk best
//     of all nodes scored so far and its worst key never rises, so a forgotten
//     node that is scored again is rejected again; list members are always in the
//     visited set and are never scored twice.  Only the rows gathered grow.
//   * per round: parent ids, surviving neighbour ids and their packed keys in LDS.
//
// One round (Fantasy Sec. 3.2, stage 3: beam width w, out-degree d_g):
//   pick <= width unexpanded list heads -> read their graph rows -> drop ids that
//   are invalid or in the visited table -> gather the surviving rows (G lanes per
//   row, contiguous 16-byte pieces) and compute keys -> sort the new keys (bitonic,
//   in registers) -> merge with the list, keep the itopk smallest.
#pragma once

#include "row_ops.h"

namespace ann {

struct SearchParams {
    const uint8_t* vectors;
    int64_t n;
    int64_t row_stride;
    int32_t row_bytes;
    const int32_t* graph;
    int32_t degree;
    uint32_t degree_inv;  // ceil(2^20 / degree): s / degree == (s * degree_inv) >> 20 for s < 1024
    const uint8_t* queries;
    int64_t nq;
    int64_t q_base, q_count;  // this launch serves queries [q_base, q_base + q_count)
    int32_t k, itopk, width, max_iters;
    int32_t n_entry, entry_mode;
    uint64_t seed;
    const int32_t* route;            // nq * route_c nearest clusters (routed mode)
    const int64_t* cluster_offsets;  // routed mode
    int32_t route_c;
    int32_t n_clusters;   // routed mode: a route id outside [0, n_clusters) names no cluster (no window, no entries)
    int32_t hash_bits;    // visited hash has 1 << hash_bits slots
    int32_t window_bits;  // bits of the visited bitmap (multiple of 32; 0 = none)
    int32_t cap;        // most candidates one round can produce, multiple of 64
    int32_t* out_ids;
    uint32_t* out_dists;
    int32_t* out_counters;  // nq * 4 or null
    const int32_t* order;   // execution order: the launch's i-th query is order[q_base + i]; null = identity
    int64_t q_per_xcd;      // queries of this launch handed to each of the 8 XCDs
};

constexpr uint32_t kEmptySlot = 0xffffffffu;

__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t counter) {
    uint64_t z = seed + (counter + 1) * 0x9E3779B97F4A7C15ull;
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

// True if `id` was not in the hash (and now is).  The hash is never full.
__device__ __forceinline__ bool hash_insert(uint32_t* table, int hash_bits, uint32_t id) {
    const uint32_t mask = (1u << hash_bits) - 1u;
    uint32_t h = (id * 0x9E3779B1u) >> (32 - hash_bits);
    for (;;) {
        const uint32_t old = atomicCAS(&table[h], kEmptySlot, id);
        if (old == kEmptySlot) return true;
        if (old == id) return false;
        h = (h + 1) & mask;
    }
}

// TEAM wavefronts serve one query (one workgroup of 64 * TEAM lanes).  Wavefront 0, the leader, owns
// the candidate list, the visited set and the choice of parents; all wavefronts share the gathers and
// keys of a round, which is where the time of a round with long rows goes when few queries are in
// flight (a wavefront has only so many loads in flight; TEAM of them have TEAM times as many).
template <class Row, int LPL, int CPL, int TEAM = 1>
struct BeamSearch {
    static constexpr int G = Row::G;
    static constexpr int NCH = Row::NCH;
    static constexpr int RPS = 64 / G;                                // rows per gather step
    static constexpr int U = NCH >= 8 ? 1 : (NCH >= 4 ? 2 : (NCH >= 2 ? 3 : 4));  // gather steps in flight
    static constexpr int BR = LPL >= 2 ? 2 : 1;                       // registers of a sort batch
    static constexpr int kInsertMax = 8;                // at most this many new keys are inserted one by one

    const SearchParams& p;
    int lane;
    int wave;        // 0 .. TEAM-1, uniform
    uint32_t* team;  // words the wavefronts of a team exchange (TEAM > 1)
    enum { kTeamM = 0, kTeamDone = 1, kTeamKept = 2, kTeamWorst = 4, kTeamWords = 8 };
    uint32_t* table;
    uint64_t* ckey;
    uint32_t* cid;
    uint32_t* parents;
    uint32_t* wtab;    // per window: first id, ids covered, first bit
    uint32_t* bitmap;  // window_bits / 32 words
    Row row;
    uint64_t L[LPL];
    int n_windows;
    uint32_t w0_lo, w0_size;  // first window: ids [w0_lo, w0_lo + w0_size) are bits 0..
    int n_table;  // ids in the visited hash
    uint64_t worst;  // list entry number itopk-1 (the empty key while the list is not full), kept up to date by merge_all
    int n_dist, n_parents, n_resets;

    // LDS layout, in 32-bit words.  Everything but the hash sits at a compile-time offset, so the
    // addresses fold into the DS instructions' immediate offsets:
    //   [0, kScratchWords)   packed keys of a round (2 words each), then its surviving ids; the same
    //                        words hold a copy of the whole list while a few keys are inserted
    //   parents (64)  window table (32)  team words (8)  bitmap (window_bits / 32)  hash (1 << hash_bits)
    static constexpr int kCap = 64 * CPL;
    static constexpr int kScratchWords = 3 * kCap > 128 * LPL ? 3 * kCap : 128 * LPL;

    __device__ __forceinline__ BeamSearch(const SearchParams& p_, uint32_t* lds, int lane_, int wave_)
        : p(p_), lane(lane_), wave(wave_) {
        ckey = reinterpret_cast<uint64_t*>(lds);
        cid = lds + 2 * kCap;
        parents = lds + kScratchWords;
        wtab = parents + 64;
        team = wtab + 32;
        bitmap = team + kTeamWords;
        table = bitmap + (p.window_bits >> 5);
        n_windows = n_table = n_dist = n_parents = n_resets = 0;
        w0_lo = w0_size = 0;
    }

    // Orders this wavefront's LDS accesses: what it wrote before is what its lanes read after.  A lone
    // wavefront uses the workgroup barrier (which is then no more than that); in a team the leader's own
    // steps must not wait for the other wavefronts, so it only fences (a wavefront's LDS instructions
    // execute in the order they were issued).
    __device__ __forceinline__ void lds_sync() const {
        if constexpr (TEAM == 1) {
            __syncthreads();
        } else {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        }
    }

    __device__ __forceinline__ void clear_table() {
        for (int i = lane; i < (1 << p.hash_bits); i += 64) table[i] = kEmptySlot;
        n_table = 0;
    }

    // Bit of `id` in the visited bitmap, or -1 if no window covers it.  The first window
    // (the nearest cluster, where nearly all ids fall) is kept in registers.
    __device__ __forceinline__ int window_bit(uint32_t id) const {
        const uint32_t rel0 = id - w0_lo;
        int bit = rel0 < w0_size ? (int)rel0 : -1;
        if (n_windows > 1 && bit < 0)
            for (int w = 1; w < n_windows; ++w) {
            const uint32_t rel = id - wtab[3 * w];
            if (rel < wtab[3 * w + 1]) bit = (int)(wtab[3 * w + 2] + rel);
        }
        return bit;
    }

    // 0: seen before; 1: new, remembered in the bitmap; 2: new, remembered in the hash.
    __device__ __forceinline__ int visited_insert(uint32_t id) {
        const int bit = window_bit(id);
        if (bit >= 0) {
            const uint32_t m = 1u << (bit & 31);
            return (atomicOr(&bitmap[bit >> 5], m) & m) ? 0 : 1;
        }
        return hash_insert(table, p.hash_bits, id) ? 2 : 0;
    }

    // Empties the hash and puts back the list's ids that no window covers.
    __device__ __forceinline__ void reset_table() {
        clear_table();
        lds_sync();
#pragma unroll
        for (int r = 0; r < LPL; ++r) {
            const uint32_t id = (uint32_t)L[r] >> 1;
            const bool put = L[r] != kInfKey && window_bit(id) < 0;
            if (put) hash_insert(table, p.hash_bits, id);
            n_table += __builtin_popcountll(__ballot(put));
        }
        ++n_resets;
    }

    // Candidate ids held one per lane: keep the unseen ones, packed into cid[0..m).
    __device__ __forceinline__ void filter_into(int32_t id, bool valid, int& m) {
        const int how = (valid && (uint32_t)id < (uint32_t)p.n) ? visited_insert((uint32_t)id) : 0;  // n < 2^31: a negative id fails too
        const uint64_t b = __ballot(how != 0);
        if (how != 0) cid[rank_below(b, m)] = (uint32_t)id;
        m += __builtin_popcountll(b);
        n_table += __builtin_popcountll(__ballot(how == 2));
    }

    // The list entry number itopk-1: a new key that is not below it cannot enter the list
    // (the empty key while the list is not full).
    __device__ __forceinline__ uint64_t list_worst() const {
        const int e = p.itopk - 1;
        // lane e % 64 of every register is read and the register chosen among the scalars: choosing the
        // register first would index the list by a run-time value and push the whole search state into
        // scratch memory
        uint64_t w = kInfKey;
#pragma unroll
        for (int r = 0; r < LPL; ++r) {
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)L[r], e & 63);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(L[r] >> 32), e & 63);
            if ((e >> 6) == r) w = ((uint64_t)hi << 32) | lo;
        }
        return w;
    }

    // Gathers rows cid[0..m) and writes the packed keys that can enter the list to
    // ckey[0..returned count).
    __device__ __forceinline__ int score(int m) { return row.full ? score_rows<true>(m) : score_rows<false>(m); }

    // FULL: the row fills every piece of every lane, so the row buffers need no clearing (RowOps::blank_row); else
    // they are zeroed once and a piece this lane does not load keeps its zeros (RowOps::reload_row).
    template <bool FULL>
    __device__ __forceinline__ int score_rows(int m) {
        const int grp = lane / G;
        const uint64_t worst = this->worst;
        // the host keeps the stride below 2^31, so a row's address is one 32 x 32 -> 64 bit multiply-add
        const uint8_t* const piece0 = row.lane_piece(p.vectors);
        const uint32_t stride = (uint32_t)p.row_stride;
        int kept = 0;
        u32x4 x[U][NCH];
        if constexpr (!FULL) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < NCH; ++c) x[u][c] = u32x4{0, 0, 0, 0};
        }
        for (int j0 = 0; j0 < m; j0 += RPS * U) {
            uint32_t id[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (j0 + u * RPS >= m) break;  // whole step beyond the last row
                const int j = j0 + u * RPS + grp;
                const bool live = j < m;
                id[u] = live ? cid[j] : 0u;
                if constexpr (FULL) {
                    row.blank_row(x[u]);
                    row.load_full_row(x[u], piece0 + (uint64_t)id[u] * stride, live);
                } else {
                    row.reload_row(x[u], piece0 + (uint64_t)id[u] * stride, live);
                }
            }
            // Every lane of a group ends up with the group's key, so lane u of a group takes the key of step u:
            // one filter, one ballot and one store then serve all U steps (G >= U for every row variant).
            static_assert(G >= U, "one lane of a group per gather step");
            uint64_t mine = kInfKey;  // is not below `worst`, whatever that is
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (j0 + u * RPS >= m) break;
                const int j = j0 + u * RPS + grp;
                const uint32_t okey = row.key(x[u], lane);
                const uint64_t packed = ((uint64_t)okey << 32) | (uint64_t)(id[u] << 1);  // ids are below 2^31
                mine = (row.lg == u && j < m) ? packed : mine;
            }
            const bool keep = mine < worst;
            const uint64_t b = __ballot(keep);
            if (keep) ckey[rank_below(b, kept)] = mine;
            kept += __builtin_popcountll(b);
        }
        n_dist += m;
        return kept;
    }

    // The same for a team: wavefront w takes the blocks of RPS * U rows number w, w + TEAM, ...  The keys
    // that can enter the list are appended to ckey through a counter the team shares; their order in ckey
    // is whatever the atomics give, which the merge does not depend on (it orders them).
    __device__ __forceinline__ void score_team(int m) {
        if (row.full) score_team_rows<true>(m);
        else score_team_rows<false>(m);
    }

    template <bool FULL>
    __device__ __forceinline__ void score_team_rows(int m) {
        const int grp = lane / G;
        const uint64_t worst = this->worst;
        const uint8_t* const piece0 = row.lane_piece(p.vectors);
        const uint32_t stride = (uint32_t)p.row_stride;
        u32x4 x[U][NCH];
        if constexpr (!FULL) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < NCH; ++c) x[u][c] = u32x4{0, 0, 0, 0};
        }
        for (int j0 = wave * (RPS * U); j0 < m; j0 += RPS * U * TEAM) {
            uint32_t id[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (j0 + u * RPS >= m) break;
                const int j = j0 + u * RPS + grp;
                const bool live = j < m;
                id[u] = live ? cid[j] : 0u;
                if constexpr (FULL) {
                    row.blank_row(x[u]);
                    row.load_full_row(x[u], piece0 + (uint64_t)id[u] * stride, live);
                } else {
                    row.reload_row(x[u], piece0 + (uint64_t)id[u] * stride, live);
                }
            }
            uint64_t packed[U], b[U];
            bool keep[U];
            int cnt = 0;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                b[u] = 0;
                keep[u] = false;
                packed[u] = 0;
                if (j0 + u * RPS < m) {
                    const int j = j0 + u * RPS + grp;
                    const uint32_t okey = row.key(x[u], lane);
                    packed[u] = ((uint64_t)okey << 32) | (uint64_t)(id[u] << 1);
                    keep[u] = j < m && row.lg == 0 && packed[u] < worst;
                    b[u] = __ballot(keep[u]);
                    cnt += __builtin_popcountll(b[u]);
                }
            }
            if (cnt > 0) {  // uniform
                int base = 0;
                if (lane == 0) base = (int)atomicAdd(&team[kTeamKept], (uint32_t)cnt);
                base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (keep[u]) ckey[rank_below(b[u], base)] = packed[u];
                    base += __builtin_popcountll(b[u]);
                }
            }
        }
    }

    // list <- itopk smallest of list U ckey[base .. base + 64*R), R registers per lane;
    // KMAX >= the number of real keys in the batch (a power of two, at most 64*R).
    template <int R, int KMAX>
    __device__ __forceinline__ void merge_batch(int base, int m) {
        // The networks below test lane bits (dozens of per-lane conditions).  They do not change from
        // round to round, so the compiler would compute them once, keep them as 64-bit scalar masks across
        // the whole search loop and spill the loop's own scalars to make room; an opaque copy of the lane
        // number makes it compute them here, on this rarely taken path.
        int lane = this->lane;
        asm volatile("" : "+v"(lane));
        uint64_t c[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int j = base + lane * R + r;
            c[r] = j < m ? ckey[j] : kInfKey;
        }
        bitonic_sort_runs<R, KMAX>(c, lane);
        lds_sync();  // all reads of this batch done before it is overwritten
#pragma unroll
        for (int r = 0; r < R; ++r) ckey[base + lane * R + r] = c[r];
        lds_sync();
        // smallest 64*LPL of (list, sorted batch): list entry e against batch element 64*LPL-1-e, which
        // leaves one run that rises and then falls.  Register r holds entries 64r .. 64r+63, so whole
        // registers either have a partner in the batch or not.
#pragma unroll
        for (int r = 0; r < LPL; ++r)
            if (LPL - r <= R) {  // known at compile time
                const uint64_t o = ckey[base + 64 * LPL - 1 - (r * 64 + lane)];
                L[r] = o < L[r] ? o : L[r];
            }
        striped_merge<LPL>(L, lane);
#pragma unroll
        for (int r = 0; r < LPL; ++r)
            if (r * 64 + lane >= p.itopk) L[r] = kInfKey;
        lds_sync();
    }

    // list <- itopk smallest of list U ckey[0..s) for a handful of keys (1 <= s <= 64, meant for
    // s <= 8), without sorting: an entry moves up by the number of new keys below it, a new key
    // lands at (entries below it) + (new keys below it); the moves go through a copy in LDS.
    __device__ __forceinline__ void insert_few(int s) {
        uint64_t* lcopy = ckey;
        const uint64_t mine = lane < s ? ckey[lane] : kInfKey;
        lds_sync();  // the new keys are in registers; their words may now be overwritten
        int cnt[LPL];
#pragma unroll
        for (int r = 0; r < LPL; ++r) cnt[r] = 0;
        int rank = 0, pos = 0;
        for (int j = 0; j < s; ++j) {
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)mine, j);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(mine >> 32), j);
            const uint64_t c = ((uint64_t)hi << 32) | lo;
            int below = 64 * LPL;
#pragma unroll
            for (int r = 0; r < LPL; ++r) {
                const bool lt = c < L[r];
                cnt[r] += lt ? 1 : 0;
                below -= __builtin_popcountll(__ballot(lt));
            }
            rank += c < mine ? 1 : 0;
            pos = lane == j ? below : pos;
        }
        // Every key goes to its place without a test: a place may lie up to s <= kInsertMax entries beyond
        // the copy (entries pushed off the end), which is still inside this round's scratch or in the
        // first words of `parents` (32 keys wide), dead until the next round rewrites them.
        // Whatever landed at or beyond itopk is then overwritten with the empty key.
        static_assert(kInsertMax <= 32, "trash slots beyond the list copy");
#pragma unroll
        for (int r = 0; r < LPL; ++r) lcopy[r * 64 + lane + cnt[r]] = L[r];
        if (lane < s) lcopy[pos + rank] = mine;
        lds_sync();
        for (int i = p.itopk + lane; i < 64 * LPL; i += 64) lcopy[i] = kInfKey;
        lds_sync();
#pragma unroll
        for (int r = 0; r < LPL; ++r) L[r] = lcopy[r * 64 + lane];
        worst = lcopy[p.itopk - 1];  // one broadcast read of the sorted copy
        lds_sync();
    }

    __device__ __forceinline__ void merge_all(int m) {
        if (m >= 1 && m <= kInsertMax) {
            insert_few(m);
            return;
        }
        int base = 0;
        if constexpr (BR == 2) {
            for (; m - base > 64; base += 128) merge_batch<2, 128>(base, m);
        }
        if (m - base > 32) {
            for (; base < m; base += 64) merge_batch<1, 64>(base, m);
        } else if (m - base > 16) {
            merge_batch<1, 32>(base, m);
        } else if (m - base > 0) {
            merge_batch<1, 16>(base, m);
        }
        if (m > 0) worst = list_worst();
    }

    // The first list of a query: the list is still empty, so the sorted keys of the entries are the list
    // (register 0 of the striped layout is the blocked layout of 64 keys); no merge network.
    __device__ __forceinline__ void first_list(int m) {
        if (m > 64) {
            merge_all(m);
            return;
        }
        int lane = this->lane;
        asm volatile("" : "+v"(lane));  // see merge_batch
        uint64_t c[1] = {lane < m ? ckey[lane] : kInfKey};
        if (m > 32) bitonic_sort_runs<1, 64>(c, lane);
        else bitonic_sort_runs<1, 32>(c, lane);
        L[0] = lane < p.itopk ? c[0] : kInfKey;
        lds_sync();
        if (m > 0) worst = list_worst();
    }

    // Empty list and visited set, the windows of the routed clusters, and the entry ids (duplicates collapse
    // in the visited set) in cid[0..returned count).
    __device__ __forceinline__ int start(int64_t qi) {
#pragma unroll
        for (int r = 0; r < LPL; ++r) L[r] = kInfKey;
        worst = kInfKey;
        clear_table();
        for (int i = lane; i < (p.window_bits >> 5); i += 64) bitmap[i] = 0u;
        if (p.entry_mode == 1 && p.window_bits > 0) {
            // one window per routed cluster, in routing order, until the bitmap is used up
            uint32_t bit = 0;
            for (int w = 0; w < p.route_c; ++w) {
                const int32_t c = p.route[qi * p.route_c + w];
                const bool known = (uint32_t)c < (uint32_t)p.n_clusters;
                const int64_t lo = known ? p.cluster_offsets[c] : 0, hi = known ? p.cluster_offsets[c + 1] : 0;
                const uint32_t room = (uint32_t)p.window_bits - bit;
                const uint32_t size = hi <= lo ? 0u : (uint64_t)(hi - lo) < room ? (uint32_t)(hi - lo) : room;
                if (lane == 0) {
                    wtab[3 * w] = (uint32_t)lo;
                    wtab[3 * w + 1] = size;
                    wtab[3 * w + 2] = bit;
                }
                if (w == 0) {
                    w0_lo = (uint32_t)lo;
                    w0_size = size;
                }
                bit += size;
            }
            n_windows = p.route_c;
        }
        lds_sync();
        int m = 0;
#pragma unroll
        for (int t = 0; t < CPL; ++t) {
            const int j = t * 64 + lane;
            const bool valid = j < p.n_entry;
            int32_t e = -1;
            if (valid) {
                const uint64_t z = splitmix64_at(p.seed, (uint64_t)qi * (uint64_t)p.n_entry + (uint64_t)j);
                if (p.entry_mode == 0) {
                    e = (int32_t)(z % (uint64_t)p.n);
                } else {
                    const int32_t c = p.route[qi * p.route_c + (j % p.route_c)];
                    const bool known = (uint32_t)c < (uint32_t)p.n_clusters;
                    const int64_t lo = known ? p.cluster_offsets[c] : 0, hi = known ? p.cluster_offsets[c + 1] : 0;
                    if (hi > lo) e = (int32_t)(lo + (int64_t)(z % (uint64_t)(hi - lo)));
                }
            }
            filter_into(e, valid, m);
        }
        return m;
    }

    // One round up to the gathers: marks the first <= width unexpanded list entries as expanded, reads their
    // graph rows and leaves the ids that were never scored in cid[0..returned count); -1 if nothing is
    // left to expand.
    __device__ __forceinline__ int expand() {
        // Register r holds entries 64r .. 64r+63, so the registers are walked in order and the walk stops
        // once `width` parents are found.
        int total = 0;
#pragma unroll
        for (int r = 0; r < LPL; ++r) {
            if (total < p.width) {  // uniform
                uint32_t ex;  // taken in the 32-bit low word (the compiler otherwise widens the test to the whole key)
                asm("v_and_b32 %0, 1, %1" : "=v"(ex) : "v"((uint32_t)L[r]));
                const bool un = ex == 0;
                const uint64_t b = __ballot(un);
                const int rank = rank_below(b, total);
                const bool take = un && rank < p.width;
                if (take) parents[rank] = (uint32_t)L[r] >> 1;
                L[r] |= (uint64_t)(take ? 1u : 0u);
                total += __builtin_popcountll(b);
            }
        }
        if (total == 0) return -1;
        const int np = total < p.width ? total : p.width;
        n_parents += np;
        if (n_table + np * p.degree > ((3 << p.hash_bits) >> 2)) reset_table();
        lds_sync();

        // neighbour ids of the parents, 64 per step, all loads issued first
        const int nref = np * p.degree;
        int32_t nb[CPL];
#pragma unroll
        for (int t = 0; t < CPL; ++t) {
            const int s = t * 64 + lane;
            nb[t] = -1;
            if (s < nref) {
                const int pi = (int)(((uint32_t)s * p.degree_inv) >> 20);
                // unsigned 32 x 32 -> 64 bit: one multiply-add
                nb[t] = p.graph[(uint64_t)parents[pi] * (uint32_t)p.degree + (uint32_t)(s - pi * p.degree)];
            }
        }
        int m = 0;
#pragma unroll
        for (int t = 0; t < CPL; ++t) filter_into(nb[t], t * 64 + lane < nref, m);
        return m;
    }

    // First k list entries and the counters.
    __device__ __forceinline__ void finish(int64_t qi, int iters) {
#pragma unroll
        for (int r = 0; r < LPL; ++r) {
            const int e = r * 64 + lane;
            if (e < p.k) {
                const bool have = L[r] != kInfKey;
                p.out_ids[qi * p.k + e] = have ? (int32_t)((uint32_t)L[r] >> 1) : -1;
                p.out_dists[qi * p.k + e] = have ? Row::key_to_output((uint32_t)(L[r] >> 32)) : Row::pad_output();
            }
        }
        if (p.out_counters && lane == 0) {
            int32_t* c = p.out_counters + qi * 4;
            c[0] = iters;
            c[1] = n_dist;
            c[2] = n_parents;
            c[3] = n_resets;
        }
    }

    __device__ __forceinline__ void run(int64_t qi) {
        row.load_query(p.queries + qi * (int64_t)p.row_bytes, p.row_bytes, lane);
        if constexpr (TEAM > 1) {
            run_team(qi);
            return;
        }
        int m = start(qi);
        lds_sync();
        m = score(m);
        lds_sync();
        first_list(m);
        int iters = 0;
        for (; iters < p.max_iters; ++iters) {
            m = expand();
            if (m < 0) break;
            lds_sync();
            m = score(m);
            lds_sync();
            merge_all(m);
        }
        finish(qi, iters);
    }

    // The leader tells the team what the next scoring step works on.
    __device__ __forceinline__ void publish(int m, int done) {
        if (lane == 0) {
            team[kTeamM] = (uint32_t)m;
            team[kTeamDone] = (uint32_t)done;
            team[kTeamKept] = 0u;
            team[kTeamWorst] = (uint32_t)worst;
            team[kTeamWorst + 1] = (uint32_t)(worst >> 32);
        }
    }

    // Two workgroup barriers per round: before the scoring step (the leader has left the round's ids, their
    // count and the list's worst key in LDS) and after it (every wavefront's keys are in ckey).  Between the
    // second barrier and the next first one only the leader works: merge, parents, graph rows, visited filter.
    // Every wavefront leaves the loop in the same round, on the flag the leader publishes.
    __device__ __forceinline__ void run_team(int64_t qi) {
        const bool leader = wave == 0;
        int iters = 0;
        if (leader) {
            const int m = start(qi);
            lds_sync();
            publish(m, 0);
        }
        for (;;) {
            __syncthreads();
            const int m = (int)team[kTeamM];
            if (team[kTeamDone] != 0u) break;
            worst = ((uint64_t)team[kTeamWorst + 1] << 32) | team[kTeamWorst];
            score_team(m);
            __syncthreads();
            if (leader) {
                n_dist += m;
                merge_all((int)team[kTeamKept]);
                int next = -1;
                if (iters < p.max_iters) next = expand();
                if (next >= 0) ++iters;
                lds_sync();
                publish(next < 0 ? 0 : next, next < 0 ? 1 : 0);
            }
        }
        if (leader) finish(qi, iters);
    }
};

// Workgroup b runs on XCD b % 8 (round-robin dispatch), so consecutive queries are
// kept on one XCD and its L2: query = (b % 8) * q_per_xcd + b / 8.
// The small uint8 variants (rows of at most 256 bytes) are asked to fit 7 wavefronts per SIMD (72 vector registers; 8 would need spills):
// with about 5.5 KB of LDS per query that is also what a compute unit's LDS holds, 28 queries in flight.
template <class Row, int LPL, int CPL, int TEAM>
__global__ void __launch_bounds__(64 * TEAM, (TEAM == 1 && Row::kDtype == kU8 && Row::G * Row::NCH <= 16 && LPL <= 4 && CPL <= 2) ? 7 : 1)
    beam_search_kernel(const SearchParams p) {
    extern __shared__ uint32_t lds[];
    const int64_t b = blockIdx.x;
    const int64_t local = (b & 7) * p.q_per_xcd + (b >> 3);
    if (local >= p.q_count) return;  // the whole workgroup
    BeamSearch<Row, LPL, CPL, TEAM> s(p, lds, lane_id(), TEAM == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)));
    s.run(p.order ? (int64_t)p.order[p.q_base + local] : p.q_base + local);
}

}  // namespace ann

// Replay kernel, block-table formulation (any trace).
//
// The cache of a replica is a hashed table key -> stamp of the last touch (stamp = request * stride + (stride - 1 -
// position): within a request the root is the newest), and "cached" means "stamp not below the replica's eviction
// threshold".  Least-recently-used eviction only raises that threshold: the cursor behind it walks the replica's
// log of routed requests, oldest first, deepest block first, and a logged touch still counts iff the table holds
// exactly its stamp.  Nothing about the trace is assumed (the same id may follow different ids in different
// requests), so the match probes block by block.
//
// A replay is run by two wavefronts of one workgroup.  The queue wavefront is the segment formulation's, unchanged:
// service slots, load signal (Eq. 2), service step, per-request outputs, and with them the online tuner, the
// engine model and the epochs of the proxy's round-trip estimates.  The cache wavefront here does per request:
// match against every replica's table; meet (A: the queue terms are there); score (Eq. 3) or apply the baseline
// policy, lowest-index minimum, announce the choice; meet (B); table update and eviction on the chosen replica.
// Both wavefronts execute exactly two barriers per request, whatever the data.
//
// The proxy's own index of a replica (Sec. 7: the proxy does not see replica-side eviction) is a second LRU over
// the same touches with a capacity of its own.  Touches give an entry the same stamp in both, so the index is the
// same table read against a second threshold, with a cursor of its own on the same log.
#pragma once
#include "device_common.h"
#include "internal.h"
#include "replay_segments.h"

namespace gorgo {

// One cache-table slot.  key 0 = never used (then stamp = -1).  An entry is held by an LRU iff stamp >= that
// LRU's threshold; entries below every threshold are garbage whose slots can be taken over by inserts.
struct Slot {
    uint64_t key;
    int64_t stamp;
};

struct BlockArgs {
    SegArgs q;               // what the queue wavefront reads, and the model, weights and policy inputs
    const int64_t* blk_off;  // [N+1]
    const uint32_t* key;     // [T] dense block keys, 0 never occurs
    const uint8_t* first;    // [T] 1 where the key occurs for the first time within its request
    Slot* tables;            // [P][R][cap]
    Slot* spare;             // [P][cap] scratch of the compaction
    uint8_t* routed;         // [P][N] the cache wavefront's log of choices (what its eviction cursors walk)
    int64_t cap;             // slots per table, a power of two
    int32_t cap_log2;
};

// per replica: two thresholds (int64), then live x2, cursor request x2, cursor position x2, used slots (int32)
__host__ __device__ inline size_t replay_blocks_state_bytes(int R) { return (size_t)R * (2 * 8 + 7 * 4); }
__host__ __device__ inline size_t replay_blocks_lds_bytes(int R, int B, int window) {
    return ((replay_segments_lds_bytes(R, B, window) + 15) & ~(size_t)15) + replay_blocks_state_bytes(R);
}

__device__ __forceinline__ bool cas_stamp(int64_t* p, int64_t expected, int64_t desired) {
    return __hip_atomic_compare_exchange_strong(p, &expected, desired, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ uint64_t home_slot(uint64_t key, int cap_log2) {
    return (key * 0x9E3779B97F4A7C15ull) >> (64 - cap_log2);
}

// Physical lookup: slot index of `key`, or -1 when the probe sequence reaches a never-used slot.
__device__ __forceinline__ int64_t find_slot(const Slot* tab, uint64_t key, uint64_t mask, int cap_log2) {
    uint64_t h = home_slot(key, cap_log2);
    for (;;) {
        uint64_t k = ld(&tab[h].key);
        if (k == key) return (int64_t)h;
        if (k == 0) return -1;
        h = (h + 1) & mask;
    }
}

// Stamp of `key` in the table, -1 (below every threshold) when it is not there.
__device__ __forceinline__ int64_t stamp_of(const Slot* tab, uint64_t key, uint64_t mask, int cap_log2) {
    const int64_t s = find_slot(tab, key, mask, cap_log2);
    return s >= 0 ? ld(&tab[s].stamp) : -1;
}

// Takes over the first never-used or garbage slot of the probe sequence (stamp below `tau`, the lowest threshold).
// Returns true when a never-used slot was consumed.  Only called for keys known to be physically absent, by lanes
// with distinct keys.
__device__ __forceinline__ bool insert_new(Slot* tab, uint64_t key, int64_t stamp, int64_t tau, uint64_t mask,
                                           int cap_log2) {
    uint64_t h = home_slot(key, cap_log2);
    for (;;) {
        int64_t s = ld(&tab[h].stamp);
        if (s < tau && cas_stamp(&tab[h].stamp, s, stamp)) {
            st(&tab[h].key, key);
            return s == -1;
        }
        h = (h + 1) & mask;
    }
}

__global__ void __launch_bounds__(256) fill_slots(Slot* s, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        s[i].key = 0;
        s[i].stamp = -1;
    }
}

// What the lanes of this wavefront have written to global memory is there for its other lanes to read (the cache
// wavefront is the only one that touches the tables and the log of choices).
__device__ __forceinline__ void wave_settle() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    __builtin_amdgcn_wave_barrier();
}

// Cache wavefront of a replay over block tables.  Lane = replica for the first-block probe, the scores and the
// minimum; lane = block of the request for the prefix match, the table update and the eviction walk.
template <int MODE, bool PROXY>
__device__ __forceinline__ void block_cache_wave(const BlockArgs& b, int p, int lane, unsigned char* state,
                                                 Handover* comm) {
    constexpr bool ONLINE = MODE == MODE_ONLINE;
    constexpr bool SCORED = MODE == MODE_COST_MODEL || MODE == MODE_ONLINE;
    const SegArgs& a = b.q;
    const int R = a.R;
    const int64_t N = a.N;
    const bool in = lane < R;
    const uint64_t mask = (uint64_t)b.cap - 1;
    const int cap_log2 = b.cap_log2;
    // the proxy's own index: a second LRU (capacity index_blocks, 0 = it never forgets) over the same touches
    const bool two = PROXY && a.index_blocks >= 0;
    const int64_t C1 = a.C, C2 = two ? a.index_blocks : 0;

    int64_t* const tau1 = reinterpret_cast<int64_t*>(state);      // [R] the cache's eviction threshold
    int64_t* const tau2 = tau1 + R;                               // [R] the index's
    int32_t* const live1 = reinterpret_cast<int32_t*>(tau2 + R);  // [R] blocks the cache holds
    int32_t* const live2 = live1 + R;                             // [R] blocks the index holds
    int32_t* const cur_r1 = live2 + R;                            // [R] eviction cursors: request ...
    int32_t* const cur_r2 = cur_r1 + R;
    int32_t* const cur_k1 = cur_r2 + R;                           // [R] ... and position (blocks >= cur_k are gone)
    int32_t* const cur_k2 = cur_k1 + R;
    int32_t* const used = cur_k2 + R;                             // [R] slots ever used since the last compaction
    for (int i = lane; i < R; i += WAVE) {
        tau1[i] = tau2[i] = 0;
        live1[i] = live2[i] = 0;
        cur_r1[i] = cur_r2[i] = -1;
        cur_k1[i] = cur_k2[i] = 0;
        used[i] = 0;
    }
    wave_sync();

    const double w_rtt = a.params[3 * (size_t)p + 0];             // (with the online tuner the weights come with
    const double w_prefill = a.params[3 * (size_t)p + 1];         // the queue terms instead)
    const double my_rtt = !PROXY && in ? a.rtt[lane] : 0.0;       // (proxy variants: comes with the queue terms)
    const uint64_t seed = MODE == MODE_RANDOM ? a.seeds[p] : 0;

    Slot* const tables = b.tables + (size_t)p * R * b.cap;
    Slot* const spare = b.spare + (size_t)p * b.cap;
    uint8_t* const routed = b.routed + (size_t)p * N;
    const int64_t rebuild_at = b.cap - b.cap / 8;

    meet(false);        // (the queue wavefront has set itself up)
    for (int64_t r = 0; r < N; ++r) {
        const int64_t off = b.blk_off[r];
        const int n = (int)(b.blk_off[r + 1] - off);
        const int L = a.in_len[r];

        // ---- prefix match: first block on every replica, then the whole list on the replicas that hold it; against
        // the cache's threshold and, with an index, against the index's as well
        int my_m = 0, my_seen = 0;
        {
            bool has0 = false;
            if (n > 0 && in) {
                const int64_t t1 = tau1[lane], t2 = two ? tau2[lane] : t1;
                has0 = stamp_of(tables + (size_t)lane * b.cap, b.key[off], mask, cap_log2) >= (t2 < t1 ? t2 : t1);
            }
            unsigned long long holders = ballot(has0);
            while (holders) {
                const int i = __builtin_ctzll(holders);
                holders &= holders - 1;
                const Slot* tab = tables + (size_t)i * b.cap;
                const int64_t t1 = tau1[i], t2 = two ? tau2[i] : t1;
                int m1 = 0, m2 = 0;
                bool open1 = true, open2 = two;
                for (int base = 0; base < n && (open1 || open2); base += WAVE) {
                    const int k = base + lane;
                    const int64_t s = k < n ? stamp_of(tab, b.key[off + k], mask, cap_log2) : -1;
                    const int width = n - base < WAVE ? n - base : WAVE;
                    const unsigned long long want = width == WAVE ? ~0ull : ((1ull << width) - 1);
                    const unsigned long long got1 = ballot(k < n && s >= t1), got2 = ballot(k < n && s >= t2);
                    if (open1) {
                        if (got1 == want) m1 += width;
                        else {
                            m1 += __builtin_ctzll(~got1);
                            open1 = false;
                        }
                    }
                    if (open2) {
                        if (got2 == want) m2 += width;
                        else {
                            m2 += __builtin_ctzll(~got2);
                            open2 = false;
                        }
                    }
                }
                if (lane == i) {
                    my_m = m1;
                    my_seen = m2;
                }
            }
        }
        // uncached tokens, really and as Eq. 3 sees them (block_tokens * blocks fits: below 2^15 and 2^16)
        int hit_tok = a.block_tokens * my_m;
        hit_tok = hit_tok > L ? L : hit_tok;
        const int my_u = L - hit_tok;
        int seen_tok = a.block_tokens * (two ? my_seen : my_m);
        seen_tok = seen_tok > L ? L : seen_tok;
        const int my_u_seen = L - seen_tok;
        // the replica a baseline policy dictates (Sec. 4): hash of the first block, or a counter-based draw
        int target = 0;
        if (MODE == MODE_AFFINITY) target = n > 0 ? spread(a.first_hash[r], R) : 0;
        else if (MODE == MODE_RANDOM)
            target = spread(philox4x32_10_first((uint32_t)r, (uint32_t)((uint64_t)r >> 32), (uint32_t)seed,
                                                (uint32_t)(seed >> 32)), R);

        meet(true);                                                  // A(r): the queue terms of r are there
        // ---- score (Eq. 3: rtt and prefill terms here, the queue term from the queue wavefront), lowest-index minimum
        const double sq = SCORED || MODE == MODE_LEAST_REQUEST ? comm->sq[lane] : 0.0;
        double rtt_now = my_rtt, now_rtt = w_rtt, now_prefill = w_prefill;
        if (PROXY) rtt_now = comm->rtt[lane];
        if (ONLINE) {
            now_rtt = comm->w[0];
            now_prefill = comm->w[1];
        }
        double my_score;
        if (SCORED) {
            const double pf = a.a_pf * (double)my_u_seen;
            const double s_rtt = now_rtt * rtt_now;
            const double s_pf = now_prefill * pf;
            const double rtt_and_prefill = s_rtt + s_pf;
            my_score = rtt_and_prefill + sq;
        } else if (MODE == MODE_LEAST_REQUEST) {
            my_score = sq;                      // requests in flight
        } else {
            my_score = lane == target ? 0.0 : 1.0;
        }
        const int best = argmin_lanes(my_score, in);
        const int m_best = __builtin_amdgcn_readlane(my_m, best);
        const int seen_best = two ? __builtin_amdgcn_readlane(my_seen, best) : m_best;
        const unsigned u_best = (unsigned)__builtin_amdgcn_readlane(my_u, best);
        if (lane == 0) {
            comm->choice = ((unsigned long long)((unsigned)best | ((unsigned)m_best << 8)) << 32) | u_best;
            if (PROXY) comm->seen = seen_best;
            st(&routed[r], (uint8_t)best);
        }
        meet(true);                                                  // B(r): the choice is there

        // ---- update on the chosen replica
        Slot* const tab = tables + (size_t)best * b.cap;
        if ((int64_t)used[best] + n > rebuild_at) {
            // compact: keep what some LRU still holds, so that never-used slots exist again
            const int64_t t1 = tau1[best], t2 = two ? tau2[best] : t1;
            const int64_t keep_from = t2 < t1 ? t2 : t1;
            int64_t kept = 0;
            for (int64_t base = 0; base < b.cap; base += WAVE) {
                const uint64_t k = ld(&tab[base + lane].key);
                const int64_t s = ld(&tab[base + lane].stamp);
                const bool keep = k != 0 && s >= keep_from;
                const unsigned long long mk = ballot(keep);
                if (keep) {
                    const int64_t pos = kept + __builtin_popcountll(mk & ((1ull << lane) - 1));
                    st(&spare[pos].key, k);
                    st(&spare[pos].stamp, s);
                }
                kept += __builtin_popcountll(mk);
            }
            wave_settle();
            for (int64_t base = 0; base < b.cap; base += WAVE) {
                st(&tab[base + lane].key, (uint64_t)0);
                st(&tab[base + lane].stamp, (int64_t)-1);
            }
            wave_settle();
            for (int64_t base = 0; base < kept; base += WAVE) {
                if (base + lane < kept)
                    insert_new(tab, ld(&spare[base + lane].key), ld(&spare[base + lane].stamp), 0, mask, cap_log2);
                wave_settle();
            }
            if (lane == 0) used[best] = (int32_t)kept;
            wave_sync();
        }
        {
            // every block of the request becomes (or stays) held, with this request's stamp
            const int64_t t1 = tau1[best], t2 = two ? tau2[best] : t1;
            const int64_t garbage_below = t2 < t1 ? t2 : t1;
            int add1 = 0, add2 = 0, add_used = 0;
            for (int base = 0; base < n; base += WAVE) {
                const int k = base + lane;
                const bool mine = k < n && b.first[off + k] != 0;
                const uint64_t key = mine ? b.key[off + k] : 0;
                const int64_t stamp = r * STAMP_STRIDE + (STAMP_STRIDE - 1 - k);
                int64_t slot = -1, before = -1;
                if (mine) {
                    slot = find_slot(tab, key, mask, cap_log2);
                    if (slot >= 0) {
                        before = ld(&tab[slot].stamp);
                        st(&tab[slot].stamp, stamp);          // touch, or revive an evicted entry in place
                    }
                }
                wave_settle();
                bool took_fresh = false;
                if (mine && slot < 0) took_fresh = insert_new(tab, key, stamp, garbage_below, mask, cap_log2);
                wave_settle();
                add1 += __builtin_popcountll(ballot(mine && before < t1));
                add2 += __builtin_popcountll(ballot(mine && before < t2));
                add_used += __builtin_popcountll(ballot(took_fresh));
            }
            if (lane == 0) {
                live1[best] += add1;
                live2[best] += add2;
                used[best] += add_used;
            }
            wave_sync();
        }

        // ---- eviction: advance the threshold past the least recently used blocks until the LRU fits.  The log of
        // (request, position) touches on this replica is the log of choices, walked from the oldest request routed
        // here; a logged touch still counts iff the table holds exactly its stamp.
        auto evict = [&](int64_t C, int64_t* tau, int32_t* live, int32_t* cur_r, int32_t* cur_k) {
            if (C <= 0 || live[best] <= C) return;
            int E = (int)(live[best] - C);
            int cr = cur_r[best], ck = cur_k[best];
            while (E > 0) {
                if (ck == 0) {
                    const int64_t x = next_routed(routed, cr, r, best, lane);
                    if (x >= r) break;          // cannot happen while E > 0; bounds the loop regardless
                    cr = (int)x;
                    ck = (int)(b.blk_off[x + 1] - b.blk_off[x]);
                    continue;
                }
                const int64_t ooff = b.blk_off[cr];
                const int k = ck - 1 - lane;               // lane order = eviction order (deepest first)
                bool alive = false;
                if (k >= 0 && b.first[ooff + k] != 0)
                    alive = stamp_of(tab, b.key[ooff + k], mask, cap_log2) ==
                            (int64_t)cr * STAMP_STRIDE + (STAMP_STRIDE - 1 - k);
                const unsigned long long mk = ballot(alive);
                const int cnt = __builtin_popcountll(mk);
                if (cnt <= E) {
                    E -= cnt;
                    ck = ck > WAVE ? ck - WAVE : 0;
                } else {
                    const int rank = __builtin_popcountll(mk & ((1ull << lane) - 1));
                    const unsigned long long last = ballot(alive && rank == E - 1);
                    const int j = __builtin_ctzll(last);
                    ck = ck - 1 - j;
                    E = 0;
                }
            }
            if (lane == 0) {
                cur_r[best] = cr;
                cur_k[best] = ck;
                tau[best] = (int64_t)cr * STAMP_STRIDE + (STAMP_STRIDE - ck);
                live[best] = (int32_t)C + E;
            }
            wave_sync();
        };
        evict(C1, tau1, live1, cur_r1, cur_k1);
        if (two) evict(C2, tau2, live2, cur_r2, cur_k2);
        wave_settle();
    }
}

template <int MODE, bool ENGINE, bool PROXY>
__global__ void __launch_bounds__(SEG_THREADS) replay_blocks_kernel(BlockArgs b) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ __align__(16) Handover comm;
    const int lane = threadIdx.x & (WAVE - 1);
    const int p = blockIdx.x;
    if (threadIdx.x == 0) {
        comm.w[0] = b.q.params[3 * (size_t)p + 0];
        comm.w[1] = b.q.params[3 * (size_t)p + 1];
    }
    __syncthreads();
    if (threadIdx.x >= WAVE) {
        queue_wave<MODE, ENGINE, PROXY, false, false>(b.q, p, lane, lds_raw, &comm);
    } else if (b.q.N > 0) {
        unsigned char* const state =
            lds_raw + ((replay_segments_lds_bytes(b.q.R, b.q.B, MODE == MODE_ONLINE ? b.q.window : 0) + 15) & ~(size_t)15);
        block_cache_wave<MODE, PROXY>(b, p, lane, state, &comm);
    }
}

}  // namespace gorgo

// Replay kernel, segment formulation (chain-consistent traces).
//
// On a chain-consistent trace every request is a root-to-node path of the key forest and a whole number of
// segments.  With the root-newest stamp order a replica's cache is always closed under taking prefixes,
// every block of a segment carries the same last-touching request, and a block is cached iff its
// (last request, position) is not below the replica's eviction cursor.  The cache state of a replay is
// therefore one 32-bit "last request that touched it" per (segment, replica), stored as dense rows of R
// cells addressed by segment id: no hashing, no probing.
//
// Eviction (least recently used block first) only moves a cursor and writes no cell.  The cursor of a
// replica walks that replica's log of routed requests, oldest first.  A logged request still *owns* the
// blocks of its path that no later request on the same replica has touched again; because paths of a forest
// share prefixes only, that is always a suffix [own, n) of its path.  `own` is kept up to date when a later
// request takes segments over (the cells just read say whom they belonged to), so the walk needs one small
// record per logged request (next request on the replica, own, n) and never re-reads cells.
//
// The request loop is one dependent chain per replay, so the kernel is arranged around memory latency, not
// bandwidth: a batch of 64 requests is staged at once (scalars in registers, segment references in LDS);
// the rows of request i+2 are requested while request i is still being processed, and re-requested only if
// request i+1 wrote into them (same root segment); the log records of the next two eviction victims of every
// replica are held in registers; all stores are fire-and-forget.
#pragma once
#include <type_traits>

#include "device_common.h"
#include "internal.h"

namespace gorgo {

// Log record of a routed request: next request routed to the same replica, start of the owned suffix of its
// path, and its number of blocks.  Read and written as one 64-bit word: next | own << 32 | n << 48.
struct LogRec {
    int32_t next;
    uint16_t own;
    uint16_t n;
};

struct SegArgs {
    const int64_t* ts;
    const int32_t* in_len;
    const int32_t* out_len;
    const int64_t* seg_off;
    const SegRef* seg;
    int64_t N;
    int32_t R, B;
    int64_t C;
    int64_t nseg;
    int32_t block_tokens;
    double a_pf, a_dec;
    const double* rtt;
    const double* params;
    const double* scale;
    int32_t* last;   // [P][nseg][R], -1 = never touched
    LogRec* log;     // [P][N]
    Rec* rec;        // [P][N]
    uint8_t* route;  // [P][N], nullable
    uint16_t* hit;   // nullable
    double* ttft;    // nullable
    double* e2e;     // nullable
};

constexpr int SEG_STAGE = 512;   // segment references of a 64-request batch staged in LDS
constexpr int SEG_CHUNK = 8;     // segments of a request whose rows are loaded together

__host__ __device__ inline size_t replay_segments_lds_bytes(int R, int B) {   // dynamic part
    return Queues::bytes(R, B);
}

// Rows of one request's first SEG_CHUNK segments as seen by this lane (= replica), with the segments' end
// positions (the same in every lane).
struct RowSet {
    int32_t cell[SEG_CHUNK];
    int end[SEG_CHUNK];
};

__global__ void __launch_bounds__(WAVE) replay_segments_kernel(SegArgs a) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ SegRef stage[SEG_STAGE + SEG_CHUNK];    // padded: whole chunks are read unconditionally
    const int lane = threadIdx.x;
    const int p = blockIdx.x;
    const int R = a.R, B = a.B;
    const int64_t N = a.N;

    Queues Q;
    Q.carve(lds_raw, R, B);
    Q.init(lane);
    for (int x = lane; x < SEG_CHUNK; x += WAVE) stage[SEG_STAGE + x] = SegRef{0, 0};
    __syncthreads();

    const double w_rtt = a.params[3 * (size_t)p + 0];
    const double w_prefill = a.params[3 * (size_t)p + 1];
    const double w_queue = a.params[3 * (size_t)p + 2];
    const double sc = a.scale[p];
    const double my_rtt = lane < R ? a.rtt[lane] : 0.0;

    // Per-replica eviction state, held by lane = replica.  Blocks last touched by a request before cur_r, or
    // by cur_r at positions >= cur_k, are evicted; cur_own is where cur_r's owned suffix starts.  nx_* is
    // the log record after cur_r and n2_* the one after that (kept as the raw 64-bit word so that the load
    // that fetches it is not waited for until it is needed; changes made to that record meanwhile are kept
    // beside it in n2_own / n2_next and override the loaded fields).  tail_r is the youngest request routed
    // here and my_live the number of blocks cached on the replica.
    int cur_r = -1, cur_k = 0, cur_own = 0;
    int nx_r = -1, nx_n = 0, nx_own = 0;
    int n2_r = -1, n2_own = -1, n2_next = -1;
    unsigned long long n2_raw = 0;
    int tail_r = -1;
    int my_live = 0;

    int32_t* const last = a.last + (size_t)p * a.nseg * R;
    LogRec* const log = a.log + (size_t)p * N;
    unsigned long long* const log64 = reinterpret_cast<unsigned long long*>(log);
    Rec* const rec = a.rec + (size_t)p * N;

    // cached blocks of one segment [pos, end) whose row cell holds rl, against a cursor (c_r, c_k)
    auto cached_in = [](int32_t rl, int pos, int end, int c_r, int c_k) -> int {
        const int len = end - pos;
        if (rl > c_r) return len;
        if (rl == c_r && rl >= 0) {
            const int c = c_k - pos;
            return c < 0 ? 0 : (c > len ? len : c);
        }
        return 0;
    };

    int64_t r0 = 0;
    while (r0 < N) {
        // ---- stage a batch of up to 64 requests: per-request scalars in registers (lane = request), their
        // segment references in LDS.  The batch is cut where the references stop fitting; a single request
        // with more references than the stage holds is processed alone, reading them from global memory.
        const int nb0 = N - r0 < WAVE ? (int)(N - r0) : WAVE;
        const int64_t rr = r0 + (lane < nb0 ? lane : nb0 - 1);
        const double m_t = (double)a.ts[rr] * sc;          // time scale: gaps scale linearly
        const int m_L = a.in_len[rr];
        const int m_O = a.out_len[rr];
        const int64_t my_j0 = a.seg_off[rr], my_j1 = a.seg_off[rr + 1];
        const int64_t J0 = a.seg_off[r0];
        const int fit = __popcll(__ballot(lane < nb0 && my_j1 - J0 <= SEG_STAGE));   // a prefix of the lanes
        const bool staged = fit > 0;
        const int nb = staged ? fit : 1;
        const int m_a0 = (int)(my_j0 - J0);
        const int m_s = (int)(my_j1 - my_j0);
        const SegRef* const gref = a.seg + J0;
        if (staged) {
            const int cnt = __builtin_amdgcn_readlane(m_a0 + m_s, nb - 1);
            for (int x = lane; x < cnt; x += WAVE) stage[x] = gref[x];
        }
        __syncthreads();
        int m_n = 0, m_root = -1;       // blocks of the request; its first segment (the root of its tree)
        if (m_s > 0 && lane < nb) {
            m_n = staged ? stage[m_a0 + m_s - 1].end : gref[m_a0 + m_s - 1].end;
            m_root = staged ? stage[m_a0].id : gref[m_a0].id;
        }

        int o_route = 0, o_hit = 0;
        double o_ttft = 0.0, o_e2e = 0.0;

        // requests the rows of the first segments of request i of the batch (staged batches only)
        auto request_rows = [&](int i, RowSet& w) {
            const int a0 = __builtin_amdgcn_readlane(m_a0, i);
            const int s = __builtin_amdgcn_readlane(m_s, i);
            SegRef sr[SEG_CHUNK];
#pragma unroll
            for (int k = 0; k < SEG_CHUNK; ++k) sr[k] = stage[a0 + k];
#pragma unroll
            for (int k = 0; k < SEG_CHUNK; ++k) {
                w.cell[k] = -1;
                w.end[k] = sr[k].end;
                if (k < s && lane < R) w.cell[k] = ld(&last[(size_t)sr[k].id * R + lane]);
            }
        };

        // Processes request i of the batch.  `mine` holds its rows when PRELOADED; `other` holds the rows of
        // request i+1 and is refreshed if this request writes into them.
        auto process = [&](int i, auto ref, auto preloaded, RowSet& mine, RowSet& other) {
            constexpr bool PRELOADED = decltype(preloaded)::value;
            const int64_t r = r0 + i;
            const double t = readlane_f64(m_t, i);
            const int64_t L = __builtin_amdgcn_readlane(m_L, i);
            const int64_t O = __builtin_amdgcn_readlane(m_O, i);
            const int a0 = __builtin_amdgcn_readlane(m_a0, i);
            const int s = __builtin_amdgcn_readlane(m_s, i);
            const int n = __builtin_amdgcn_readlane(m_n, i);

            Q.retire(t, rec, lane);

            // ---- prefix match: lane = replica
            int my_m = 0;
            bool open = lane < R;
            int pos = 0;
            if (PRELOADED) {
#pragma unroll
                for (int k = 0; k < SEG_CHUNK; ++k) {
                    if (k < s) {
                        if (open) {
                            const int cnt = cached_in(mine.cell[k], pos, mine.end[k], cur_r, cur_k);
                            my_m += cnt;
                            open = cnt == mine.end[k] - pos;
                        }
                        pos = mine.end[k];
                    }
                }
            }
            if ((!PRELOADED || s > SEG_CHUNK) && __ballot(open) != 0) {
                for (int c0 = PRELOADED ? SEG_CHUNK : 0; c0 < s; c0 += SEG_CHUNK) {
                    int32_t cell[SEG_CHUNK];
                    int send[SEG_CHUNK];
#pragma unroll
                    for (int k = 0; k < SEG_CHUNK; ++k) {
                        cell[k] = -1;
                        send[k] = 0;
                        if (c0 + k < s) {
                            const SegRef sr = ref(a0 + c0 + k);
                            send[k] = sr.end;
                            if (open) cell[k] = ld(&last[(size_t)sr.id * R + lane]);
                        }
                    }
#pragma unroll
                    for (int k = 0; k < SEG_CHUNK; ++k) {
                        if (c0 + k < s) {
                            if (open) {
                                const int cnt = cached_in(cell[k], pos, send[k], cur_r, cur_k);
                                my_m += cnt;
                                open = cnt == send[k] - pos;
                            }
                            pos = send[k];
                        }
                    }
                    if (__ballot(open) == 0) break;
                }
            }

            // ---- score (Eq. 3) and lowest-index minimum
            int64_t my_u = 0;
            double my_score = INFINITY;
            if (lane < R) {
                int64_t hit_tok = (int64_t)a.block_tokens * my_m;
                if (hit_tok > L) hit_tok = L;
                my_u = L - hit_tok;
                my_score = eq3_score(w_rtt, w_prefill, w_queue, my_rtt, a.a_pf, my_u, Q.my_q);
            }
            const int best = wave_argmin(my_score, lane, R).idx;
            const int m_best = __builtin_amdgcn_readlane(my_m, best);

            // ---- ownership: the segments this request takes over on the chosen replica stop belonging to
            // their previous requests.  Along the path the previous owners form runs; each run moves its
            // owner's `own` to the end of the run.  Only cached segments matter (evicted ones belong to
            // requests the cursor has passed, or to the cursor request beyond its position).
            if (m_best > 0) {
                const int cb_r = __builtin_amdgcn_readlane(cur_r, best), cb_k = __builtin_amdgcn_readlane(cur_k, best);
                int run_owner = -1, run_end = 0, vpos = 0;
                auto flush = [&]() {
                    if (run_owner >= 0) {
                        if (lane == 0) st(&log[run_owner].own, (uint16_t)run_end);
                        if (lane == best) {
                            if (run_owner == cur_r) cur_own = run_end;
                            if (run_owner == nx_r) nx_own = run_end;
                            if (run_owner == n2_r) n2_own = run_end;
                        }
                    }
                };
                auto visit = [&](int32_t rl, int end) -> bool {      // returns false once the prefix ends
                    const int cnt = cached_in(rl, vpos, end, cb_r, cb_k);
                    const bool full = cnt == end - vpos;
                    if (cnt > 0) {
                        if (rl != run_owner) {
                            flush();
                            run_owner = rl;
                        }
                        run_end = end;
                    }
                    vpos = end;
                    return full;
                };
                if (PRELOADED && s <= SEG_CHUNK) {
                    bool go = true;
#pragma unroll
                    for (int k = 0; k < SEG_CHUNK; ++k) {
                        if (go && k < s) {
                            const int32_t rl = __builtin_amdgcn_readlane(mine.cell[k], best);
                            const int end = __builtin_amdgcn_readfirstlane(mine.end[k]);
                            go = visit(rl, end);
                        }
                    }
                } else {
                    for (int j = 0; j < s; ++j) {
                        const SegRef sr = ref(a0 + j);
                        if (!visit(ld(&last[(size_t)sr.id * R + best]), sr.end)) break;
                    }
                }
                flush();
            }

            // ---- cache update: every segment of the request is now last touched by r on the chosen replica
            for (int base = 0; base < s; base += WAVE) {
                const int j = base + lane;
                if (j < s) st(&last[(size_t)ref(a0 + j).id * R + best], (int32_t)r);
            }
            // ---- log: append r to the chosen replica's list of routed requests
            const unsigned long long fresh = 0xFFFFFFFFull | ((unsigned long long)n << 48);   // next -1, own 0, n
            if (lane == 0) st(&log64[r], fresh);
            if (lane == best) {
                if (tail_r >= 0) st(&log[tail_r].next, (int32_t)r);
                if (tail_r < 0) {
                    cur_r = (int)r;
                    cur_k = n;
                    cur_own = 0;
                } else if (cur_r == tail_r) {
                    nx_r = (int)r;
                    nx_n = n;
                    nx_own = 0;
                } else if (nx_r == tail_r) {
                    n2_r = (int)r;               // record known without a load: own 0, next none
                    n2_raw = fresh;
                    n2_own = -1;
                    n2_next = -1;
                } else if (n2_r == tail_r) {
                    n2_next = (int)r;
                }
                tail_r = (int)r;

                // ---- eviction: move the cursor forward until the cache fits
                if (a.C > 0) {
                    my_live += n - m_best;
                    if (my_live > a.C) {
                        int E = my_live - (int)a.C;
                        for (;;) {
                            const int avail = cur_k - cur_own;
                            if (avail >= E) {
                                cur_k -= E;
                                E = 0;
                                break;
                            }
                            if (avail > 0) E -= avail;
                            if (nx_r < 0) break;      // cannot happen while E > 0; bounds the loop regardless
                            cur_r = nx_r;
                            cur_k = nx_n;
                            cur_own = nx_own;
                            nx_r = n2_r;
                            if (nx_r >= 0) {
                                nx_n = (int)(n2_raw >> 48);
                                nx_own = n2_own >= 0 ? n2_own : (int)((n2_raw >> 32) & 0xFFFF);
                                n2_r = n2_next >= 0 ? n2_next : (int)(unsigned int)n2_raw;
                                n2_own = -1;
                                n2_next = -1;
                                if (n2_r >= 0) n2_raw = ld(&log64[n2_r]);
                            }
                        }
                        my_live = (int)a.C + E;
                    }
                }
            }

            // ---- service on the chosen replica, outputs (kept in registers until the batch ends)
            double ttft, e2e;
            Q.serve(r, best, t, my_rtt, my_u, L, O, a.a_pf, a.a_dec, rec, lane, &ttft, &e2e);
            if (lane == i) {
                o_route = best;
                o_hit = m_best;
                o_ttft = ttft;
                o_e2e = e2e;
            }

            // ---- rows for later requests, requested after this request's stores (a wavefront's memory
            // operations are performed in order): request i+2 into the set just consumed; request i+1 again
            // if it shares this request's root segment, because its rows were requested before these stores.
            if (PRELOADED) {
                if (i + 1 < nb && s > 0 &&
                    __builtin_amdgcn_readlane(m_root, i + 1) == __builtin_amdgcn_readlane(m_root, i))
                    request_rows(i + 1, other);
                if (i + 2 < nb) request_rows(i + 2, mine);
            }
            __syncthreads();
        };

        if (staged) {
            RowSet A, Bset;
            request_rows(0, A);
            if (nb > 1) request_rows(1, Bset);
            const auto from_stage = [&](int x) -> SegRef { return stage[x]; };
            for (int i = 0; i < nb; i += 2) {
                process(i, from_stage, std::true_type{}, A, Bset);
                if (i + 1 < nb) process(i + 1, from_stage, std::true_type{}, Bset, A);
            }
        } else {
            RowSet A, Bset;
            process(0, [&](int x) -> SegRef { return gref[x]; }, std::false_type{}, A, Bset);
        }
        if (lane < nb) {
            const size_t o = (size_t)p * N + r0 + lane;
            if (a.route) a.route[o] = (uint8_t)o_route;
            if (a.hit) a.hit[o] = (uint16_t)o_hit;
            if (a.ttft) a.ttft[o] = o_ttft;
            if (a.e2e) a.e2e[o] = o_e2e;
        }
        __syncthreads();
        r0 += nb;
    }
}

}  // namespace gorgo

// Replay kernel, segment formulation, two replays per wavefront pair (fixed weights, up to 32 replicas).
//
// A replay keeps one lane per replica, so with 32 replicas or fewer half of every wavefront idles, and a lone
// wavefront issues an instruction every four to five cycles whatever it does.  Here the two halves of the cache
// wavefront and of the queue wavefront run two replays of the same launch side by side: lanes 0..31 hold
// the replicas of replay 2b, lanes 32..63 those of replay 2b + 1 (b = workgroup).  Both replays walk the same
// trace in lockstep, so everything derived from the trace (request scalars, segment references, batch staging,
// loop control) is shared and wavefront-uniform as before; what belongs to a replay (weights, time scale, rows,
// log, cursors, queues, the chosen replica) lives per lane or, for the handful of values that were scalars, as a
// pair of scalars.  The arithmetic per replay is that of replay_segments_kernel, operation for operation.
#pragma once
#include "replay_segments.h"

namespace gorgo {

constexpr int HALF = WAVE / 2;

// Hand-over words of a packed pair of replays (see SegComm): the load signals of both replays come with one tag,
// the two choices are written one after the other and the second carries the tag that is polled.
struct PackComm {
    double q[WAVE];                   // load signal per (replay, replica), valid when seq_q == r + 1
    unsigned seq_q;
    int abandoned;
    unsigned long long choice[2];     // per replay: uncached tokens | (((r + 1) mod 2^26) << 6 | replica) << 32
    unsigned long long look[(LOOK_RING + 1) * WAVE];      // look-ahead of the eviction cursors, see EvictCursor
};

__host__ __device__ inline size_t replay_segments_packed_lds_bytes(int B) { return Queues::bytes(WAVE, B); }

// Minimum of x over each half of the wavefront: row shifts inside the rows of 16 lanes, then lane 15 of rows 0
// and 2 into rows 1 and 3; lanes 31 and 63 hold the results.
__device__ __forceinline__ void half_min_u32(unsigned x, unsigned* m0, unsigned* m1) {
    x = dpp_min_u32<0x111, 0xf>(x);   // row_shr:1
    x = dpp_min_u32<0x112, 0xf>(x);   // row_shr:2
    x = dpp_min_u32<0x114, 0xf>(x);   // row_shr:4
    x = dpp_min_u32<0x118, 0xf>(x);   // row_shr:8
    x = dpp_min_u32<0x142, 0xa>(x);   // row_bcast:15 into rows 1, 3
    *m0 = (unsigned)__builtin_amdgcn_readlane((int)x, HALF - 1);
    *m1 = (unsigned)__builtin_amdgcn_readlane((int)x, WAVE - 1);
}

// wave_argmin for the two halves at once: lowest index (within its half) of the minimum over the lanes of each
// half whose index within the half is below `count`.
__device__ __forceinline__ void half_argmin(double v, int lane, int count, int* best0, int* best1) {
    const unsigned long long bits = (unsigned long long)__double_as_longlong(v + 0.0);
    const unsigned hi = (unsigned)(bits >> 32), lo = (unsigned)bits;
    const unsigned neg = (unsigned)((int)hi >> 31);
    const bool in = (lane & (HALF - 1)) < count;
    const bool upper = lane >= HALF;
    const unsigned khi = in ? hi ^ (neg | 0x80000000u) : 0xffffffffu;
    const unsigned klo = lo ^ neg;
    unsigned m0, m1;
    half_min_u32(khi, &m0, &m1);
    const bool tie = in && khi == (upper ? m1 : m0);
    unsigned long long ties = __ballot(tie);
    unsigned t0 = (unsigned)ties, t1 = (unsigned)(ties >> 32);
    if (((t0 & (t0 - 1)) | (t1 & (t1 - 1))) != 0) {       // some half has several lanes on its smallest high word
        half_min_u32(tie ? klo : 0xffffffffu, &m0, &m1);
        ties = __ballot(tie && klo == (upper ? m1 : m0));
        t0 = (unsigned)ties;
        t1 = (unsigned)(ties >> 32);
    }
    *best0 = __ffs(t0) - 1;
    *best1 = __ffs(t1) - 1;
}

// Queue side of a packed pair: lane = (replay, replica).  As queue_wave of replay_segments.h for fixed weights.
__device__ __forceinline__ void queue_wave_packed(const SegArgs& a, int lane, unsigned char* lds_raw, PackComm* comm) {
    const int R = a.R;
    const int64_t N = a.N;
    const bool upper = lane >= HALF;
    const int rl = lane & (HALF - 1);
    const size_t p0 = 2 * (size_t)blockIdx.x;
    const size_t p = p0 + (upper ? 1 : 0);
    Queues Q;
    Q.carve(lds_raw, WAVE, a.B, lane);      // every lane has its own slots; those of lanes without a replica stay idle
    Q.init(lane);
    wave_sync();
    const double sc = a.scale[p];
    const double my_rtt = rl < R ? a.rtt[rl] : 0.0;
    Rec* const rec = a.rec + p * N;
    bool dead = false;
    for (int64_t r0 = 0; r0 < N && !dead; r0 += WAVE) {
        const int nb = N - r0 < WAVE ? (int)(N - r0) : WAVE;
        const int64_t rr = r0 + (lane < nb ? lane : nb - 1);
        const double m_ts = (double)a.ts[rr];              // lane = request of the batch
        const int m_L = a.in_len[rr];
        const int m_O = a.out_len[rr];
        double o_ttft0 = 0.0, o_e2e0 = 0.0, o_ttft1 = 0.0, o_e2e1 = 0.0;
        for (int i = 0; i < nb; ++i) {
            const int64_t r = r0 + i;
            const double t = readlane_f64(m_ts, i) * sc;    // time scale of this lane's replay
            const int L = __builtin_amdgcn_readlane(m_L, i);
            const int O = __builtin_amdgcn_readlane(m_O, i);
            Q.retire(t, rec);
            st(&comm->q[lane], Q.my_q);
            lds_release();
            if (lane == 0) st(&comm->seq_q, (unsigned)(r + 1));
            const unsigned long long idle_now = Q.idle;
            if (r + 1 < N) {
                const double ts_next = i + 1 < nb ? readlane_f64(m_ts, i + 1) : (double)a.ts[r + 1];
                Q.retire(ts_next * sc, rec);
            }
            const unsigned want = (unsigned)(r + 1) & 0x3FFFFFFu;
            unsigned hi1, lo1;
            for (int spins = 0;; ++spins) {
                const unsigned long long w = ld(&comm->choice[1]);
                hi1 = __builtin_amdgcn_readfirstlane((unsigned)(w >> 32));
                lo1 = __builtin_amdgcn_readfirstlane((unsigned)w);
                if ((hi1 >> 6) == want) break;
                if (spins > a.spin_limit || ld(&comm->abandoned) != 0) {
                    dead = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            if (dead) break;
            lds_acquire();
            const unsigned long long w0 = ld(&comm->choice[0]);      // written before choice[1]
            const unsigned hi0 = __builtin_amdgcn_readfirstlane((unsigned)(w0 >> 32));
            const unsigned lo0 = __builtin_amdgcn_readfirstlane((unsigned)w0);
            const int best0 = (int)(hi0 & 63u), best1 = (int)(hi1 & 63u);
            const int best_lane = upper ? HALF + best1 : best0;
            const int64_t uncached = (int64_t)(int)(upper ? lo1 : lo0);
            double ttft, e2e;
            Q.template serve<false, true>(r, best_lane, t, my_rtt, uncached, L, O, a.a_pf, a.a_dec, rec, lane, idle_now,
                                          &ttft, &e2e);
            const double t0 = readlane_f64(ttft, best0), e0 = readlane_f64(e2e, best0);
            const double t1 = readlane_f64(ttft, HALF + best1), e1 = readlane_f64(e2e, HALF + best1);
            o_ttft0 = lane == i ? t0 : o_ttft0;
            o_e2e0 = lane == i ? e0 : o_e2e0;
            o_ttft1 = lane == i ? t1 : o_ttft1;
            o_e2e1 = lane == i ? e1 : o_e2e1;
        }
        if (lane < nb && !dead) {
            const size_t o = p0 * N + r0 + lane;
            if (a.ttft) {
                a.ttft[o] = o_ttft0;
                a.ttft[o + N] = o_ttft1;
            }
            if (a.e2e) {
                a.e2e[o] = o_e2e0;
                a.e2e[o + N] = o_e2e1;
            }
        }
    }
    if (dead) {
        // the partner never answered (cannot happen unless the kernel is wrong): leave, and make sure nobody
        // mistakes these replays' latencies for results
        st(&comm->abandoned, 1);
        for (int64_t x = lane; x < 2 * N; x += WAVE) {
            if (a.ttft) a.ttft[p0 * N + x] = NAN;
            if (a.e2e) a.e2e[p0 * N + x] = NAN;
        }
    }
}

// One workgroup = replays 2b and 2b + 1.  Needs R <= 32, an even number of replays, and the rows of two replays
// within 4 GiB (checked by the host).
__global__ void __launch_bounds__(SEG_THREADS) replay_segments_packed_kernel(SegArgs a) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ SegRef stage[SEG_STAGE + SEG_CHUNK];    // padded: whole chunks are read unconditionally
    __shared__ PackComm comm;
    const int lane = threadIdx.x & (WAVE - 1);
    const int R = a.R;
    const int64_t N = a.N;
    const int C = (int)a.C;

    if (threadIdx.x == 0) {
        comm.seq_q = 0;
        comm.abandoned = 0;
        comm.choice[0] = 0;
        comm.choice[1] = 0;
    }
    __syncthreads();
    if (threadIdx.x >= WAVE) {
        queue_wave_packed(a, lane, lds_raw, &comm);
        return;
    }
    __builtin_amdgcn_s_setprio(3);      // the cache wavefront has the longer loop: it goes first at issue
    bool dead = false;

    for (int x = lane; x < SEG_CHUNK; x += WAVE) stage[SEG_STAGE + x] = SegRef{0, 0};
    wave_sync();

    const bool upper = lane >= HALF;
    const int rl = lane & (HALF - 1);               // replica of this lane
    const size_t p0 = 2 * (size_t)blockIdx.x;
    const size_t p = p0 + (upper ? 1 : 0);          // replay of this lane
    const double w_rtt = a.params[3 * p + 0];
    const double w_prefill = a.params[3 * p + 1];
    const double w_queue = a.params[3 * p + 2];
    const double my_rtt = rl < R ? a.rtt[rl] : 0.0;

    // Per-(replay, replica) eviction state, held by the lane: the same cursor as in replay_segments_kernel.
    EvictCursor c1;
    c1.ring = &comm.look[lane];
    for (int k = 0; k <= LOOK_RING; ++k) c1.ring[k * WAVE] = ~0ull;
    int tail_r = -1;          // youngest request routed to this replica

    // rows of the two replays follow each other; a cell is addressed by a 32-bit byte offset from the first
    int32_t* const last = a.last + p0 * (size_t)a.nseg * R;
    const unsigned row_bytes = (unsigned)R * 4u;
    const unsigned replay_off = upper ? (unsigned)a.nseg * row_bytes : 0u;
    const unsigned lane_off = replay_off + (unsigned)(rl < R ? rl : 0) * 4u;
    auto cell_at = [&](int seg_id) -> int32_t* {      // this lane's cell of a segment's row
        return reinterpret_cast<int32_t*>(reinterpret_cast<char*>(last) + ((unsigned)seg_id * row_bytes + lane_off));
    };
    auto cell_of = [&](int seg_id, int replica) -> int32_t* {      // the cell of `replica` in this lane's replay
        return reinterpret_cast<int32_t*>(reinterpret_cast<char*>(last) +
                                          ((unsigned)seg_id * row_bytes + replay_off + (unsigned)replica * 4u));
    };
    LogRec* const log = a.log + p * (N + 1);
    unsigned long long* const log64 = reinterpret_cast<unsigned long long*>(log);
    const int spare = (int)N;           // the log record behind the last request's: where loads with nothing to fetch go

    int64_t r0 = 0;
    while (r0 < N && !dead) {
        // ---- stage a batch of up to 64 requests (shared by the two replays): per-request scalars in registers
        // (lane = request), their segment references in LDS
        const int nb0 = N - r0 < WAVE ? (int)(N - r0) : WAVE;
        const int64_t rr = r0 + (lane < nb0 ? lane : nb0 - 1);
        const int m_L = a.in_len[rr];
        const int64_t my_j0 = a.seg_off[rr], my_j1 = a.seg_off[rr + 1];
        const int64_t J0 = a.seg_off[r0];
        const int fit = __popcll(__ballot(lane < nb0 && my_j1 - J0 <= SEG_STAGE));   // a prefix of the lanes
        const bool staged = fit > 0;
        const int nb = staged ? fit : 1;
        const int m_a0 = (int)(my_j0 - J0);
        const int m_s = (int)(my_j1 - my_j0);
        const SegRef* const gref = a.seg + J0;
        int m_n = 0, m_root = -1;       // blocks of the request; its first segment (the root of its tree)
        if (staged) {
            const int cnt = __builtin_amdgcn_readlane(m_a0 + m_s, nb - 1);
            for (int x = lane; x < cnt; x += WAVE) stage[x] = gref[x];
            wave_sync();
            if (m_s > 0 && lane < nb) {
                m_n = stage[m_a0 + m_s - 1].end & SEG_END_MASK;
                m_root = stage[m_a0].id;
            }
        } else if (m_s > 0 && lane == 0) {
            m_n = gref[m_s - 1].end & SEG_END_MASK;
            m_root = gref[0].id;
        }

        int o_route0 = 0, o_hit0 = 0, o_route1 = 0, o_hit1 = 0;

        // requests the rows of the first SEG_CHUNK segments of request i of the batch (each half its replay's)
        auto request_rows = [&](int i, auto ref, RowSet& w) {
            const int a0 = __builtin_amdgcn_readlane(m_a0, i);
            const int s = __builtin_amdgcn_readlane(m_s, i);
            const int n = __builtin_amdgcn_readlane(m_n, i);
            w.of_lane = ref(a0 + (rl < SEG_CHUNK ? rl : 0), rl < s && rl < SEG_CHUNK);
            w.fresh = 0;
#pragma unroll
            for (int k = 0; k < SEG_CHUNK; ++k) w.end[k] = n;       // (cells past the last segment are never read)
#pragma unroll
            for (int h = 0; h < SEG_CHUNK; h += 4) {
                if (h >= s) break;
                SegRef sr[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) sr[k] = ref(a0 + h + k, h + k < s);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (h + k >= s) break;
                    w.end[h + k] = sr[k].end & SEG_END_MASK;
                    if (sr[k].end & SEG_FRESH) {
                        // the row slot starts over with this request: what it holds belongs to a segment of the past
                        w.fresh |= 1 << (h + k);
                        w.cell[h + k] = NEVER_CACHED;
                    } else {
                        w.cell[h + k] = ld(cell_at(sr[k].id));       // lanes beyond R read a neighbouring cell, unused
                    }
                }
            }
        };

        // Processes request i of the batch for both replays.
        auto process = [&](int i, auto ref, RowSet& mine, RowSet& other) {
            const int64_t r = r0 + i;
            const int L = __builtin_amdgcn_readlane(m_L, i);
            const int a0 = __builtin_amdgcn_readlane(m_a0, i);
            const int s = __builtin_amdgcn_readlane(m_s, i);
            const int n = __builtin_amdgcn_readlane(m_n, i);

            // ---- prefix match (lane = replica of its replay): as in replay_segments_kernel
            int e_gt = 0, e_ge = 0;
            int32_t own_gt = -1;
#pragma unroll
            for (int k = 0; k < SEG_CHUNK; ++k) {
                if (k >= s) break;
                const bool gt = mine.cell[k] > c1.cur_r;
                const bool ge = mine.cell[k] >= c1.cur_r;
                e_gt = gt ? mine.end[k] : e_gt;
                own_gt = gt ? mine.cell[k] : own_gt;
                e_ge = ge ? mine.end[k] : e_ge;
            }
            const int below_cursor = c1.cur_k < e_ge ? c1.cur_k : e_ge;
            const bool some_eq = below_cursor > e_gt;
            int my_m = some_eq ? below_cursor : e_gt;
            const int k_end = some_eq ? e_ge : e_gt;
            const bool one_owner = some_eq ? e_gt == 0 : own_gt == mine.cell[0];
            int pos = mine.end[SEG_CHUNK - 1];
            bool open = my_m == pos;
            bool deep = false;          // the match of some lane went past the preloaded segments
            if (s > SEG_CHUNK && __ballot(open && rl < R) != 0) {
                deep = true;
                for (int c0 = SEG_CHUNK; c0 < s; c0 += SEG_CHUNK) {
                    int32_t cell[SEG_CHUNK];
                    int send[SEG_CHUNK];
#pragma unroll
                    for (int k = 0; k < SEG_CHUNK; ++k) {
                        cell[k] = NEVER_CACHED;
                        send[k] = pos;
                        if (c0 + k < s) {
                            const SegRef sr = ref(a0 + c0 + k, true);
                            send[k] = sr.end & SEG_END_MASK;
                            if (open && rl < R && !(sr.end & SEG_FRESH)) cell[k] = ld(cell_at(sr.id));
                        }
                    }
#pragma unroll
                    for (int k = 0; k < SEG_CHUNK; ++k) {
                        if (c0 + k < s) {
                            const int cnt = cached_in(cell[k], pos, send[k], c1.cur_r, c1.cur_k);
                            my_m += open ? cnt : 0;
                            open = open && cnt == send[k] - pos;
                            pos = send[k];
                        }
                    }
                    if (__ballot(open && rl < R) == 0) break;
                }
            }

            // ---- the single point of the iteration that waited for memory is behind us
            c1.take_pending(c1.pend_raw);
            if (i + 1 < nb) request_rows(i + 1, ref, other);
            c1.issue_fill(log64, spare);

            // ---- score (Eq. 3) and lowest-index minimum, per replay
            int hit_tok = a.block_tokens * my_m;
            hit_tok = hit_tok > L ? L : hit_tok;
            int my_u = L - hit_tok;
            const double score_rp = eq3_without_queue(w_rtt, w_prefill, my_rtt, a.a_pf, my_u);
            asm volatile("" : "+v"(my_u), "+v"(my_m));
            double score_rp_ready = score_rp;
            asm volatile("" : "+v"(score_rp_ready));
            double my_q;
            for (int spins = 0;; ++spins) {
                const unsigned seq = __builtin_amdgcn_readfirstlane(ld(&comm.seq_q));
                lds_acquire();
                my_q = ld(&comm.q[lane]);
                if (seq == (unsigned)(r + 1)) break;
                if (spins > a.spin_limit || ld(&comm.abandoned) != 0) {
                    dead = true;
                    break;
                }
            }
            if (dead) {
                st(&comm.abandoned, 1);
                return;
            }
            const double my_score = eq3_with_queue(score_rp_ready, w_queue, a.a_pf, my_q);
            int best0, best1;
            half_argmin(my_score, lane, R, &best0, &best1);
            const int best = upper ? best1 : best0;              // the replica this lane's replay chose
            const bool is_best = rl == best;
            const int m_best0 = __builtin_amdgcn_readlane(my_m, best0);
            const int m_best1 = __builtin_amdgcn_readlane(my_m, HALF + best1);
            const int m_best = upper ? m_best1 : m_best0;
            if (lane == 0) {
                const unsigned u0 = (unsigned)__builtin_amdgcn_readlane(my_u, best0);
                const unsigned u1 = (unsigned)__builtin_amdgcn_readlane(my_u, HALF + best1);
                const unsigned tag = ((unsigned)(r + 1) & 0x3FFFFFFu) << 6;
                st(&comm.choice[0], ((unsigned long long)(tag | (unsigned)best0) << 32) | u0);
                lds_release();
                st(&comm.choice[1], ((unsigned long long)(tag | (unsigned)best1) << 32) | u1);
            }

            // ---- ownership, per replay: see replay_segments_kernel
            auto disown = [&](int owner, int end) {       // chosen lane: owner's owned suffix now starts at end
                st(&log[owner].own, (uint16_t)end);
                c1.disowned_anywhere(owner, end);
            };
            if ((m_best0 | m_best1) > 0) {
                const bool simple0 = !deep && __builtin_amdgcn_readlane((int)one_owner, best0) != 0;
                const bool simple1 = !deep && __builtin_amdgcn_readlane((int)one_owner, HALF + best1) != 0;
                const bool simple = upper ? simple1 : simple0;
                if (is_best && m_best > 0 && simple) disown(mine.cell[0], k_end);
                if ((m_best0 > 0 && !simple0) || (m_best1 > 0 && !simple1)) {
                    // several previous owners, or a prefix longer than the preloaded rows: walk it (all lanes of a
                    // half follow their replay's chosen replica; halves that need no walk stay out)
                    const int cb_r0 = __builtin_amdgcn_readlane(c1.cur_r, best0), cb_r1 = __builtin_amdgcn_readlane(c1.cur_r, HALF + best1);
                    const int cb_k0 = __builtin_amdgcn_readlane(c1.cur_k, best0), cb_k1 = __builtin_amdgcn_readlane(c1.cur_k, HALF + best1);
                    const int cb_r = upper ? cb_r1 : cb_r0, cb_k = upper ? cb_k1 : cb_k0;
                    bool walking = m_best > 0 && !simple;
                    int run_owner = -1, run_end = 0, vpos = 0;
                    for (int j = 0; j < s && __ballot(walking) != 0; ++j) {
                        SegRef sr = ref(a0 + j, true);
                        const bool fresh = (sr.end & SEG_FRESH) != 0;
                        sr.end &= SEG_END_MASK;
                        if (walking) {
                            const int32_t rlast = fresh ? NEVER_CACHED : ld(cell_of(sr.id, best));
                            const int cnt = cached_in(rlast, vpos, sr.end, cb_r, cb_k);
                            if (cnt > 0) {
                                if (rlast != run_owner) {
                                    if (run_owner >= 0 && is_best) disown(run_owner, run_end);
                                    run_owner = rlast;
                                }
                                run_end = sr.end;
                            }
                            walking = cnt == sr.end - vpos;
                            vpos = sr.end;
                        }
                    }
                    if (run_owner >= 0 && is_best && m_best > 0 && !simple) disown(run_owner, run_end);
                }
            }

            // ---- cache update: every segment of the request is now last touched by r on the chosen replica of
            // each replay (lane k of a half stores the cell of segment k)
            if (rl < s && rl < SEG_CHUNK) st(cell_of(mine.of_lane.id, best), (int32_t)r);
            for (int j = SEG_CHUNK + rl; j < s; j += HALF) st(cell_of(ref(a0 + j, true).id, best), (int32_t)r);
            // A segment that this request is the first to reference has taken over a row slot from a segment of the
            // past: the row starts over, every replica's cell of either replay, never cached except on the chosen one.
            if (mine.fresh != 0 || s > SEG_CHUNK) {
                const int32_t fresh_cell = is_best ? (int32_t)r : NEVER_CACHED;
                for (unsigned rest = (unsigned)mine.fresh; rest != 0; rest &= rest - 1) {      // (mostly one)
                    const SegRef sr = ref(a0 + __builtin_ctz(rest), true);
                    if (rl < R) st(cell_at(sr.id), fresh_cell);
                }
                for (int j = SEG_CHUNK; j < s; ++j) {
                    const SegRef sr = ref(a0 + j, true);
                    if ((sr.end & SEG_FRESH) && rl < R) st(cell_at(sr.id), fresh_cell);
                }
            }

            // ---- log and eviction, in the chosen replicas' lanes
            if (is_best) {
                st(&log64[r], 0xFFFFFFFFull | ((unsigned long long)n << 48));      // next -1, own 0, n
                if (tail_r >= 0) st(&log[tail_r].next, (int32_t)r);
            }
            c1.appended(is_best, (int)r, n, tail_r);
            tail_r = is_best ? (int)r : tail_r;
            c1.evict(is_best && C > 0, n - m_best, C, log64, spare);

            // ---- the rows of request i+1 were requested before this request's stores: if it continues the
            // same tree, the cells this request just wrote are patched into them (common prefix of the paths)
            if (i + 1 < nb && s > 0 && __builtin_amdgcn_readlane(m_root, i + 1) == __builtin_amdgcn_readlane(m_root, i)) {
                const int s_next = __builtin_amdgcn_readlane(m_s, i + 1);
                // (a fresh segment of the next request may sit in the slot that this request's segment just gave up)
                const bool same = rl < s && rl < s_next && !(other.of_lane.end & SEG_FRESH) &&
                                  other.of_lane.id == mine.of_lane.id &&
                                  (other.of_lane.end & SEG_END_MASK) == (mine.of_lane.end & SEG_END_MASK);
                const unsigned differ = ~(unsigned)__ballot(same && rl < SEG_CHUNK) | (1u << SEG_CHUNK);   // (lower half)
                const int common = __ffs(differ) - 1;              // leading segments the two paths share
                // (where this request has just started the row over, what was loaded is the past's: never cached)
#pragma unroll
                for (int k = 0; k < SEG_CHUNK; ++k) {
                    const int32_t elsewhere = (mine.fresh >> k) & 1 ? NEVER_CACHED : other.cell[k];
                    other.cell[k] = k < common ? (is_best ? (int32_t)r : elsewhere) : other.cell[k];
                }
            }

            // ---- outputs of the cache side (kept in registers until the batch ends)
            if (a.route) {
                o_route0 = lane == i ? best0 : o_route0;
                o_route1 = lane == i ? best1 : o_route1;
            }
            if (a.hit) {
                o_hit0 = lane == i ? m_best0 : o_hit0;
                o_hit1 = lane == i ? m_best1 : o_hit1;
            }
        };

        RowSet A, Bset;
        if (staged) {
            const auto from_stage = [&](int x, bool) -> SegRef { return stage[x]; };
            request_rows(0, from_stage, A);
            for (int i = 0; i < nb && !dead; i += 2) {
                process(i, from_stage, A, Bset);
                if (i + 1 < nb && !dead) process(i + 1, from_stage, Bset, A);
            }
        } else {
            const auto from_global = [&](int x, bool in) -> SegRef { return in ? gref[x] : SegRef{0, 0}; };
            request_rows(0, from_global, A);
            process(0, from_global, A, Bset);
        }
        if (lane < nb && !dead) {
            const size_t o = p0 * N + r0 + lane;
            if (a.route) {
                a.route[o] = (uint8_t)o_route0;
                a.route[o + N] = (uint8_t)o_route1;
            }
            if (a.hit) {
                a.hit[o] = (uint16_t)o_hit0;
                a.hit[o + N] = (uint16_t)o_hit1;
            }
        }
        wave_sync();
        r0 += nb;
    }
}

}  // namespace gorgo

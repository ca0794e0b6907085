// Device helpers shared by the replay kernels: workgroup-scope memory accessors, wavefront reductions and
// the per-replay queue state (service slots, in-flight records, load signal) kept in LDS.
#pragma once
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

namespace gorgo {

constexpr int64_t STAMP_STRIDE = 65536;   // stamp = request * stride + (stride - 1 - position): root newest
constexpr int WAVE = 64;

// In-flight request record, linked per (replica, service slot) in dispatch order.
struct Rec {
    double done;       // time the completion event reaches the proxy
    int32_t next;      // next request on the same service slot, -1 = none
    int32_t tokens;    // input tokens counted in the load signal
};

// All mutable per-replay state in global memory is private to one workgroup; relaxed workgroup-scope
// atomics plus workgroup barriers between phases are what the memory model asks for.
template <class T>
__device__ __forceinline__ T ld(const T* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
template <class T>
__device__ __forceinline__ void st(T* p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ double readlane_f64(double v, int src) {
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)b, src);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), src);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

__device__ __forceinline__ int64_t readlane_i64(int64_t v, int src) {
    const int lo = __builtin_amdgcn_readlane((int)v, src);
    const int hi = __builtin_amdgcn_readlane((int)(v >> 32), src);
    return ((int64_t)hi << 32) | (unsigned int)lo;
}

// Unsigned minimum of x over the wavefront on the data-parallel-primitive path (no LDS round trip): shifts by
// 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of a row is broadcast into the next row (rows 1
// and 3), then lane 31 into rows 2 and 3; lane 63 holds the result.  Each step is one instruction (the moved
// operand is folded into the minimum); lanes without a source see 0xffffffff.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned dpp_min_u32(unsigned x) {
    const unsigned moved = (unsigned)__builtin_amdgcn_update_dpp((int)0xffffffffu, (int)x, CTRL, ROW_MASK, 0xf, false);
    return moved < x ? moved : x;
}
__device__ __forceinline__ unsigned wave_min_u32(unsigned x) {
    x = dpp_min_u32<0x111, 0xf>(x);   // row_shr:1
    x = dpp_min_u32<0x112, 0xf>(x);   // row_shr:2
    x = dpp_min_u32<0x114, 0xf>(x);   // row_shr:4
    x = dpp_min_u32<0x118, 0xf>(x);   // row_shr:8
    x = dpp_min_u32<0x142, 0xa>(x);   // row_bcast:15 into rows 1, 3
    x = dpp_min_u32<0x143, 0xc>(x);   // row_bcast:31 into rows 2, 3
    return (unsigned)__builtin_amdgcn_readlane((int)x, 63);
}

// Sum of x over the wavefront on the same path (lanes without a source add 0); the sum must fit 32 bits.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned dpp_add_u32(unsigned x) {
    return x + (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ unsigned wave_sum_u32(unsigned x) {
    x = dpp_add_u32<0x111, 0xf>(x);   // row_shr:1
    x = dpp_add_u32<0x112, 0xf>(x);   // row_shr:2
    x = dpp_add_u32<0x114, 0xf>(x);   // row_shr:4
    x = dpp_add_u32<0x118, 0xf>(x);   // row_shr:8: lane 15 of each row holds the row's sum
    x = dpp_add_u32<0x142, 0xa>(x);   // row_bcast:15 into rows 1, 3
    x = dpp_add_u32<0x143, 0xc>(x);   // row_bcast:31 into rows 2, 3
    return (unsigned)__builtin_amdgcn_readlane((int)x, 63);
}

// Lowest-index minimum over the lanes below `count` (count >= 1; values must not be NaN).  The values are
// compared through the usual order-preserving map of an IEEE double to an unsigned 64-bit key (zeros of
// either sign made equal first), high word first, then the low word among the lanes that tie on the high
// word: two 32-bit reductions instead of one on register pairs, and only one when the high words already decide
// (scores that differ by more than a part in a million).
__device__ __forceinline__ int wave_argmin(double v, int lane, int count) {
    const unsigned long long bits = (unsigned long long)__double_as_longlong(v + 0.0);
    const unsigned hi = (unsigned)(bits >> 32), lo = (unsigned)bits;
    const unsigned neg = (unsigned)((int)hi >> 31);
    const bool in = lane < count;
    const unsigned khi = in ? hi ^ (neg | 0x80000000u) : 0xffffffffu;
    const unsigned klo = lo ^ neg;
    const unsigned mhi = wave_min_u32(khi);
    const bool tie = in && khi == mhi;
    const unsigned long long ties = __ballot(tie);
    if ((ties & (ties - 1)) == 0) return __ffsll(ties) - 1;      // one lane holds the smallest high word: done
    const unsigned mlo = wave_min_u32(tie ? klo : 0xffffffffu);
    const unsigned long long at = __ballot(tie && klo == mlo);
    return __ffsll(at) - 1;
}

// Queue side of one replay.  Lane i owns replica i: its load signal q (Eq. 2: tokens of requests without a
// completion event at the proxy), its earliest pending completion and the set of its idle service slots live
// in that lane's registers, the B service slots themselves in LDS (slot b of replica i at index
// i * Bp + b, Bp = B rounded up to 8).  The in-flight requests of a slot form a FIFO (completion times
// increase along a slot); the two oldest are in LDS, deeper ones are Rec records in global memory linked in
// dispatch order, fetched when they become the second oldest.  Only the owning lane ever touches a
// replica's queue state, so every lane runs the same code on its own replica and no barrier is needed.
struct Queues {
    double* free_at;     // [R*Bp] time the service slot becomes free (+inf in the padding)
    double* h_done;      // [R*Bp] completion time of the oldest in-flight request (+inf: none)
    double* s_done;      // [R*Bp] ... of the second oldest
    int32_t* h_tok;      // [R*Bp] tokens of the oldest
    int32_t* s_tok;      // [R*Bp] tokens of the second oldest
    int32_t* s_next;     // [R*Bp] request after the second oldest (-1: none)
    int32_t* tail;       // [R*Bp] youngest request of the slot
    int32_t* depth;      // [R*Bp] requests in flight on the slot
    uint32_t* kv;        // [R*Bp] engine model: KV tokens held by the request that frees the slot at free_at
    int R, B, Bp, base;
    double my_min;       // earliest head completion among this lane's slots ...
    int my_min_k;        // ... and its slot
    unsigned long long idle;   // slots of this lane's replica with nothing in flight (bit b = slot b)
    double my_q;         // outstanding tokens of replica = lane (an integer below 2^53, exact in fp64)
    double my_cnt;       // requests in flight on replica = lane
    double my_last_start;      // engine model: admission time of the latest request of replica = lane

    static __host__ __device__ size_t bytes(int R, int B) {
        return (size_t)R * ((B + 7) & ~7) * (8 * 3 + 4 * 6);
    }

    __device__ void carve(unsigned char* lds, int R_, int B_, int lane) {
        R = R_;
        B = B_;
        Bp = (B + 7) & ~7;
        base = (lane < R ? lane : 0) * Bp;
        const int n = R * Bp;
        free_at = reinterpret_cast<double*>(lds);
        h_done = free_at + n;
        s_done = h_done + n;
        h_tok = reinterpret_cast<int32_t*>(s_done + n);
        s_tok = h_tok + n;
        s_next = s_tok + n;
        tail = s_next + n;
        depth = tail + n;
        kv = reinterpret_cast<uint32_t*>(depth + n);
    }

    __device__ void init(int lane) {
        for (int x = lane; x < R * Bp; x += WAVE) {
            free_at[x] = (x % Bp) < B ? 0.0 : INFINITY;
            h_done[x] = INFINITY;
            depth[x] = 0;
            tail[x] = -1;
            kv[x] = 0;
        }
        my_min = INFINITY;
        my_min_k = 0;
        idle = B >= 64 ? ~0ull : (1ull << B) - 1;
        my_q = 0.0;
        my_cnt = 0.0;
        my_last_start = 0.0;
    }

    // Drop requests whose completion event has reached the proxy (done <= t).
    __device__ void retire(double t, const Rec* rec) {
        while (__ballot(my_min <= t) != 0) {
            if (my_min <= t) {
                const int s = base + my_min_k;
                my_q -= (double)h_tok[s];
                my_cnt -= 1.0;
                const int d = depth[s];
                if (d > 1) {
                    h_done[s] = s_done[s];
                    h_tok[s] = s_tok[s];
                    if (d >= 3) {
                        const int x = s_next[s];
                        s_done[s] = ld(&rec[x].done);
                        s_tok[s] = ld(&rec[x].tokens);
                        s_next[s] = ld(&rec[x].next);
                    }
                } else {
                    h_done[s] = INFINITY;
                    idle |= 1ull << my_min_k;
                }
                depth[s] = d - 1;
                // earliest head of this lane's slots again
                double mn = INFINITY;
                int mk = 0;
                for (int b0 = 0; b0 < Bp; b0 += 8) {
                    double hd[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) hd[k] = h_done[base + b0 + k];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const bool lt = hd[k] < mn;
                        mn = lt ? hd[k] : mn;
                        mk = lt ? b0 + k : mk;
                    }
                }
                my_min = mn;
                my_min_k = mk;
            }
        }
    }

    // The completion times along a slot's in-flight list increase as long as a replica's round trip time is
    // constant.  When it changes between dispatches (probe epochs), a request can complete at the proxy before one
    // dispatched earlier on the same slot; the list is then kept sorted by completion time instead: this inserts
    // request r (completion `done`, `tok` tokens) into the list of slot s = base + k, which holds d >= 1 requests
    // the last of which completes after `done`.  An element that has to leave the two LDS positions moves into
    // the record of request r, which r itself does not need then.  tail[s] stays the record of the last element.
    __device__ void insert_sorted(int s, int k, int d, int64_t r, double done, int32_t tok, Rec* rec) {
        if (done < h_done[s] || (d >= 2 && done < s_done[s])) {
            // r goes into LDS; the element in second position, if any, moves to global memory behind it
            if (d >= 2) {
                st(&rec[r].done, s_done[s]);
                st(&rec[r].tokens, s_tok[s]);
                st(&rec[r].next, d >= 3 ? s_next[s] : (int32_t)-1);
                s_next[s] = (int32_t)r;
                if (d == 2) tail[s] = (int32_t)r;
            } else {
                s_next[s] = -1;
            }
            if (done < h_done[s]) {
                s_done[s] = h_done[s];
                s_tok[s] = h_tok[s];
                h_done[s] = done;
                h_tok[s] = tok;
                if (done < my_min) {
                    my_min = done;
                    my_min_k = k;
                }
            } else {
                s_done[s] = done;
                s_tok[s] = tok;
            }
        } else {
            // r goes between two elements further down (d >= 3): walk to the last one that completes no later
            int32_t prev = -1;               // -1: the second position
            int32_t x = s_next[s];
            for (int steps = 0; steps < d && x >= 0 && !(done < ld(&rec[x].done)); ++steps) {
                prev = x;
                x = ld(&rec[x].next);
            }
            st(&rec[r].done, done);
            st(&rec[r].tokens, tok);
            st(&rec[r].next, x);
            if (prev < 0) s_next[s] = (int32_t)r;
            else st(&rec[prev].next, (int32_t)r);
        }
        depth[s] = d + 1;
    }

    // Service of request r on replica `best` (the stated linear model; reproduces Eq. 1: ttft = rtt + wait +
    // prefill) on the earliest-free slot.  Which of several free slots takes the request changes no latency
    // and no load signal: a slot with nothing in flight has seen its completion event reach the proxy, so it
    // has been free since before any later arrival at the replica, exactly like the earliest-free one.  The
    // slots are therefore only searched for their earliest free time (lowest index on ties) when every slot
    // still has a request in flight.  `idle_then` is the set of idle slots at the request's time t; the lists
    // themselves may already have been retired further (to the next request's time), which only makes more
    // slots idle.  The chosen replica's lane works, its latencies are broadcast (LOCAL: left in that lane; `best`,
    // `t` and `uncached_mine` may then differ between lanes, for wavefronts that serve two replays at once).
    template <bool REORDER, bool LOCAL = false>
    __device__ void serve(int64_t r, int best, double t, double rtt_mine, int64_t uncached_mine, int64_t L, int64_t O,
                          double a_pf, double a_dec, Rec* rec, int lane, unsigned long long idle_then,
                          double* ttft_out, double* e2e_out) {
        double ttft = 0.0, e2e = 0.0;
        if (lane == best) {
            const double half = 0.5 * rtt_mine;
            const double arrive = t + half;
            double start = arrive;
            int k;
            if (idle_then != 0) {
                k = __ffsll(idle_then) - 1;
            } else {
                double fv = INFINITY;
                k = 0;
                for (int b0 = 0; b0 < Bp; b0 += 8) {
                    double v[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) v[j] = free_at[base + b0 + j];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const bool lt = v[j] < fv;
                        fv = lt ? v[j] : fv;
                        k = lt ? b0 + j : k;
                    }
                }
                start = arrive > fv ? arrive : fv;
            }
            const double pf = a_pf * (double)uncached_mine;
            const double first_tok = start + pf;
            const double dec = a_dec * (double)O;
            const double end = first_tok + dec;
            const double done = end + half;
            ttft = (first_tok + half) - t;
            e2e = done - t;
            const int s = base + k;
            free_at[s] = end;
            if ((idle >> k) & 1ull) {
                idle &= ~(1ull << k);
                h_done[s] = done;
                h_tok[s] = (int32_t)L;
                depth[s] = 1;
                tail[s] = (int32_t)r;
                if (done < my_min) {
                    my_min = done;
                    my_min_k = k;
                }
            } else {
                const int d = depth[s];         // at least 1
                if (REORDER && done < (d == 1 ? h_done[s] : (d == 2 ? s_done[s] : ld(&rec[tail[s]].done)))) {
                    insert_sorted(s, k, d, r, done, (int32_t)L, rec);
                } else {
                    if (d == 1) {
                        s_done[s] = done;
                        s_tok[s] = (int32_t)L;
                        s_next[s] = -1;
                    } else {
                        // third or deeper: goes to global memory, linked behind the youngest
                        st(&rec[r].done, done);
                        st(&rec[r].next, (int32_t)-1);
                        st(&rec[r].tokens, (int32_t)L);
                        if (d == 2) s_next[s] = (int32_t)r;
                        else st(&rec[tail[s]].next, (int32_t)r);
                    }
                    depth[s] = d + 1;
                    tail[s] = (int32_t)r;
                }
            }
            my_q += (double)L;
            my_cnt += 1.0;
        }
        *ttft_out = LOCAL ? ttft : readlane_f64(ttft, best);
        *e2e_out = LOCAL ? e2e : readlane_f64(e2e, best);
    }

    // Service of request r on replica `best` under the engine model of a replica (continuous batching, Sec. 2.2;
    // decode slow-down, Sec. 5 "Exploiting Continuous Batching"; replicas of different speed, Sec. 7).  Requests
    // are admitted in arrival order; a request holding L + O KV tokens is admitted at the first time s, not
    // before its arrival nor its predecessor's admission, at which fewer than B requests are running and either
    // none is or their KV tokens plus its own fit the replica's budget (0 = no budget); its decode takes
    // (a_dec * O) * (1 + slowdown * n) with n the requests running at s.  All requests admitted earlier have
    // started by s, so those running at s are the slots with free_at > s.  The slots of the chosen replica are
    // spread over the lanes (B <= 64): a ballot counts the running ones and finds a free slot, their tokens are
    // summed and the next time one ends is found with wavefront reductions; the scan is repeated from that time
    // until the request fits (at most B times: each repeat has one request fewer running).  The request takes
    // the lowest slot that is free at s; its record joins that slot's in-flight list.
    template <bool REORDER>
    __device__ void serve_engine(int64_t r, int best, double t, double rtt_mine, int64_t uncached_mine, int64_t L,
                                 int64_t O, double a_pf_mine, double a_dec_mine, double budget_mine, double slowdown,
                                 Rec* rec, int lane, double* ttft_out, double* e2e_out) {
        double ttft = 0.0, e2e = 0.0;
        // The scan runs across the lanes: lane j looks at slot j of the chosen replica (B <= 64).
        const double half = 0.5 * readlane_f64(rtt_mine, best);
        const double arrive = t + half;
        const double tokens = (double)(L + O);
        const double budget = readlane_f64(budget_mine, best);
        const double last_start = readlane_f64(my_last_start, best);
        double start = arrive > last_start ? arrive : last_start;
        const int slot = best * Bp + (lane < B ? lane : 0);
        const double f = lane < B ? free_at[slot] : 0.0;
        const unsigned h = lane < B ? kv[slot] : 0u;
        int n, k;
        for (int scans = 0;; ++scans) {
            const bool running = lane < B && f > start;
            const unsigned long long run_mask = __ballot(running);
            n = __popcll(run_mask);
            k = __ffsll(~run_mask & (B >= 64 ? ~0ull : (1ull << B) - 1)) - 1;
            if (n == 0) break;
            bool fits = n < B;
            if (fits && budget != 0.0) {
                // tokens held by the running requests: two 16-bit halves summed apart (each sum below 2^22)
                const unsigned lo = wave_sum_u32(running ? h & 0xffffu : 0u);
                const unsigned hi = wave_sum_u32(running ? h >> 16 : 0u);
                const double held = (double)hi * 65536.0 + (double)lo;
                fits = held + tokens <= budget;
            }
            if (fits || scans >= B) break;       // (the second test is not reached: every repeat has fewer running)
            // the next time a running request ends (running ones end after `start`: positive, finite)
            const double ends = running ? f : INFINITY;
            start = readlane_f64(ends, wave_argmin(ends, lane, WAVE));
        }
        k = k < 0 ? 0 : k;                       // (a free slot exists whenever fewer than B are running)
        if (lane == best) {
            my_last_start = start;
            const double pf = a_pf_mine * (double)uncached_mine;
            const double first_tok = start + pf;
            const double dec_alone = a_dec_mine * (double)O;
            const double factor = 1.0 + slowdown * (double)n;
            const double dec = dec_alone * factor;
            const double end = first_tok + dec;
            const double done = end + half;
            ttft = (first_tok + half) - t;
            e2e = done - t;
            const int s = base + k;
            free_at[s] = end;
            kv[s] = (uint32_t)(L + O);         // two counts below 2^31 each
            if ((idle >> k) & 1ull) {
                idle &= ~(1ull << k);
                h_done[s] = done;
                h_tok[s] = (int32_t)L;
                depth[s] = 1;
                if (done < my_min) {
                    my_min = done;
                    my_min_k = k;
                }
                tail[s] = (int32_t)r;
            } else {
                const int d = depth[s];         // at least 1
                if (REORDER && done < (d == 1 ? h_done[s] : (d == 2 ? s_done[s] : ld(&rec[tail[s]].done)))) {
                    insert_sorted(s, k, d, r, done, (int32_t)L, rec);
                } else {
                    if (d == 1) {
                        s_done[s] = done;
                        s_tok[s] = (int32_t)L;
                        s_next[s] = -1;
                    } else {
                        st(&rec[r].done, done);
                        st(&rec[r].next, (int32_t)-1);
                        st(&rec[r].tokens, (int32_t)L);
                        if (d == 2) s_next[s] = (int32_t)r;
                        else st(&rec[tail[s]].next, (int32_t)r);
                    }
                    depth[s] = d + 1;
                    tail[s] = (int32_t)r;
                }
            }
            my_q += (double)L;
            my_cnt += 1.0;
        }
        *ttft_out = readlane_f64(ttft, best);
        *e2e_out = readlane_f64(e2e, best);
    }
};

__device__ __forceinline__ unsigned long long ballot(bool c) { return __builtin_amdgcn_ballot_w64(c); }

// Queue side of one replay with one lane per service slot instead of one per replica, for shapes whose slots fit
// four passes of the wavefront (replicas x slots rounded up to a power of two <= 256): slot b of replica i is slot
// g = i * Bp + b, handled by lane g mod 64 in pass g / 64, so the slots of a replica are Bp neighbouring lanes of one
// pass.  Every slot keeps its list of in-flight requests as Queues does, but nothing has to be searched: "which
// slots' oldest request has completed by t" is one comparison per pass for all slots at once, and an idle slot of
// the chosen replica is one ballot.  The oldest request of every slot and the number in flight are in registers
// (one set per pass), and so are the time the slot becomes free and the youngest request of its list, so that the
// usual request -- nothing or one request retired, an idle slot taken -- needs no LDS access at all and the search
// for the earliest free slot no LDS round trip; the second oldest is in LDS at index g (every lane only ever
// addresses its own slots: no conflicts), deeper requests are Rec records in global memory.  The load signal and
// the request count stay per replica (lane = replica), as the cache side reads them.  Same arithmetic as Queues,
// operation for operation.
struct SlotHead {
    double done;         // completion time of the slot's oldest in-flight request (+inf: none)
    int tok;             // its tokens
    int depth;           // requests in flight on the slot
    int rep;             // replica of the slot (-1 where there is no slot)
    double free;         // time the slot becomes free (+inf where there is no slot)
    int tail;            // youngest request of the slot's list
};

// the slots with nothing in flight, per pass (to be handed to serve after the lists have been retired further)
struct SlotIdle {
    unsigned long long m0, m1, m2, m3;
};

// DEFER: the record that moves up in a deep list is fetched without waiting (see f_slot below).  The registers it
// arrives in live across the request loop; an instantiation in which the compiler copies them around on the usual
// path (it then has to wait for memory there, with whatever stores are under way) does better without.
template <bool DEFER>
struct SlotQueuesT {
    static constexpr int PASSES = 4;
    static constexpr int SLOTS = PASSES * WAVE;
    SlotHead H0, H1, H2, H3;
    double* s_done;      // [SLOTS] completion time of the second oldest
    int32_t* s_tok;      // [SLOTS] tokens of the second oldest
    int32_t* s_next;     // [SLOTS] request after the second oldest (-1: none)
    double my_q;         // outstanding tokens of replica = lane (an integer below 2^53, exact in fp64)
    double my_cnt;       // requests in flight on replica = lane
    int log2bp;
    // One record per lane can be on its way from global memory: the new second oldest of slot f_slot (-1: none), whose
    // LDS words are not valid until settle() has written them -- one request later, so that a slot whose list goes
    // deeper than two does not make the wavefront wait for memory when its oldest request completes.  (While the
    // record is on its way the slot's `next` word in LDS already works: -1, or the request queued behind the record
    // since; the loaded `next` replaces it only if the record had a successor when it was requested.)
    int f_slot, f_tok, f_next;
    double f_done;
    bool f_any;          // some lane has a record on its way (the same in every lane)

    // whether a model's slots fit: Bp = B rounded up to a power of two, R * Bp <= SLOTS
    static __host__ __device__ bool fits(int R, int B) {
        int bp = 1;
        while (bp < B) bp <<= 1;
        return R * bp <= SLOTS;
    }
    static __host__ __device__ size_t bytes() { return (size_t)SLOTS * (8 + 2 * 4); }

    __device__ __forceinline__ void init_head(SlotHead& h, int pass, int R, int B, int lane) {
        const int g = pass * WAVE + lane;
        const int i = g >> log2bp, b = g & ((1 << log2bp) - 1);
        h.rep = i < R && b < B ? i : -1;
        h.done = INFINITY;
        h.tok = 0;
        h.depth = 0;
        h.free = h.rep >= 0 ? 0.0 : INFINITY;
        h.tail = -1;
        s_done[g] = INFINITY;
        s_tok[g] = 0;
        s_next[g] = -1;
    }
    __device__ __forceinline__ void init(unsigned char* lds, int R, int B, int lane) {
        s_done = reinterpret_cast<double*>(lds);
        s_tok = reinterpret_cast<int32_t*>(s_done + SLOTS);
        s_next = s_tok + SLOTS;
        log2bp = 0;
        while ((1 << log2bp) < B) ++log2bp;
        init_head(H0, 0, R, B, lane);
        init_head(H1, 1, R, B, lane);
        init_head(H2, 2, R, B, lane);
        init_head(H3, 3, R, B, lane);
        my_q = 0.0;
        my_cnt = 0.0;
        f_slot = f_next = -1;
        f_any = false;
        f_tok = 0;
        f_done = INFINITY;
    }

    // The record that was requested by an earlier pop has arrived: it becomes the slot's second oldest.
    __device__ __forceinline__ void settle() {
        if (!DEFER || !f_any) return;
        f_any = false;
        if (f_slot >= 0) {
            s_done[f_slot] = f_done;
            s_tok[f_slot] = f_tok;
            if (f_next >= 0) s_next[f_slot] = f_next;
        }
        f_slot = -1;
    }

    // The slots of one pass whose oldest request has completed by t drop it (and whatever else of theirs has
    // completed by t).  A slot with a single request in flight -- the usual case -- only changes its registers.
    __device__ __forceinline__ void pop(SlotHead& h, int g, bool due, double t, const Rec* rec, int lane) {
        const unsigned long long mask = ballot(due);
        if (mask == 0) return;
        // load signal and request count of the replicas concerned: one scalar step per completed request
        for (unsigned long long rest = mask; rest != 0; rest &= rest - 1) {
            const int l = __builtin_ctzll(rest);
            const int tok = __builtin_amdgcn_readlane(h.tok, l);
            const int i = __builtin_amdgcn_readlane(h.rep, l);
            my_q -= lane == i ? (double)tok : 0.0;
            my_cnt -= lane == i ? 1.0 : 0.0;
        }
        const int d = h.depth;
        double n_done = INFINITY;
        int n_tok = 0, n_depth = 0;
        if (ballot(due && d > 1) != 0) {
            // slots with more in flight: the list moves up, as long as its head has completed as well
            double dq = 0.0, dc = 0.0;          // what further leaves the load signal of this lane's slot
            if (due && d > 1) {
                n_done = s_done[g];
                n_tok = s_tok[g];
                n_depth = d - 1;
                int x = n_depth >= 2 ? s_next[g] : -1;      // the request that moves into second position
                if (DEFER && !(n_done <= t) && x >= 0 && f_slot < 0) {
                    // the usual case of a deep list: the new head stays, its successor is requested and settled later
                    f_slot = g;
                    s_next[g] = -1;
                    f_done = ld(&rec[x].done);
                    f_tok = ld(&rec[x].tokens);
                    f_next = ld(&rec[x].next);
                } else {
                    for (;;) {
                        const bool again = n_depth > 0 && n_done <= t;     // the new head has completed too
                        if (again) {
                            dq += (double)n_tok;
                            dc += 1.0;
                            --n_depth;
                        }
                        double x_done = INFINITY;
                        int x_tok = 0, x_next = -1;
                        if (x >= 0) {
                            x_done = ld(&rec[x].done);
                            x_tok = ld(&rec[x].tokens);
                            x_next = ld(&rec[x].next);
                        }
                        if (!again) {
                            // settled: x (if any) is the second oldest
                            s_done[g] = x_done;
                            s_tok[g] = x_tok;
                            s_next[g] = x_next;
                            break;
                        }
                        n_done = x_done;            // x moves up to the head (+inf when the list is empty)
                        n_tok = x_tok;
                        x = x_next;
                    }
                }
            }
            if (DEFER) f_any = f_any || ballot(f_slot >= 0) != 0;
            // (further completions are rare: their tokens reach the replicas' lanes one slot at a time)
            for (unsigned long long rest = ballot(dc != 0.0); rest != 0; rest &= rest - 1) {
                const int l = __builtin_ctzll(rest);
                const double q1 = readlane_f64(dq, l), c1 = readlane_f64(dc, l);
                const int i = __builtin_amdgcn_readlane(h.rep, l);
                my_q -= lane == i ? q1 : 0.0;
                my_cnt -= lane == i ? c1 : 0.0;
            }
        }
        h.done = due ? n_done : h.done;
        h.tok = due ? n_tok : h.tok;
        h.depth = due ? n_depth : d;
    }

    // Drop requests whose completion event has reached the proxy (done <= t).
    __device__ __forceinline__ void retire(double t, const Rec* rec, int lane) {
        const bool due0 = H0.done <= t, due1 = H1.done <= t, due2 = H2.done <= t, due3 = H3.done <= t;
        if (ballot(due0 || due1 || due2 || due3) == 0) return;
        settle();
        pop(H0, lane, due0, t, rec, lane);
        pop(H1, WAVE + lane, due1, t, rec, lane);
        pop(H2, 2 * WAVE + lane, due2, t, rec, lane);
        pop(H3, 3 * WAVE + lane, due3, t, rec, lane);
    }

    // Service of request r on replica `best` (the stated linear model; reproduces Eq. 1: ttft = rtt + wait +
    // prefill).  A slot of the replica with nothing in flight has been free since before any later arrival at the
    // replica (its completion event has already reached the proxy), and which of several such slots takes the
    // request changes no latency and no load signal; only when every slot has a request in flight are they
    // searched for the earliest free time (lowest index on ties).  rtt_best: the chosen replica's round trip time.
    // idle_then: the slots of this pass that had nothing in flight at the request's time t (the lists may have been
    // retired further since, to the next request's time, which only makes more slots idle).  The latencies come
    // back the same in every lane, and so does the time the request's completion reaches the proxy.
    __device__ __forceinline__ void serve_in(SlotHead& h, int g, unsigned long long idle_then, int64_t r, int best, double t,
                                            double rtt_best, int uncached, int L, int O, double a_pf, double a_dec, Rec* rec,
                                            int lane, double* ttft_out, double* e2e_out, double* done_out) {
        const bool mine = h.rep == best;
        const int d = h.depth;
        const double half = 0.5 * rtt_best;
        const double arrive = t + half;
        double start = arrive;
        int k;
        const unsigned long long idle = ballot(mine) & idle_then;
        if (idle != 0) {
            k = __builtin_ctzll(idle);
        } else {
            // every slot is busy: the earliest free one (times are >= 0: the order of the bits is the order of the
            // values; mostly one slot alone holds the smallest high word and the low words need not be looked at)
            const double f = mine ? h.free : INFINITY;
            const unsigned long long bits = (unsigned long long)__double_as_longlong(f);
            const unsigned hi = (unsigned)(bits >> 32), lo = (unsigned)bits;
            const unsigned mhi = wave_min_u32(hi);
            const bool tie = hi == mhi;
            const unsigned long long ties = ballot(tie);
            if (__builtin_popcountll(ties) == 1) {
                k = __builtin_ctzll(ties);
            } else {
                const unsigned mlo = wave_min_u32(tie ? lo : 0xffffffffu);
                k = __builtin_ctzll(ballot(tie && lo == mlo));
            }
            const double fv = readlane_f64(f, k);
            start = arrive > fv ? arrive : fv;
        }
        const double pf = a_pf * (double)uncached;
        const double first_tok = start + pf;
        const double dec = a_dec * (double)O;
        const double end = first_tok + dec;
        const double done = end + half;
        *ttft_out = (first_tok + half) - t;
        *e2e_out = done - t;
        *done_out = done;
        const bool on = lane == k;
        if (ballot(on && d > 0) != 0) {
            // the slot still has requests in flight: the new one queues behind them
            if (on) {
                if (d == 1) {
                    s_done[g] = done;
                    s_tok[g] = L;
                    s_next[g] = -1;
                } else {
                    // third or deeper: goes to global memory, linked behind the youngest
                    st(&rec[r].done, done);
                    st(&rec[r].next, (int32_t)-1);
                    st(&rec[r].tokens, (int32_t)L);
                    if (d == 2) s_next[g] = (int32_t)r;      // (behind the second oldest, whose record may still be on its way)
                    else st(&rec[h.tail].next, (int32_t)r);
                }
            }
        }
        h.free = on ? end : h.free;
        h.tail = on ? (int)r : h.tail;
        h.done = on && d == 0 ? done : h.done;
        h.tok = on && d == 0 ? L : h.tok;
        h.depth = on ? d + 1 : d;
        my_q += lane == best ? (double)L : 0.0;
        my_cnt += lane == best ? 1.0 : 0.0;
    }
    __device__ __forceinline__ SlotIdle idle_slots() const {
        return SlotIdle{ballot(H0.depth == 0), ballot(H1.depth == 0), ballot(H2.depth == 0), ballot(H3.depth == 0)};
    }
    __device__ __forceinline__ void serve(int64_t r, int best, double t, double rtt_best, int uncached, int L, int O,
                                          double a_pf, double a_dec, Rec* rec, int lane, const SlotIdle& idle_then,
                                          double* ttft_out, double* e2e_out, double* done_out) {
        switch ((best << log2bp) >> 6) {       // the pass that holds the replica's slots
            case 0: serve_in(H0, lane, idle_then.m0, r, best, t, rtt_best, uncached, L, O, a_pf, a_dec, rec, lane, ttft_out, e2e_out, done_out); break;
            case 1: serve_in(H1, WAVE + lane, idle_then.m1, r, best, t, rtt_best, uncached, L, O, a_pf, a_dec, rec, lane, ttft_out, e2e_out, done_out); break;
            case 2: serve_in(H2, 2 * WAVE + lane, idle_then.m2, r, best, t, rtt_best, uncached, L, O, a_pf, a_dec, rec, lane, ttft_out, e2e_out, done_out); break;
            default: serve_in(H3, 3 * WAVE + lane, idle_then.m3, r, best, t, rtt_best, uncached, L, O, a_pf, a_dec, rec, lane, ttft_out, e2e_out, done_out); break;
        }
    }
};

using SlotQueues = SlotQueuesT<true>;

// Weighted score of Eq. 3 for one replica, in the fixed association (w_rtt*rtt + w_prefill*pf) + w_queue*qd
// with every product and sum rounded on its own.  The first two terms do not depend on the load signal and
// can be formed before it is known.
__device__ __forceinline__ double eq3_without_queue(double w_rtt, double w_prefill, double rtt, double a_pf,
                                                    int uncached) {
    const double pf = a_pf * (double)uncached;
    const double s_rtt = w_rtt * rtt;
    const double s_pf = w_prefill * pf;
    return s_rtt + s_pf;
}
__device__ __forceinline__ double eq3_with_queue(double rtt_and_prefill, double w_queue, double a_pf,
                                                 double outstanding) {
    const double qd = a_pf * outstanding;
    const double s_q = w_queue * qd;
    return rtt_and_prefill + s_q;
}
__device__ __forceinline__ double eq3_score(double w_rtt, double w_prefill, double w_queue, double rtt, double a_pf,
                                            int uncached, double outstanding) {
    return eq3_with_queue(eq3_without_queue(w_rtt, w_prefill, rtt, a_pf, uncached), w_queue, a_pf, outstanding);
}

// Index of the next request after `after` (exclusive) and before `limit` that was routed to `replica`, or
// `limit` if there is none: the per-replica touch log is the route array itself.
__device__ __forceinline__ int64_t next_routed(const uint8_t* route, int64_t after, int64_t limit, int replica,
                                               int lane) {
    int64_t x = after + 1;
    while (x < limit) {
        const int64_t y = x + lane;
        const bool hitb = y < limit && ld(&route[y]) == (uint8_t)replica;
        const uint64_t mk = __ballot(hitb);
        if (mk) return x + __ffsll((unsigned long long)mk) - 1;
        x += WAVE;
    }
    return limit;
}

}  // namespace gorgo

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

struct Best {
    double v;
    int idx;
};

// Cross-lane move through the data-parallel-primitive path (no LDS round trip).  Lanes whose source is
// outside the row, or that row_mask excludes, keep their own value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double x) {
    const long long b = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_update_dpp((int)b, (int)b, CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp((int)(b >> 32), (int)(b >> 32), CTRL, ROW_MASK, 0xf, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
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

__device__ __forceinline__ double min_keep_first(double x, double y) { return y < x ? y : x; }

// Minimum over the 64 lanes: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of a row is
// broadcast into the next row (rows 1 and 3), then lane 31 into rows 2 and 3; lane 63 holds the result.
__device__ __forceinline__ double wave_min_f64(double x) {
    x = min_keep_first(x, dpp_f64<0x111, 0xf>(x));   // row_shr:1
    x = min_keep_first(x, dpp_f64<0x112, 0xf>(x));   // row_shr:2
    x = min_keep_first(x, dpp_f64<0x114, 0xf>(x));   // row_shr:4
    x = min_keep_first(x, dpp_f64<0x118, 0xf>(x));   // row_shr:8
    x = min_keep_first(x, dpp_f64<0x142, 0xa>(x));   // row_bcast:15 into rows 1, 3
    x = min_keep_first(x, dpp_f64<0x143, 0xc>(x));   // row_bcast:31 into rows 2, 3
    return readlane_f64(x, 63);
}

// Lowest-index minimum over the lanes below `count` (count >= 1; values must not be NaN).
__device__ __forceinline__ Best wave_argmin(double v, int lane, int count) {
    const double mine = lane < count ? v : INFINITY;
    const double mn = wave_min_f64(mine);
    const unsigned long long at = __ballot(lane < count && mine == mn);
    return Best{mn, __ffsll(at) - 1};
}

// Queue side of one replay.  Lane i owns replica i: its load signal q (Eq. 2: tokens of requests without a
// completion event at the proxy), its earliest pending completion and its earliest-free service slot live
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
    int R, B, Bp, base;
    double my_min;       // earliest head completion among this lane's slots ...
    int my_min_k;        // ... and its slot
    double f_min;        // earliest free time among this lane's slots (lowest slot on ties) ...
    int f_k;             // ... and its slot
    double my_q;         // outstanding tokens of replica = lane (an integer below 2^53, exact in fp64)

    static __host__ __device__ size_t bytes(int R, int B) {
        return (size_t)R * ((B + 7) & ~7) * (8 * 3 + 4 * 5);
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
    }

    __device__ void init(int lane) {
        for (int x = lane; x < R * Bp; x += WAVE) {
            free_at[x] = (x % Bp) < B ? 0.0 : INFINITY;
            h_done[x] = INFINITY;
            depth[x] = 0;
            tail[x] = -1;
        }
        my_min = INFINITY;
        my_min_k = 0;
        f_min = 0.0;
        f_k = 0;
        my_q = 0.0;
    }

    // Drop requests whose completion event has reached the proxy (done <= t).
    __device__ void retire(double t, const Rec* rec) {
        while (__ballot(my_min <= t) != 0) {
            if (my_min <= t) {
                const int s = base + my_min_k;
                my_q -= (double)h_tok[s];
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

    // Service of request r on replica `best` (the stated linear model; reproduces Eq. 1: ttft = rtt + wait +
    // prefill): earliest-free slot, lowest index on ties.  Every lane evaluates the schedule its own replica
    // would give; the chosen replica's lane commits it and its latencies are broadcast.
    __device__ void serve(int64_t r, int best, double t, double rtt_mine, int64_t uncached_mine, int64_t L, int64_t O,
                          double a_pf, double a_dec, Rec* rec, int lane, double* ttft_out, double* e2e_out) {
        const double half = 0.5 * rtt_mine;
        const double arrive = t + half;
        const double start = arrive > f_min ? arrive : f_min;
        const double pf = a_pf * (double)uncached_mine;
        const double first_tok = start + pf;
        const double dec = a_dec * (double)O;
        const double end = first_tok + dec;
        const double done = end + half;
        const double ttft = (first_tok + half) - t;
        const double e2e = done - t;
        if (lane == best) {
            const int s = base + f_k;
            free_at[s] = end;
            const int d = depth[s];
            if (d == 0) {
                h_done[s] = done;
                h_tok[s] = (int32_t)L;
                if (done < my_min) {
                    my_min = done;
                    my_min_k = f_k;
                }
            } else if (d == 1) {
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
            tail[s] = (int32_t)r;
            depth[s] = d + 1;
            my_q += (double)L;
            // earliest-free slot of this replica again
            double fv = INFINITY;
            int fk = 0;
            for (int b0 = 0; b0 < Bp; b0 += 8) {
                double v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] = free_at[base + b0 + k];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const bool lt = v[k] < fv;
                    fv = lt ? v[k] : fv;
                    fk = lt ? b0 + k : fk;
                }
            }
            f_min = fv;
            f_k = fk;
        }
        *ttft_out = readlane_f64(ttft, best);
        *e2e_out = readlane_f64(e2e, best);
    }
};

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

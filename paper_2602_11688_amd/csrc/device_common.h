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

// Queue side of one replay (LDS): B service slots per replica, the in-flight requests of every slot as a
// FIFO (completion times increase along a slot), and the load signal q (Eq. 2: tokens of requests without a
// completion event at the proxy).  The two oldest requests of a slot live in LDS; deeper ones are Rec
// records in global memory linked in dispatch order, fetched when they become the second oldest.
struct Queues {
    double* free_at;     // [R*B] time the service slot becomes free
    double* h_done;      // [R*B] completion time of the oldest in-flight request (+inf: none)
    double* s_done;      // [R*B] ... of the second oldest
    int64_t* q;          // [R]
    int32_t* h_tok;      // [R*B] tokens of the oldest
    int32_t* s_tok;      // [R*B] tokens of the second oldest
    int32_t* s_next;     // [R*B] request after the second oldest (-1: none)
    int32_t* tail;       // [R*B] youngest request of the slot
    int32_t* depth;      // [R*B] requests in flight on the slot
    uint8_t* rep_of;     // [R*B] replica of the slot
    int R, B;

    static __host__ __device__ size_t bytes(int R, int B) {
        return (size_t)R * B * (8 * 3 + 4 * 5) + (size_t)R * 8 + (((size_t)R * B + 3) & ~(size_t)3);
    }

    __device__ void carve(unsigned char* lds, int R_, int B_) {
        R = R_;
        B = B_;
        const int RB = R * B;
        free_at = reinterpret_cast<double*>(lds);
        h_done = free_at + RB;
        s_done = h_done + RB;
        q = reinterpret_cast<int64_t*>(s_done + RB);
        h_tok = reinterpret_cast<int32_t*>(q + R);
        s_tok = h_tok + RB;
        s_next = s_tok + RB;
        tail = s_next + RB;
        depth = tail + RB;
        rep_of = reinterpret_cast<uint8_t*>(depth + RB);
    }

    __device__ void init(int lane) {
        for (int s = lane; s < R * B; s += WAVE) {
            free_at[s] = 0.0;
            h_done[s] = INFINITY;
            depth[s] = 0;
            tail[s] = -1;
            rep_of[s] = (uint8_t)(s / B);
        }
        for (int i = lane; i < R; i += WAVE) q[i] = 0;
    }

    // Drop requests whose completion event has reached the proxy (done <= t).  `my_min` is a per-lane
    // register holding the earliest head completion among the slots this lane owns (slot s belongs to lane
    // s % 64), so the common case -- nothing to retire -- touches no memory.
    __device__ void retire(double t, const Rec* rec, int lane, double& my_min) {
        if (__ballot(my_min <= t) == 0) return;
        if (my_min <= t) {
            double mn = INFINITY;
            for (int s = lane; s < R * B; s += WAVE) {
                double hd = h_done[s];
                while (hd <= t) {
                    atomicAdd(reinterpret_cast<unsigned long long*>(&q[rep_of[s]]),
                              (unsigned long long)(-(int64_t)h_tok[s]));
                    const int d = depth[s];
                    if (d == 1) {
                        hd = INFINITY;
                    } else {
                        hd = s_done[s];
                        h_tok[s] = s_tok[s];
                        if (d >= 3) {
                            const int x = s_next[s];
                            s_done[s] = ld(&rec[x].done);
                            s_tok[s] = ld(&rec[x].tokens);
                            s_next[s] = ld(&rec[x].next);
                        }
                    }
                    h_done[s] = hd;
                    depth[s] = d - 1;
                }
                mn = hd < mn ? hd : mn;
            }
            my_min = mn;
        }
        __syncthreads();
    }

    // Service of request r on replica `best` (the stated linear model; reproduces Eq. 1: ttft = rtt + wait +
    // prefill): earliest-free slot, lowest index on ties.  Lane 0 updates the state; the caller places a
    // barrier before the next use.
    __device__ void serve(int64_t r, int best, double t, double rtt_best, int64_t uncached, int64_t L, int64_t O,
                          double a_pf, double a_dec, Rec* rec, int lane, double& my_min, double* ttft_out,
                          double* e2e_out) {
        const Best slot = wave_argmin(lane < B ? free_at[best * B + lane] : INFINITY, lane, B);
        const double half = 0.5 * rtt_best;
        const double arrive = t + half;
        const double start = arrive > slot.v ? arrive : slot.v;
        const double pf = a_pf * (double)uncached;
        const double first_tok = start + pf;
        const double dec = a_dec * (double)O;
        const double end = first_tok + dec;
        const double done = end + half;
        *ttft_out = (first_tok + half) - t;
        *e2e_out = done - t;
        const int s = best * B + slot.idx;
        const int d = depth[s];
        if (d == 0 && lane == (s & (WAVE - 1))) my_min = done < my_min ? done : my_min;   // new head of the slot
        if (lane == 0) {
            free_at[s] = end;
            if (d == 0) {
                h_done[s] = done;
                h_tok[s] = (int32_t)L;
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
            q[best] += L;
        }
    }
};

// Weighted score of Eq. 3 for one replica, in the fixed association (w_rtt*rtt + w_prefill*pf) + w_queue*qd
// with every product and sum rounded on its own.
__device__ __forceinline__ double eq3_score(double w_rtt, double w_prefill, double w_queue, double rtt, double a_pf,
                                            int64_t uncached, int64_t outstanding) {
    const double pf = a_pf * (double)uncached;
    const double qd = a_pf * (double)outstanding;
    const double s_rtt = w_rtt * rtt;
    const double s_pf = w_prefill * pf;
    const double s_q = w_queue * qd;
    return (s_rtt + s_pf) + s_q;
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

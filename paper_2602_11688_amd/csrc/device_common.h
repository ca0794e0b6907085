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

// Lowest-index minimum over the wavefront.
__device__ __forceinline__ Best wave_argmin(double v, int idx) {
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        double ov = __shfl_xor(v, d);
        int oi = __shfl_xor(idx, d);
        if (ov < v || (ov == v && oi < idx)) {
            v = ov;
            idx = oi;
        }
    }
    return Best{v, idx};
}

// Queue side of one replay (LDS): B service slots per replica, the in-flight requests of every slot as a
// FIFO linked through the Rec array (completion times increase along a slot), and the load signal q
// (Eq. 2: tokens of requests without a completion event at the proxy).
struct Queues {
    double* free_at;     // [R*B] time the service slot becomes free
    double* head_done;   // [R*B] completion time of the oldest in-flight request of the slot (+inf: none)
    int64_t* q;          // [R]
    int32_t* head;       // [R*B]
    int32_t* tail;       // [R*B]
    int R, B;

    static __host__ __device__ size_t bytes(int R, int B) {
        return (size_t)R * B * (8 + 8 + 4 + 4) + (size_t)R * 8;
    }

    __device__ void carve(unsigned char* lds, int R_, int B_) {
        R = R_;
        B = B_;
        const int RB = R * B;
        free_at = reinterpret_cast<double*>(lds);
        head_done = free_at + RB;
        q = reinterpret_cast<int64_t*>(head_done + RB);
        head = reinterpret_cast<int32_t*>(q + R);
        tail = head + RB;
    }

    __device__ void init(int lane) {
        for (int s = lane; s < R * B; s += WAVE) {
            free_at[s] = 0.0;
            head_done[s] = INFINITY;
            head[s] = -1;
            tail[s] = -1;
        }
        for (int i = lane; i < R; i += WAVE) q[i] = 0;
    }

    // Drop requests whose completion event has reached the proxy (done <= t).  Ends with a barrier.
    __device__ void retire(double t, const Rec* rec, int lane) {
        for (int s = lane; s < R * B; s += WAVE) {
            while (head_done[s] <= t) {
                const int h = head[s];
                const int32_t nx = ld(&rec[h].next);
                const int32_t tok = ld(&rec[h].tokens);
                atomicAdd(reinterpret_cast<unsigned long long*>(&q[s / B]), (unsigned long long)(-(int64_t)tok));
                head[s] = nx;
                if (nx < 0) {
                    head_done[s] = INFINITY;
                    tail[s] = -1;
                } else {
                    head_done[s] = ld(&rec[nx].done);
                }
            }
        }
        __syncthreads();
    }

    // Service of request r on replica `best` (the stated linear model; reproduces Eq. 1: ttft = rtt + wait +
    // prefill): earliest-free slot, lowest index on ties.  Lane 0 updates the state; the caller places a
    // barrier before the next use.
    __device__ void serve(int64_t r, int best, double t, double rtt_best, int64_t uncached, int64_t L, int64_t O,
                          double a_pf, double a_dec, Rec* rec, int lane, double* ttft_out, double* e2e_out) {
        const Best slot = wave_argmin(lane < B ? free_at[best * B + lane] : INFINITY, lane < B ? lane : 255);
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
        if (lane == 0) {
            const int s = best * B + slot.idx;
            free_at[s] = end;
            st(&rec[r].done, done);
            st(&rec[r].next, (int32_t)-1);
            st(&rec[r].tokens, (int32_t)L);
            const int tl = tail[s];
            if (tl >= 0) {
                st(&rec[tl].next, (int32_t)r);
            } else {
                head[s] = (int32_t)r;
                head_done[s] = done;
            }
            tail[s] = (int32_t)r;
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

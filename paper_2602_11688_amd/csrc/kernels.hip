// Device side: the block-table replay kernel (one wavefront per replay), table fill, exact percentile
// selection, and the launches (the segment-row replay kernel is in replay_segments.h).
//
// The replay kernel follows the request loop of the routing policy (Sec. 2.2-2.3): retire completed
// requests from the load signal (Eq. 2), longest-prefix match of the request's blocks against every
// replica's cache (the x_r \ c_i of Eq. 1), weighted score (Eq. 3), lowest-index minimum over replicas, cache
// and queue update on the chosen replica, and the stated linear service model.  Replays are independent,
// so the grid is one 64-lane workgroup per replay; inside a replay the lanes spread over replicas (first-
// block probes, scores), over the blocks of the request (prefix match, cache update, eviction walk) and over
// the service slots (retirement, earliest-free slot).
//
// Decision arithmetic is fp64 with every product and sum rounded separately (built with -ffp-contract=off)
// in the association (w_rtt*rtt + w_prefill*pf) + w_queue*qd, so that routes are reproducible bit for bit.
#include <atomic>
#include <hip/hip_runtime.h>
#include <mutex>

#include <cmath>
#include <cstdint>
#include <string>

#include "device_common.h"
#include "internal.h"
#include "replay_segments.h"
#include "replay_segments_packed.h"

namespace gorgo {

namespace {

// One cache-table slot.  key 0 = never used (then stamp = -1).  An entry is cached iff stamp >= tau of its
// replica; entries below tau are evicted garbage whose slots can be taken over by inserts.
struct Slot {
    uint64_t key;
    int64_t stamp;
};

struct ReplayArgs {
    const int64_t* ts;
    const int32_t* in_len;
    const int32_t* out_len;
    const int64_t* blk_off;
    const uint32_t* key;
    const uint8_t* first;
    int64_t N;
    int32_t R, B;
    int64_t C;
    int64_t cap;
    int32_t cap_log2;
    int32_t block_tokens;
    double a_pf, a_dec;
    const double* rtt;
    const double* params;
    const double* scale;
    Slot* tables;   // [P][R][cap]
    Slot* spare;    // [P][cap]
    Rec* rec;       // [P][N]
    uint8_t* route; // [P][N] never null (workspace stand-in when the caller does not want it)
    uint16_t* hit;  // nullable
    double* ttft;   // nullable
    double* e2e;    // nullable
};

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

__device__ __forceinline__ bool is_cached(const Slot* tab, uint64_t key, int64_t tau, uint64_t mask, int cap_log2) {
    int64_t s = find_slot(tab, key, mask, cap_log2);
    return s >= 0 && ld(&tab[s].stamp) >= tau;
}

// Takes over the first never-used or evicted slot of the probe sequence.  Returns true when a never-used
// slot was consumed.  Only called for keys known to be physically absent, by lanes with distinct keys.
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

__global__ void __launch_bounds__(WAVE) replay_blocks_kernel(ReplayArgs a) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int lane = threadIdx.x;
    const int p = blockIdx.x;
    const int R = a.R, B = a.B;
    const int64_t N = a.N;
    const uint64_t mask = (uint64_t)a.cap - 1;
    const int cap_log2 = a.cap_log2;

    Queues Q;
    Q.carve(lds_raw, R, B, lane);
    int64_t* tau = reinterpret_cast<int64_t*>(lds_raw + Queues::bytes(R, B));   // [R] eviction threshold
    int32_t* live = reinterpret_cast<int32_t*>(tau + R);          // [R] cached blocks
    int32_t* used = live + R;                                     // [R] slots ever used since the last rebuild
    int32_t* cur_r = used + R;                                    // [R] eviction cursor: request ...
    int32_t* cur_k = cur_r + R;                                   // [R] ... and position (blocks >= cur_k are gone)

    Q.init(lane);
    for (int i = lane; i < R; i += WAVE) {
        tau[i] = 0;
        live[i] = 0;
        used[i] = 0;
        cur_r[i] = -1;
        cur_k[i] = 0;
    }
    __syncthreads();

    const double w_rtt = a.params[3 * (size_t)p + 0];
    const double w_prefill = a.params[3 * (size_t)p + 1];
    const double w_queue = a.params[3 * (size_t)p + 2];
    const double sc = a.scale[p];
    const double my_rtt = lane < R ? a.rtt[lane] : 0.0;

    Slot* const tables = a.tables + (size_t)p * R * a.cap;
    Slot* const spare = a.spare + (size_t)p * a.cap;
    Rec* const rec = a.rec + (size_t)p * N;
    uint8_t* const route = a.route + (size_t)p * N;
    const int64_t rebuild_at = a.cap - a.cap / 8;

    for (int64_t r = 0; r < N; ++r) {
        const int64_t off = a.blk_off[r];
        const int n = (int)(a.blk_off[r + 1] - off);
        const int64_t L = a.in_len[r];
        const int64_t O = a.out_len[r];
        const double t = (double)a.ts[r] * sc;     // time scale: gaps scale linearly

        Q.retire(t, rec);

        // ---- prefix match: first block on every replica, then the whole list on replicas that hold it
        int my_m = 0;
        {
            bool has0 = false;
            if (n > 0 && lane < R)
                has0 = is_cached(tables + (size_t)lane * a.cap, a.key[off], tau[lane], mask, cap_log2);
            uint64_t holders = __ballot(has0);
            while (holders) {
                const int i = __ffsll((unsigned long long)holders) - 1;
                holders &= holders - 1;
                const Slot* tab = tables + (size_t)i * a.cap;
                const int64_t tau_i = tau[i];
                int m = 0;
                for (int base = 0; base < n; base += WAVE) {
                    const int k = base + lane;
                    const bool ok = k < n && is_cached(tab, a.key[off + k], tau_i, mask, cap_log2);
                    const uint64_t got = __ballot(ok);
                    const int width = n - base < WAVE ? n - base : WAVE;
                    const uint64_t want = width == WAVE ? ~0ull : ((1ull << width) - 1);
                    if (got == want) {
                        m += width;
                    } else {
                        m += __ffsll((unsigned long long)(~got)) - 1;
                        break;
                    }
                }
                if (lane == i) my_m = m;
            }
        }

        // ---- score (Eq. 3) and lowest-index minimum
        int64_t my_u = 0;
        double my_score = INFINITY;
        if (lane < R) {
            int64_t hit_tok = (int64_t)a.block_tokens * my_m;
            if (hit_tok > L) hit_tok = L;
            my_u = L - hit_tok;
            my_score = eq3_score(w_rtt, w_prefill, w_queue, my_rtt, a.a_pf, (int)my_u, Q.my_q);
        }
        const int best = wave_argmin(my_score, lane, R);
        const int m_best = __builtin_amdgcn_readlane(my_m, best);
        if (lane == 0) st(&route[r], (uint8_t)best);

        // ---- cache update on the chosen replica
        Slot* const tab = tables + (size_t)best * a.cap;
        if ((int64_t)used[best] + n > rebuild_at) {
            // compact: keep cached entries only, so that never-used slots exist again
            const int64_t tau_b = tau[best];
            int64_t kept = 0;
            for (int64_t base = 0; base < a.cap; base += WAVE) {
                const uint64_t k = ld(&tab[base + lane].key);
                const int64_t s = ld(&tab[base + lane].stamp);
                const bool keep = k != 0 && s >= tau_b;
                const uint64_t mk = __ballot(keep);
                if (keep) {
                    const int64_t pos = kept + __popcll(mk & ((1ull << lane) - 1));
                    st(&spare[pos].key, k);
                    st(&spare[pos].stamp, s);
                }
                kept += __popcll(mk);
            }
            __syncthreads();
            for (int64_t base = 0; base < a.cap; base += WAVE) {
                st(&tab[base + lane].key, (uint64_t)0);
                st(&tab[base + lane].stamp, (int64_t)-1);
            }
            __syncthreads();
            for (int64_t base = 0; base < kept; base += WAVE) {
                if (base + lane < kept)
                    insert_new(tab, ld(&spare[base + lane].key), ld(&spare[base + lane].stamp), 0, mask, cap_log2);
                __syncthreads();
            }
            if (lane == 0) used[best] = (int32_t)kept;
            __syncthreads();
        }
        {
            const int64_t tau_b = tau[best];
            int add_live = 0, add_used = 0;
            for (int base = 0; base < n; base += WAVE) {
                const int k = base + lane;
                const bool mine = k < n && a.first[off + k] != 0;
                const uint64_t key = mine ? a.key[off + k] : 0;
                const int64_t stamp = r * STAMP_STRIDE + (STAMP_STRIDE - 1 - k);
                int64_t slot = -1;
                bool was_cached = false;
                if (mine) {
                    slot = find_slot(tab, key, mask, cap_log2);
                    if (slot >= 0) {
                        was_cached = ld(&tab[slot].stamp) >= tau_b;
                        st(&tab[slot].stamp, stamp);          // touch, or revive an evicted entry in place
                    }
                }
                __syncthreads();
                bool took_fresh = false;
                if (mine && slot < 0) took_fresh = insert_new(tab, key, stamp, tau_b, mask, cap_log2);
                __syncthreads();
                add_live += __popcll(__ballot(mine && !was_cached));
                add_used += __popcll(__ballot(took_fresh));
            }
            if (lane == 0) {
                live[best] += add_live;
                used[best] += add_used;
            }
            __syncthreads();
        }

        // ---- eviction: advance the threshold past the least recently used blocks until the cache fits.
        // The log of (request, position) touches on this replica is the route array itself, walked from the
        // oldest request routed here; a logged touch still counts iff the table holds exactly its stamp.
        if (a.C > 0 && live[best] > a.C) {
            int E = (int)(live[best] - a.C);
            int cr = cur_r[best], ck = cur_k[best];
            while (E > 0) {
                if (ck == 0) {
                    const int64_t x = next_routed(route, cr, r, best, lane);
                    if (x >= r) break;          // cannot happen while E > 0; bounds the loop regardless
                    cr = (int)x;
                    ck = (int)(a.blk_off[x + 1] - a.blk_off[x]);
                    continue;
                }
                const int64_t ooff = a.blk_off[cr];
                const int k = ck - 1 - lane;               // lane order = eviction order (deepest first)
                bool alive = false;
                if (k >= 0 && a.first[ooff + k] != 0) {
                    const int64_t s = find_slot(tab, a.key[ooff + k], mask, cap_log2);
                    alive = s >= 0 && ld(&tab[s].stamp) == (int64_t)cr * STAMP_STRIDE + (STAMP_STRIDE - 1 - k);
                }
                const uint64_t mk = __ballot(alive);
                const int cnt = __popcll(mk);
                if (cnt <= E) {
                    E -= cnt;
                    ck = ck > WAVE ? ck - WAVE : 0;
                } else {
                    const int rank = __popcll(mk & ((1ull << lane) - 1));
                    const uint64_t last = __ballot(alive && rank == E - 1);
                    const int j = __ffsll((unsigned long long)last) - 1;
                    ck = ck - 1 - j;
                    E = 0;
                }
            }
            if (lane == 0) {
                cur_r[best] = cr;
                cur_k[best] = ck;
                tau[best] = (int64_t)cr * STAMP_STRIDE + (STAMP_STRIDE - ck);
                live[best] = (int32_t)a.C + E;
            }
        }

        // ---- service on the chosen replica, outputs
        double ttft, e2e;
        Q.serve<false>(r, best, t, my_rtt, my_u, L, O, a.a_pf, a.a_dec, rec, lane, Q.idle, &ttft, &e2e);
        if (lane == 0) {
            if (a.hit) a.hit[(size_t)p * N + r] = (uint16_t)m_best;
            if (a.ttft) a.ttft[(size_t)p * N + r] = ttft;
            if (a.e2e) a.e2e[(size_t)p * N + r] = e2e;
        }
        __syncthreads();
    }
}

// The last row but one of every replay's rows (the one no request touches) gets the cell value that is below any
// cursor.
__global__ void __launch_bounds__(256) fill_last_rows(int32_t* x, int32_t P, int64_t rows, int32_t R, int32_t v) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (size_t)P * R) x[((i / R) * (size_t)rows + (size_t)(rows - 2)) * R + i % R] = v;
}

// ---- exact nearest-rank percentile: k-th smallest of x[p][0..N) by most-significant-digit radix selection
// on the order-preserving integer image of the doubles.  One 256-thread workgroup per row.
constexpr int SEL_THREADS = 256;
constexpr int SEL_BITS = 11;
constexpr int SEL_BINS = 1 << SEL_BITS;

__device__ __forceinline__ uint64_t ordered_bits(double x) {
    uint64_t b = (uint64_t)__double_as_longlong(x);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

__global__ void __launch_bounds__(SEL_THREADS) select_kth(const double* x, int64_t N, int64_t kth /*1-based*/,
                                                          double* out) {
    __shared__ uint32_t hist[SEL_BINS];
    __shared__ uint32_t part[SEL_THREADS];
    __shared__ uint64_t s_prefix;
    __shared__ int64_t s_k;
    const int tid = threadIdx.x;
    const double* row = x + (size_t)blockIdx.x * N;
    if (N <= 0) {
        if (tid == 0) out[blockIdx.x] = 0.0;
        return;
    }
    if (tid == 0) {
        s_prefix = 0;
        s_k = kth;
    }
    int shift = 64;
    uint64_t prefix_mask = 0;
    while (shift > 0) {
        const int bits = shift >= SEL_BITS ? SEL_BITS : shift;
        shift -= bits;
        for (int b = tid; b < SEL_BINS; b += SEL_THREADS) hist[b] = 0;
        __syncthreads();
        const uint64_t prefix = s_prefix;
        const int64_t k = s_k;
        for (int64_t i = tid; i < N; i += SEL_THREADS) {
            const uint64_t v = ordered_bits(row[i]);
            if ((v & prefix_mask) == prefix) atomicAdd(&hist[(v >> shift) & ((1u << bits) - 1)], 1u);
        }
        __syncthreads();
        // locate the bin that holds the k-th element: per-thread partial sums, then a short serial scan
        constexpr int PER = SEL_BINS / SEL_THREADS;
        uint32_t sum = 0;
        for (int j = 0; j < PER; ++j) sum += hist[tid * PER + j];
        part[tid] = sum;
        __syncthreads();
        if (tid == 0) {
            int64_t acc = 0;
            int g = 0;
            while (g < SEL_THREADS - 1 && acc + part[g] < k) acc += part[g++];
            int b = g * PER;
            while (b < SEL_BINS - 1 && acc + hist[b] < k) acc += hist[b++];
            s_prefix = prefix | ((uint64_t)b << shift);
            s_k = k - acc;
        }
        prefix_mask |= ((bits == 64 ? ~0ull : ((1ull << bits) - 1)) << shift);
        __syncthreads();
    }
    if (tid == 0) {
        uint64_t v = s_prefix;
        uint64_t b = (v >> 63) ? (v & 0x7FFFFFFFFFFFFFFFull) : ~v;
        out[blockIdx.x] = __longlong_as_double((long long)b);
    }
}

int hip_fail(hipError_t e, const char* what) {
    return fail(GORGO_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

// HIP events bracketing the kernels of the most recent evaluation on this thread (for measurement).
struct Marks {
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};   // before fill, before replay, after replay, after select
    int device = -1;
    bool valid = false;
};
thread_local Marks g_marks;

bool marks_ready() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (g_marks.device == dev) return true;
    for (auto& e : g_marks.ev)
        if (hipEventCreate(&e) != hipSuccess) return false;
    g_marks.device = dev;
    return true;
}

thread_local bool g_marks_on = true;      // off for the evaluation that must not create or record events

void mark(int i, hipStream_t s) {
    if (g_marks_on && g_marks.device >= 0) (void)hipEventRecord(g_marks.ev[i], s);
}

// Device memory for the entry point that allocates nothing: one array per GPU, there from the moment the library
// is loaded until the process ends.  Host code only ever uses its device address, looked up once per device.
static __device__ __align__(256) unsigned char scratch[GORGO_STATIC_SCRATCH_BYTES];

}  // namespace

int upload_trace(const gorgo_trace* tc) {
    gorgo_trace* t = const_cast<gorgo_trace*>(tc);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (t->dev.base && t->dev.device == dev) return GORGO_OK;
    if (t->dev.base) release_device_trace(t);
    const size_t N = (size_t)t->N, T = (size_t)t->total_blocks;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t o_ts = 0;
    const size_t o_off = o_ts + up(N * 8);
    const size_t o_il = o_off + up((N + 1) * 8);
    const size_t o_ol = o_il + up(N * 4);
    const size_t o_key = o_ol + up(N * 4);
    const size_t o_first = o_key + up(T * 4);
    const size_t n_sr = t->seg.size();
    const size_t o_soff = o_first + up(T);
    const size_t o_seg = o_soff + up(t->seg_off.size() * 8);
    const size_t o_fh = o_seg + up(n_sr * sizeof(SegRef));
    const size_t total = o_fh + up(N * 4) + 256;
    char* base = nullptr;
    e = hipMalloc(reinterpret_cast<void**>(&base), total);
    if (e != hipSuccess) return fail(GORGO_ERR_OOM, std::string("hipMalloc(trace): ") + hipGetErrorString(e));
    auto put = [&](size_t o, const void* src, size_t bytes) {
        return bytes ? hipMemcpy(base + o, src, bytes, hipMemcpyHostToDevice) : hipSuccess;
    };
    if ((e = put(o_ts, t->ts.data(), N * 8)) != hipSuccess || (e = put(o_off, t->blk_off.data(), (N + 1) * 8)) != hipSuccess ||
        (e = put(o_il, t->in_len.data(), N * 4)) != hipSuccess || (e = put(o_ol, t->out_len.data(), N * 4)) != hipSuccess ||
        (e = put(o_key, t->key.data(), T * 4)) != hipSuccess || (e = put(o_first, t->first.data(), T)) != hipSuccess ||
        (e = put(o_soff, t->seg_off.data(), t->seg_off.size() * 8)) != hipSuccess ||
        (e = put(o_seg, t->seg.data(), n_sr * sizeof(SegRef))) != hipSuccess ||
        (e = put(o_fh, t->first_hash.data(), N * 4)) != hipSuccess) {
        (void)hipFree(base);
        return hip_fail(e, "hipMemcpy(trace)");
    }
    t->dev.device = dev;
    t->dev.base = base;
    t->dev.ts = reinterpret_cast<const int64_t*>(base + o_ts);
    t->dev.blk_off = reinterpret_cast<const int64_t*>(base + o_off);
    t->dev.in_len = reinterpret_cast<const int32_t*>(base + o_il);
    t->dev.out_len = reinterpret_cast<const int32_t*>(base + o_ol);
    t->dev.key = reinterpret_cast<const uint32_t*>(base + o_key);
    t->dev.first = reinterpret_cast<const uint8_t*>(base + o_first);
    t->dev.seg_off = reinterpret_cast<const int64_t*>(base + o_soff);
    t->dev.seg = reinterpret_cast<const SegRef*>(base + o_seg);
    t->dev.first_hash = reinterpret_cast<const uint32_t*>(base + o_fh);
    return GORGO_OK;
}

void release_device_trace(gorgo_trace* t) {
    if (t->dev.base) (void)hipFree(t->dev.base);
    t->dev = DeviceTrace();
}

int copy_small_to_device(void* dst, const void* src, size_t bytes, void* stream) {
    hipError_t e = hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GORGO_OK : hip_fail(e, "hipMemcpyAsync(H2D)");
}

// Whether a launch of fixed-weight replays runs two replays per wavefront pair.  A replay is a serial chain whose
// duration does not depend on how many others run beside it, and a packed pair takes about half as long again per
// request as a lone replay: packing pays when the replays would not all be resident at once otherwise, but the
// pairs are.
bool pack_replays(const Plan& pl, int64_t rows) {
    const int32_t mode = pl.packing;       // 0 never, 1 whenever the shape allows, 2 when the replays would not all be resident
    if (mode == 0 || pl.R > HALF || pl.B > 16 || pl.P % 2 != 0 ||
        2ull * (uint64_t)rows * (uint64_t)pl.R * 4u >= (1ull << 32))
        return false;
    if (mode == 1) return true;
    int device = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&device) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, replay_segments_kernel<MODE_COST_MODEL, false, false>,
                                                     SEG3_THREADS, replay_segments_lds_bytes(pl.R, pl.B, 0)) != hipSuccess)
        return false;
    // (measured: packed pairs win when they make one round of what would be two; with more rounds on either side
    // the unpacked kernel's shorter request step wins again)
    const int64_t resident = (int64_t)cus * per_cu;
    return (int64_t)pl.P > resident && (int64_t)pl.P <= 2 * resident;
}

int wait_for_copies(void* stream) {
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GORGO_OK : hip_fail(e, "hipStreamSynchronize");
}

int copy_small_to_host_sync(void* dst, const void* src, size_t bytes, void* stream) {
    hipError_t e = hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(D2H)");
    e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GORGO_OK : hip_fail(e, "hipStreamSynchronize");
}

namespace {

// The proxy's smoothed round trip times (Sec. 2.2: an exponentially weighted moving average of pings), one
// thread per replica: est[0] = x[0], est[e] = alpha x[e] + (1 - alpha) est[e-1], each product and sum rounded
// on its own.
__global__ void smooth_rtt(const double* x, double* est, int epochs, int R, double alpha) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= R) return;
    double prev = x[i];
    est[i] = prev;
    for (int e = 1; e < epochs; ++e) {
        const double fresh = alpha * x[(size_t)e * R + i];
        const double kept = (1.0 - alpha) * prev;
        prev = fresh + kept;
        est[(size_t)e * R + i] = prev;
    }
}

}  // namespace

int static_scratch(void** ptr, size_t* bytes) {
    static std::mutex mu;
    static void* address[64] = {};        // per device: each GPU holds its own copy of the array at its own address
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= 64) return fail(GORGO_ERR_DEVICE, "device index out of range");
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        address[dev] = p;
    }
    *ptr = address[dev];
    *bytes = sizeof(scratch);
    return GORGO_OK;
}

bool trace_is_resident(const gorgo_trace* t) {
    int dev = 0;
    return hipGetDevice(&dev) == hipSuccess && t->dev.base && t->dev.device == dev;
}

void set_event_marks(bool on) { g_marks_on = on; }

int launch_replay(const gorgo_trace* t, const Plan& pl, const double* d_rtt, const double* d_params,
                  const double* d_scale, uint8_t* route, uint16_t* hit, double* ttft, double* e2e,
                  void* workspace, void* stream, const OnlineLaunch* online, const PolicyLaunch* policy,
                  const EngineLaunch* engine, const ProxyLaunch* proxy, unsigned long long* sections) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    g_marks.valid = false;
    if (g_marks_on) marks_ready();
    mark(0, s);
    hipError_t e;
    if (pl.path == PATH_SEGMENTS) {
        SegArgs a;
        a.ts = t->dev.ts;
        a.in_len = t->dev.in_len;
        a.out_len = t->dev.out_len;
        a.seg_off = t->dev.seg_off;
        a.seg = t->dev.seg;
        a.N = pl.N;
        a.R = pl.R;
        a.B = pl.B;
        a.C = pl.C;
        a.nseg = pl.nseg + 2;             // rows of one replay: one per segment, one that no request touches, a spare
        a.block_tokens = pl.block_tokens;
        a.a_pf = pl.a_pf;
        a.a_dec = pl.a_dec;
        a.rtt = d_rtt;
        a.params = d_params;
        a.scale = d_scale;
        a.last = reinterpret_cast<int32_t*>(ws + pl.off_tables);
        a.log = reinterpret_cast<LogRec*>(ws + pl.off_spare);
        a.rec = reinterpret_cast<Rec*>(ws + pl.off_rec);
        a.route = route;
        a.hit = hit;
        a.ttft = ttft;
        a.e2e = e2e;
        a.window = a.hop = 0;
        a.steps = 0;
        a.tuner = a.ln_theta0 = a.z = nullptr;
        a.theta_step = a.fitness_step = a.theta_final = a.sigma_final = nullptr;
        a.accepted = nullptr;
        a.first_hash = t->dev.first_hash;
        a.seeds = policy ? policy->seeds : nullptr;
        a.spin_limit = pl.poll_limit;           // (only the packed kernel polls)
        a.eng_a_pf = engine ? engine->a_pf : nullptr;
        a.eng_a_dec = engine ? engine->a_dec : nullptr;
        a.eng_budget = engine ? engine->budget : nullptr;
        a.eng_slowdown = engine ? engine->slowdown : 0.0;
        a.epochs = proxy ? proxy->epochs : 0;
        a.probe_ms = proxy ? proxy->probe_ms : 0;
        a.rtt_true = proxy ? proxy->rtt_true : nullptr;
        a.rtt_est = proxy ? proxy->rtt_est : nullptr;
        a.index_blocks = proxy ? proxy->index_blocks : -1;
        a.believed = proxy ? proxy->believed : nullptr;
        a.sections = sections;
        if (sections && (online || engine || proxy || (policy && policy->policy != 0)))
            return fail(GORGO_ERR_INVALID_ARG, "section timing exists for the fixed-weight cost model with the linear replica model");
        if (proxy) {
            if (policy && policy->policy != 0)
                return fail(GORGO_ERR_INVALID_ARG, "imperfect proxy knowledge concerns the cost model, not the baseline policies");
            hipLaunchKernelGGL(smooth_rtt, dim3(1), dim3(WAVE), 0, s, proxy->rtt_true, proxy->rtt_est, proxy->epochs, pl.R,
                               proxy->alpha);
            if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "launch smooth_rtt");
        }
        // (a row is written through before it is first read -- the request that brings a segment into a row slot
        // resets the row -- so only the never-cached row needs a value beforehand)
        if (pl.P > 0) {
            hipLaunchKernelGGL(fill_last_rows, dim3((unsigned)(((size_t)pl.P * pl.R + 255) / 256)), dim3(256), 0, s, a.last,
                               pl.P, a.nseg, pl.R, NEVER_CACHED);
            if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "launch fill_last_rows");
        }
        mark(1, s);
        if (pl.N > 0 || online) {      // (an empty trace still reports the tuner's initial state)
            if (online) {
                a.window = online->window;
                a.hop = online->hop;
                a.steps = online->steps;
                a.tuner = online->tuner;
                a.ln_theta0 = online->ln_theta0;
                a.z = online->z;
                a.theta_step = online->theta_step;
                a.fitness_step = online->fitness_step;
                a.theta_final = online->theta_final;
                a.sigma_final = online->sigma_final;
                a.accepted = online->accepted;
                const size_t lds = replay_segments_lds_bytes(pl.R, pl.B, online->window);
                const dim3 grid((unsigned)pl.P), block(SEG3_THREADS);
                if (proxy && engine) hipLaunchKernelGGL((replay_segments_kernel<MODE_ONLINE, true, true>), grid, block, lds, s, a);
                else if (proxy) hipLaunchKernelGGL((replay_segments_kernel<MODE_ONLINE, false, true>), grid, block, lds, s, a);
                else if (engine) hipLaunchKernelGGL((replay_segments_kernel<MODE_ONLINE, true, false>), grid, block, lds, s, a);
                else if (SlotQueues::fits(pl.R, pl.B)) hipLaunchKernelGGL((replay_segments_kernel<MODE_ONLINE, false, false, true>), grid, block, lds, s, a);
                else hipLaunchKernelGGL((replay_segments_kernel<MODE_ONLINE, false, false>), grid, block, lds, s, a);
            } else if (proxy) {
                const size_t lds = replay_segments_lds_bytes(pl.R, pl.B, 0);
                const dim3 grid((unsigned)pl.P), block(SEG3_THREADS);
                if (engine) hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, true, true>), grid, block, lds, s, a);
                else hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, false, true>), grid, block, lds, s, a);
            } else if (engine) {
                const size_t lds = replay_segments_lds_bytes(pl.R, pl.B, 0);
                const dim3 grid((unsigned)pl.P), block(SEG3_THREADS);
                switch (policy ? policy->policy : 0) {
                    case 0: hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, true, false>), grid, block, lds, s, a); break;
                    case 1: hipLaunchKernelGGL((replay_segments_kernel<MODE_LEAST_REQUEST, true, false>), grid, block, lds, s, a); break;
                    case 2: hipLaunchKernelGGL((replay_segments_kernel<MODE_AFFINITY, true, false>), grid, block, lds, s, a); break;
                    default: hipLaunchKernelGGL((replay_segments_kernel<MODE_RANDOM, true, false>), grid, block, lds, s, a); break;
                }
            } else if (sections) {
                const dim3 grid((unsigned)pl.P), block(SEG3_THREADS);
                const size_t lds = replay_segments_lds_bytes(pl.R, pl.B, 0);
                if (SlotQueues::fits(pl.R, pl.B))
                    hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, false, false, true, true>), grid, block, lds, s, a);
                else
                    hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, false, false, false, true>), grid, block, lds, s, a);
            } else if (!(policy && policy->policy != 0) && pack_replays(pl, a.nseg)) {
                // fixed weights, at most 32 replicas: two replays per wavefront pair
                hipLaunchKernelGGL(replay_segments_packed_kernel, dim3((unsigned)(pl.P / 2)), dim3(SEG_THREADS),
                                   replay_segments_packed_lds_bytes(pl.B), s, a);
            } else {
                const size_t lds = replay_segments_lds_bytes(pl.R, pl.B, 0);
                const dim3 grid((unsigned)pl.P), block(SEG3_THREADS);
                if (SlotQueues::fits(pl.R, pl.B)) {
                    switch (policy ? policy->policy : 0) {
                        case 0: hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, false, false, true>), grid, block, lds, s, a); break;
                        case 1: hipLaunchKernelGGL((replay_segments_kernel<MODE_LEAST_REQUEST, false, false, true>), grid, block, lds, s, a); break;
                        case 2: hipLaunchKernelGGL((replay_segments_kernel<MODE_AFFINITY, false, false, true>), grid, block, lds, s, a); break;
                        default: hipLaunchKernelGGL((replay_segments_kernel<MODE_RANDOM, false, false, true>), grid, block, lds, s, a); break;
                    }
                } else {
                    switch (policy ? policy->policy : 0) {
                        case 0: hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, false, false>), grid, block, lds, s, a); break;
                        case 1: hipLaunchKernelGGL((replay_segments_kernel<MODE_LEAST_REQUEST, false, false>), grid, block, lds, s, a); break;
                        case 2: hipLaunchKernelGGL((replay_segments_kernel<MODE_AFFINITY, false, false>), grid, block, lds, s, a); break;
                        default: hipLaunchKernelGGL((replay_segments_kernel<MODE_RANDOM, false, false>), grid, block, lds, s, a); break;
                    }
                }
            }
            if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "launch replay_segments_kernel");
        }
    } else {
        if (sections) return fail(GORGO_ERR_INVALID_ARG, "section timing needs the segment formulation");
        if (online || engine || proxy || (policy && policy->policy != 0))
            return fail(GORGO_ERR_INVALID_ARG, "the online tuner, the baseline policies, the engine model and imperfect "
                                               "proxy knowledge need the segment formulation");
        ReplayArgs a;
        a.ts = t->dev.ts;
        a.in_len = t->dev.in_len;
        a.out_len = t->dev.out_len;
        a.blk_off = t->dev.blk_off;
        a.key = t->dev.key;
        a.first = t->dev.first;
        a.N = pl.N;
        a.R = pl.R;
        a.B = pl.B;
        a.C = pl.C;
        a.cap = pl.cap;
        a.cap_log2 = 0;
        while ((1ll << a.cap_log2) < pl.cap) ++a.cap_log2;
        a.block_tokens = pl.block_tokens;
        a.a_pf = pl.a_pf;
        a.a_dec = pl.a_dec;
        a.rtt = d_rtt;
        a.params = d_params;
        a.scale = d_scale;
        a.tables = reinterpret_cast<Slot*>(ws + pl.off_tables);
        a.spare = reinterpret_cast<Slot*>(ws + pl.off_spare);
        a.rec = reinterpret_cast<Rec*>(ws + pl.off_rec);
        a.route = route;
        a.hit = hit;
        a.ttft = ttft;
        a.e2e = e2e;
        const size_t nslots = (size_t)pl.P * pl.R * pl.cap;
        size_t blocks = (nslots + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(fill_slots, dim3((unsigned)blocks), dim3(256), 0, s, a.tables, nslots);
        if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "launch fill_slots");
        mark(1, s);
        if (pl.N > 0) {
            const size_t lds = Queues::bytes(pl.R, pl.B) + (size_t)pl.R * (8 + 4 * 4);
            hipLaunchKernelGGL(replay_blocks_kernel, dim3((unsigned)pl.P), dim3(WAVE), lds, s, a);
            if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "launch replay_blocks_kernel");
        }
    }
    mark(2, s);
    mark(3, s);
    g_marks.valid = g_marks_on && g_marks.device >= 0;
    return GORGO_OK;
}

int last_eval_kernel_ms(double* fill_ms, double* replay_ms, double* select_ms) {
    if (!g_marks.valid) return fail(GORGO_ERR_INVALID_ARG, "no evaluation has been enqueued on this thread");
    hipError_t e = hipEventSynchronize(g_marks.ev[3]);
    if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
    float a = 0, b = 0, c = 0;
    if ((e = hipEventElapsedTime(&a, g_marks.ev[0], g_marks.ev[1])) != hipSuccess ||
        (e = hipEventElapsedTime(&b, g_marks.ev[1], g_marks.ev[2])) != hipSuccess ||
        (e = hipEventElapsedTime(&c, g_marks.ev[2], g_marks.ev[3])) != hipSuccess)
        return hip_fail(e, "hipEventElapsedTime");
    if (fill_ms) *fill_ms = a;
    if (replay_ms) *replay_ms = b;
    if (select_ms) *select_ms = c;
    return GORGO_OK;
}

int launch_p95(const double* x, int64_t N, int32_t P, double* out, void* stream) {
    const int64_t kth = (95 * N + 99) / 100;
    hipLaunchKernelGGL(select_kth, dim3((unsigned)P), dim3(SEL_THREADS), 0, static_cast<hipStream_t>(stream), x, N,
                       kth, out);
    hipError_t e = hipGetLastError();
    mark(3, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GORGO_OK : hip_fail(e, "launch select_kth");
}

}  // namespace gorgo

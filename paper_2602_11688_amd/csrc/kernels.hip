// Device side: the launches of the replay kernels (segment rows: replay_segments.h and replay_segments_packed.h;
// block tables: replay_blocks.h), the exact percentile selection, and the trace upload.
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
#include "replay_blocks.h"
#include "replay_segments.h"
#include "replay_segments_packed.h"

namespace gorgo {

namespace {

// The last row but one of every replay's rows (the one no request touches) gets the cell value that is below any
// cursor.
__global__ void __launch_bounds__(256) fill_last_rows(int32_t* x, int32_t P, int64_t rows, int32_t R, int32_t v) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (size_t)P * R) x[((i / R) * (size_t)rows + (size_t)(rows - 2)) * R + i % R] = v;
}

// ---- exact nearest-rank percentile: k-th smallest of x[p][0..N) by most-significant-digit radix selection
// on the order-preserving integer image of the doubles.  One 256-thread workgroup per row.  Every digit is a pass
// over the row; as soon as the bin that holds the k-th element has few enough elements they are gathered into LDS
// in one more pass and the element is picked there by counting (latencies of a replay differ in the first two or
// three digits: three passes instead of six).
constexpr int SEL_THREADS = 256;
constexpr int SEL_BITS = 11;
constexpr int SEL_BINS = 1 << SEL_BITS;
constexpr int SEL_GATHER = 2048;      // candidates that are finished in LDS

__device__ __forceinline__ uint64_t ordered_bits(double x) {
    uint64_t b = (uint64_t)__double_as_longlong(x);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

__global__ void __launch_bounds__(SEL_THREADS) select_kth(const double* x, int64_t N, int64_t kth /*1-based*/,
                                                          double* out) {
    __shared__ uint32_t hist[SEL_BINS];
    __shared__ uint32_t part[SEL_THREADS];
    __shared__ uint64_t cand[SEL_GATHER];
    __shared__ uint64_t s_prefix;
    __shared__ int64_t s_k;
    __shared__ uint32_t s_in_bin, n_cand;
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
        // (four loads in flight per thread)
        int64_t i = tid;
        for (; i + 3 * SEL_THREADS < N; i += 4 * SEL_THREADS) {
            uint64_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = ordered_bits(row[i + u * SEL_THREADS]);
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if ((v[u] & prefix_mask) == prefix) atomicAdd(&hist[(v[u] >> shift) & ((1u << bits) - 1)], 1u);
        }
        for (; i < N; i += SEL_THREADS) {
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
            s_in_bin = hist[b];
            n_cand = 0;
        }
        prefix_mask |= ((bits == 64 ? ~0ull : ((1ull << bits) - 1)) << shift);
        __syncthreads();
        if (shift > 0 && s_in_bin <= (uint32_t)SEL_GATHER) {
            // few enough left: gather them, and take the one with fewer than k below it and at least k not above it
            const uint64_t want = s_prefix;
            int64_t i = tid;
            for (; i + 3 * SEL_THREADS < N; i += 4 * SEL_THREADS) {
                uint64_t v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = ordered_bits(row[i + u * SEL_THREADS]);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if ((v[u] & prefix_mask) == want) cand[atomicAdd(&n_cand, 1u)] = v[u];
            }
            for (; i < N; i += SEL_THREADS) {
                const uint64_t v = ordered_bits(row[i]);
                if ((v & prefix_mask) == want) cand[atomicAdd(&n_cand, 1u)] = v;
            }
            __syncthreads();
            const int n = (int)n_cand;
            const int64_t kk = s_k;
            for (int c = tid; c < n; c += SEL_THREADS) {
                const uint64_t mine = cand[c];
                int64_t less = 0, leq = 0;
                for (int j = 0; j < n; ++j) {
                    less += cand[j] < mine ? 1 : 0;
                    leq += cand[j] <= mine ? 1 : 0;
                }
                if (less < kk && kk <= leq) s_prefix = mine;      // (every such element has the same value)
            }
            __syncthreads();
            break;
        }
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

namespace {

// The block-table kernel's instantiations: every mode with either replica model; imperfect proxy knowledge concerns
// the cost model (fixed weights or tuned online) only.
template <int MODE>
void launch_blocks(bool engine, bool proxy, dim3 grid, size_t lds, hipStream_t s, const BlockArgs& b) {
    const dim3 block(SEG_THREADS);
    if constexpr (MODE == MODE_COST_MODEL || MODE == MODE_ONLINE) {
        if (proxy) {
            if (engine) hipLaunchKernelGGL((replay_blocks_kernel<MODE, true, true>), grid, block, lds, s, b);
            else hipLaunchKernelGGL((replay_blocks_kernel<MODE, false, true>), grid, block, lds, s, b);
            return;
        }
    }
    if (engine) hipLaunchKernelGGL((replay_blocks_kernel<MODE, true, false>), grid, block, lds, s, b);
    else hipLaunchKernelGGL((replay_blocks_kernel<MODE, false, false>), grid, block, lds, s, b);
}

}  // namespace

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
    const bool segments = pl.path == PATH_SEGMENTS;
    // what both formulations' kernels read: the trace's scalars, the model, the weights, the outputs, and what the
    // online tuner, the baseline policies, the engine model and the proxy's knowledge bring
    SegArgs a;
    a.ts = t->dev.ts;
    a.in_len = t->dev.in_len;
    a.out_len = t->dev.out_len;
    a.seg_off = segments ? t->dev.seg_off : nullptr;
    a.seg = segments ? t->dev.seg : nullptr;
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
    a.last = segments ? reinterpret_cast<int32_t*>(ws + pl.off_tables) : nullptr;
    a.log = segments ? reinterpret_cast<LogRec*>(ws + pl.off_spare) : nullptr;
    a.rec = reinterpret_cast<Rec*>(ws + pl.off_rec);
    a.route = route;
    a.hit = hit;
    a.ttft = ttft;
    a.e2e = e2e;
    a.window = online ? online->window : 0;
    a.hop = online ? online->hop : 0;
    a.steps = online ? online->steps : 0;
    a.tuner = online ? online->tuner : nullptr;
    a.ln_theta0 = online ? online->ln_theta0 : nullptr;
    a.z = online ? online->z : nullptr;
    a.theta_step = online ? online->theta_step : nullptr;
    a.fitness_step = online ? online->fitness_step : nullptr;
    a.theta_final = online ? online->theta_final : nullptr;
    a.sigma_final = online ? online->sigma_final : nullptr;
    a.accepted = online ? online->accepted : nullptr;
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
    if (sections && (!segments || online || engine || proxy || (policy && policy->policy != 0)))
        return fail(GORGO_ERR_INVALID_ARG, "section timing exists for the fixed-weight cost model with the linear replica "
                                           "model in the segment formulation");
    if (proxy) {
        if (policy && policy->policy != 0)
            return fail(GORGO_ERR_INVALID_ARG, "imperfect proxy knowledge concerns the cost model, not the baseline policies");
        hipLaunchKernelGGL(smooth_rtt, dim3(1), dim3(WAVE), 0, s, proxy->rtt_true, proxy->rtt_est, proxy->epochs, pl.R,
                           proxy->alpha);
        if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "launch smooth_rtt");
    }
    const int mode = online ? MODE_ONLINE
                            : !policy || policy->policy == 0 ? MODE_COST_MODEL
                            : policy->policy == 1 ? MODE_LEAST_REQUEST
                            : policy->policy == 2 ? MODE_AFFINITY : MODE_RANDOM;
    if (segments) {
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
                switch (mode) {
                    case MODE_COST_MODEL: hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, true, false>), grid, block, lds, s, a); break;
                    case MODE_LEAST_REQUEST: hipLaunchKernelGGL((replay_segments_kernel<MODE_LEAST_REQUEST, true, false>), grid, block, lds, s, a); break;
                    case MODE_AFFINITY: hipLaunchKernelGGL((replay_segments_kernel<MODE_AFFINITY, true, false>), grid, block, lds, s, a); break;
                    default: hipLaunchKernelGGL((replay_segments_kernel<MODE_RANDOM, true, false>), grid, block, lds, s, a); break;
                }
            } else if (sections) {
                const dim3 grid((unsigned)pl.P), block(SEG3_THREADS);
                const size_t lds = replay_segments_lds_bytes(pl.R, pl.B, 0);
                if (SlotQueues::fits(pl.R, pl.B))
                    hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, false, false, true, true>), grid, block, lds, s, a);
                else
                    hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, false, false, false, true>), grid, block, lds, s, a);
            } else if (mode == MODE_COST_MODEL && pack_replays(pl, a.nseg)) {
                // fixed weights, at most 32 replicas: two replays per wavefront pair
                hipLaunchKernelGGL(replay_segments_packed_kernel, dim3((unsigned)(pl.P / 2)), dim3(SEG_THREADS),
                                   replay_segments_packed_lds_bytes(pl.B), s, a);
            } else {
                const size_t lds = replay_segments_lds_bytes(pl.R, pl.B, 0);
                const dim3 grid((unsigned)pl.P), block(SEG3_THREADS);
                if (SlotQueues::fits(pl.R, pl.B)) {
                    switch (mode) {
                        case MODE_COST_MODEL: hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, false, false, true>), grid, block, lds, s, a); break;
                        case MODE_LEAST_REQUEST: hipLaunchKernelGGL((replay_segments_kernel<MODE_LEAST_REQUEST, false, false, true>), grid, block, lds, s, a); break;
                        case MODE_AFFINITY: hipLaunchKernelGGL((replay_segments_kernel<MODE_AFFINITY, false, false, true>), grid, block, lds, s, a); break;
                        default: hipLaunchKernelGGL((replay_segments_kernel<MODE_RANDOM, false, false, true>), grid, block, lds, s, a); break;
                    }
                } else {
                    switch (mode) {
                        case MODE_COST_MODEL: hipLaunchKernelGGL((replay_segments_kernel<MODE_COST_MODEL, false, false>), grid, block, lds, s, a); break;
                        case MODE_LEAST_REQUEST: hipLaunchKernelGGL((replay_segments_kernel<MODE_LEAST_REQUEST, false, false>), grid, block, lds, s, a); break;
                        case MODE_AFFINITY: hipLaunchKernelGGL((replay_segments_kernel<MODE_AFFINITY, false, false>), grid, block, lds, s, a); break;
                        default: hipLaunchKernelGGL((replay_segments_kernel<MODE_RANDOM, false, false>), grid, block, lds, s, a); break;
                    }
                }
            }
            if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "launch replay_segments_kernel");
        }
    } else {
        BlockArgs b;
        b.q = a;
        b.blk_off = t->dev.blk_off;
        b.key = t->dev.key;
        b.first = t->dev.first;
        b.cap = pl.cap;
        b.cap_log2 = 0;
        while ((1ll << b.cap_log2) < pl.cap) ++b.cap_log2;
        b.tables = reinterpret_cast<Slot*>(ws + pl.off_tables);
        b.spare = reinterpret_cast<Slot*>(ws + pl.off_spare);
        b.routed = reinterpret_cast<uint8_t*>(ws + pl.off_route);
        const size_t nslots = (size_t)pl.P * pl.R * pl.cap;
        size_t blocks = (nslots + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(fill_slots, dim3((unsigned)blocks), dim3(256), 0, s, b.tables, nslots);
        if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "launch fill_slots");
        mark(1, s);
        if (pl.N > 0 || online) {      // (an empty trace still reports the tuner's initial state)
            const size_t lds = replay_blocks_lds_bytes(pl.R, pl.B, a.window);
            const dim3 grid((unsigned)pl.P);
            switch (mode) {
                case MODE_COST_MODEL: launch_blocks<MODE_COST_MODEL>(engine != nullptr, proxy != nullptr, grid, lds, s, b); break;
                case MODE_ONLINE: launch_blocks<MODE_ONLINE>(engine != nullptr, proxy != nullptr, grid, lds, s, b); break;
                case MODE_LEAST_REQUEST: launch_blocks<MODE_LEAST_REQUEST>(engine != nullptr, false, grid, lds, s, b); break;
                case MODE_AFFINITY: launch_blocks<MODE_AFFINITY>(engine != nullptr, false, grid, lds, s, b); break;
                default: launch_blocks<MODE_RANDOM>(engine != nullptr, false, grid, lds, s, b); break;
            }
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

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
// record per logged request (next request on the replica, own, n) and never re-reads cells.  Records that
// own nothing any more are dropped from the walk as soon as they are seen.
//
// The request loop is one dependent chain per replay, and a lone wavefront issues about one instruction
// every four to five cycles whatever its kind, so the kernel is arranged around instruction count and
// latency, not bandwidth.  A replay is run by two wavefronts of one workgroup.  The cache wavefront keeps the
// cache side (lane = replica: cursor, the next log records) in its registers, matches, scores, picks the
// replica and updates rows and log; the queue wavefront keeps the queue side (lane = replica: load signal,
// earliest completion; service slots in LDS), retires completed requests before every request and serves it
// once the replica is known.  They meet twice per request through LDS: the queue wavefront publishes the load
// signals of request r, the cache wavefront answers with the chosen replica and its uncached tokens.  The
// queue wavefront has the shorter loop, so the cache wavefront normally finds the load signals waiting.
// In the cache wavefront a batch of 64 requests is staged at once (scalars in registers, segment references
// in LDS); the rows of request i+1 and one log record per replica are requested right after the wait for the
// rows of request i, so that an iteration has a single point where it waits for memory; stores are
// fire-and-forget.
#pragma once
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
    // online tuner (only read by the kernel's online variant)
    int32_t window, hop;
    int64_t steps;             // tuner steps of one replay
    const double* tuner;       // lo[3], hi[3], ln lo[3], ln hi[3], sigma0, exp(0.4), exp(-0.1)
    const double* ln_theta0;   // [P][3]
    const double* z;           // [P][steps][3]
    double* theta_step;        // [P][steps][3], nullable
    double* fitness_step;      // [P][steps], nullable
    double* theta_final;       // [P][3], nullable
    double* sigma_final;       // [P], nullable
    int32_t* accepted;         // [P], nullable
    // baseline policies
    const uint32_t* first_hash;   // [N] hash of the request's first block
    const uint64_t* seeds;        // [P] seed of the random policy
    int32_t spin_limit;           // polls of a hand-over word before the replay is given up
    // engine model of a replica (only read by the kernel's engine variants)
    const double* eng_a_pf;       // [R] prefill ms per token
    const double* eng_a_dec;      // [R] decode ms per token
    const double* eng_budget;     // [R] KV budget in tokens, 0 = none
    double eng_slowdown;
    // imperfect proxy knowledge (only read by the kernel's proxy variants)
    int32_t epochs, probe_ms;     // probe epochs given, and their length
    const double* rtt_true;       // [epochs][R] round trip time a request dispatched in the epoch experiences
    const double* rtt_est;        // [epochs][R] the proxy's moving average of them: what Eq. 3 scores with
    int64_t index_blocks;         // >= 0: Eq. 3 takes its cached prefix from the proxy's own index (an LRU of this
                                  // many blocks per replica, 0 = it never forgets); < 0: from the replica's cache
    uint16_t* believed;           // [P][N] blocks the proxy believed cached on the chosen replica, nullable
};

// What picks the replica: the cost model of Eq. 3 with fixed weights, the same with the online tuner, or one
// of the baseline policies of Sec. 4 (prefix-cache and proxy-only least-load are the cost model with weights
// (0, 1, 0) and (0, 0, 1)).
enum SegMode { MODE_COST_MODEL = 0, MODE_ONLINE = 1, MODE_LEAST_REQUEST = 2, MODE_AFFINITY = 3, MODE_RANDOM = 4 };

// A 32-bit value spread over R replicas: floor(h * R / 2^32).
__device__ __forceinline__ int spread(uint32_t h, int R) { return (int)(((uint64_t)h * (uint64_t)R) >> 32); }

// First word of Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11) for counter (c0, c1, 0, 0): per
// round two 32x32 -> 64 bit products of counter words 0 and 2 with the generator's multipliers, xors with the
// other two words and the key, and a Weyl step of the key.
__device__ __forceinline__ uint32_t philox4x32_10_first(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1) {
    uint32_t c2 = 0, c3 = 0;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t a = (uint64_t)0xD2511F53u * c0, b = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(b >> 32) ^ c1 ^ k0, n2 = (uint32_t)(a >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)b;
        c3 = (uint32_t)a;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c0;
}

constexpr int SEG_STAGE = 512;   // segment references of a 64-request batch staged in LDS
constexpr int SEG_CHUNK = 8;     // segments of a request whose rows are loaded together
constexpr int SEG_THREADS = 2 * WAVE;        // cache wavefront + queue wavefront
constexpr int SEG_SPIN_LIMIT = 1 << 24;      // default: polls of a hand-over word before the replay is given up (~1 s)

// Hand-over words between the two wavefronts of a replay, in LDS.  Every word carries the number of the
// request it belongs to (r + 1, so that the initial zero matches nothing).  They are read and written with
// relaxed workgroup-scope atomics on the LDS variable itself (so that they stay LDS instructions).  The LDS
// executes the instructions of one wavefront in the order they were issued, for reads as for writes, so data
// written before a word is there for whoever reads it after having read that word; the fences between data
// and word only have to keep the compiler from changing that order, and cost no wait.
struct SegComm {
    double q[WAVE];                   // load signal per replica, valid when seq_q == r + 1
    unsigned seq_q;
    int abandoned;                    // a wavefront gave up waiting: both leave, latencies become NaN
    unsigned long long choice;        // uncached tokens | (((r + 1) mod 2^26) << 6 | replica) << 32
    double w[3];                      // online tuner: weights in use, valid with seq_q like q
    double rtt[WAVE];                 // proxy variants: estimated round trip time per replica, valid like q
};

__device__ __forceinline__ void lds_release() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); }
__device__ __forceinline__ void lds_acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront"); }

// Orders the LDS accesses of one wavefront's lanes (the hardware executes them in program order).
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__host__ __device__ inline size_t replay_segments_lds_bytes(int R, int B, int window) {   // dynamic part
    return Queues::bytes(R, B) + (size_t)((window + 7) & ~7) * sizeof(double);   // queues, then the tuner's TTFT window
}

// exp(x) for |x| <= 700 from additions and multiplications only, in a fixed order, so that the weights the
// online tuner proposes (Sec. 2.3) have the same bits wherever they are computed: k = floor(x / ln 2 + 1/2),
// r = (x - k LN2_HI) - k LN2_LO with ln 2 split so that k LN2_HI is exact, exp(r) as its Taylor polynomial of
// degree 13 by Horner's rule from the highest term down, times 2^k.
__device__ __forceinline__ double tuner_exp(double x) {
    const double INV_LN2 = 1.44269504088896338700e+00;
    const double LN2_HI = 6.93147180369123816490e-01;
    const double LN2_LO = 1.90821492927058770002e-10;
    const double k = __builtin_floor(x * INV_LN2 + 0.5);
    const double r = (x - k * LN2_HI) - k * LN2_LO;
    double p = 1.0 / 6227020800.0;
    p = p * r + 1.0 / 479001600.0;
    p = p * r + 1.0 / 39916800.0;
    p = p * r + 1.0 / 3628800.0;
    p = p * r + 1.0 / 362880.0;
    p = p * r + 1.0 / 40320.0;
    p = p * r + 1.0 / 5040.0;
    p = p * r + 1.0 / 720.0;
    p = p * r + 1.0 / 120.0;
    p = p * r + 1.0 / 24.0;
    p = p * r + 1.0 / 6.0;
    p = p * r + 1.0 / 2.0;
    p = p * r + 1.0;
    p = p * r + 1.0;
    const unsigned long long bits = (unsigned long long)((long long)k + 1023) << 52;
    return p * __longlong_as_double((long long)bits);
}
__device__ __forceinline__ double clip(double x, double lo, double hi) {
    const double up = x < lo ? lo : x;
    return hi < up ? hi : up;
}

// k-th smallest (1-based) of the W values of `ring` (LDS), by counting: the element with fewer than k values
// below it and at least k not above it.  Every lane takes the elements lane, lane + 64, ..., two at a time;
// the values they are counted against are read eight at a time (the ring is padded with +inf up to a multiple
// of eight, which no count sees).
__device__ __forceinline__ double window_kth(const double* ring, int W, int kth, int lane) {
    double found = 0.0;
    bool have = false;
    const int W8 = (W + 7) & ~7;
    for (int e0 = 0; e0 < W; e0 += 2 * WAVE) {
        const int ea = e0 + lane, eb = e0 + WAVE + lane;
        const bool va = ea < W, vb = eb < W;
        const double xa = ring[va ? ea : 0], xb = ring[vb ? eb : 0];
        int less_a = 0, leq_a = 0, less_b = 0, leq_b = 0;
        for (int i = 0; i < W8; i += 8) {
            double v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = ring[i + j];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                less_a += v[j] < xa ? 1 : 0;
                leq_a += v[j] <= xa ? 1 : 0;
                less_b += v[j] < xb ? 1 : 0;
                leq_b += v[j] <= xb ? 1 : 0;
            }
        }
        if (va && less_a < kth && kth <= leq_a) {
            found = xa;
            have = true;
        }
        if (vb && less_b < kth && kth <= leq_b) {
            found = xb;
            have = true;
        }
    }
    const unsigned long long who = __ballot(have);      // every holder has the same value
    return readlane_f64(found, __ffsll(who) - 1);
}

// Rows of one request's first SEG_CHUNK segments as seen by this lane (= replica), with the segments' end
// positions (the same in every lane; entries past the request's last segment have end = n and no cell), and
// the reference of segment k in lane k.
struct RowSet {
    int32_t cell[SEG_CHUNK];
    int end[SEG_CHUNK];
    SegRef of_lane;
};

// Cached blocks of one segment [pos, end) whose row cell holds rl, against a cursor (c_r, c_k): all of them
// if a later request than the cursor's touched it last, those below the cursor position if the cursor's
// request did, none otherwise.  (A never-touched cell, -1, can only tie with the initial cursor (-1, 0).)
__device__ __forceinline__ int cached_in(int32_t rl, int pos, int end, int c_r, int c_k) {
    const int len = end - pos;
    int part = c_k - pos;
    part = part < 0 ? 0 : (part > len ? len : part);
    return rl > c_r ? len : (rl == c_r ? part : 0);
}

// Queue wavefront of a replay: for every request, retire what has completed by its arrival, publish the load
// signals, wait for the cache wavefront's choice, serve the request there.  Writes the latencies.
template <int MODE, bool ENGINE, bool PROXY>
__device__ __forceinline__ void queue_wave(const SegArgs& a, int p, int lane, unsigned char* lds_raw, SegComm* comm) {
    constexpr bool ONLINE = MODE == MODE_ONLINE;
    const int R = a.R;
    const int64_t N = a.N;
    Queues Q;
    Q.carve(lds_raw, R, a.B, lane);
    Q.init(lane);
    wave_sync();
    // Online tuner (Sec. 2.3, Sec. 4), run here because this wavefront has the TTFTs: after every hop the p95
    // TTFT of the last `window` requests is the fitness of the weights in use; they replace the parent iff they
    // beat it; the step size follows the 1/5 rule; the next offspring is a log-space mutation of the parent.
    // The state is the same in every lane.
    double* const ring = reinterpret_cast<double*>(lds_raw + Queues::bytes(R, a.B));
    const int W = ONLINE ? a.window : 0, H = ONLINE ? a.hop : 0;
    const int kth = (95 * W + 99) / 100;
    int ring_pos = 0, until_step = W;
    int64_t step = 0;
    int accepted = 0;
    bool have_parent = false;
    double ln_par[3] = {0.0, 0.0, 0.0}, ln_cur[3] = {0.0, 0.0, 0.0};
    double f_par = 0.0, sigma = 0.0;
    if (ONLINE) {
        for (int k = 0; k < 3; ++k) ln_par[k] = ln_cur[k] = a.ln_theta0[3 * (size_t)p + k];
        sigma = a.tuner[12];
        if (W + lane < ((W + 7) & ~7)) ring[W + lane] = INFINITY;     // padding (entries below W are written before use)
        wave_sync();
    }
    const double sc = a.scale[p];
    double my_rtt = lane < R ? (PROXY ? a.rtt_true[lane] : a.rtt[lane]) : 0.0;
    // imperfect proxy knowledge (Sec. 2.2, Sec. 4 RTT figure): time is cut into probe epochs, the epoch of t being
    // the largest e with e * probe_ms <= t (capped at the last one given); a request experiences the true round
    // trip time of its epoch, the cost model scores with the proxy's moving average, handed to the cache wavefront
    // with the load signals
    int epoch = 0;
    double next_probe = PROXY ? (double)a.probe_ms : 0.0;
    if (PROXY) st(&comm->rtt[lane], lane < R ? a.rtt_est[lane] : 0.0);
    // engine model: this lane's replica has its own rates and KV budget
    const double my_a_pf = ENGINE && lane < R ? a.eng_a_pf[lane] : 0.0;
    const double my_a_dec = ENGINE && lane < R ? a.eng_a_dec[lane] : 0.0;
    const double my_budget = ENGINE && lane < R ? a.eng_budget[lane] : 0.0;
    Rec* const rec = a.rec + (size_t)p * N;
    bool dead = false;
    for (int64_t r0 = 0; r0 < N && !dead; r0 += WAVE) {
        const int nb = N - r0 < WAVE ? (int)(N - r0) : WAVE;
        const int64_t rr = r0 + (lane < nb ? lane : nb - 1);
        const double m_t = (double)a.ts[rr] * sc;          // time scale: gaps scale linearly
        const int m_L = a.in_len[rr];
        const int m_O = a.out_len[rr];
        double o_ttft = 0.0, o_e2e = 0.0;
        for (int i = 0; i < nb; ++i) {
            const int64_t r = r0 + i;
            const double t = readlane_f64(m_t, i);
            const int L = __builtin_amdgcn_readlane(m_L, i);
            const int O = __builtin_amdgcn_readlane(m_O, i);
            if (PROXY) {
                bool moved = false;
                while (epoch + 1 < a.epochs && next_probe <= t) {       // (timestamps do not decrease)
                    ++epoch;
                    next_probe = (double)(epoch + 1) * (double)a.probe_ms;
                    moved = true;
                }
                if (moved) {
                    const size_t at = (size_t)epoch * R + (lane < R ? lane : 0);
                    my_rtt = a.rtt_true[at];
                    st(&comm->rtt[lane], a.rtt_est[at]);
                }
            }
            Q.retire(t, rec);
            // (the least-request policy asks for requests in flight instead of their tokens)
            st(&comm->q[lane], MODE == MODE_LEAST_REQUEST ? Q.my_cnt : Q.my_q);
            lds_release();
            if (lane == 0) st(&comm->seq_q, (unsigned)(r + 1));
            // While the cache wavefront decides, the completions up to the next request's time are retired
            // already: they do not depend on where this request goes (only this request's own completion is
            // left for the retire above, next time round).  The service step still has to see the slots that
            // were idle at this request's time, so their set is kept.
            const unsigned long long idle_now = Q.idle;
            if (r + 1 < N) {
                const double t_next = i + 1 < nb ? readlane_f64(m_t, i + 1) : (double)a.ts[r + 1] * sc;
                Q.retire(t_next, rec);
            }
            const unsigned want = (unsigned)(r + 1) & 0x3FFFFFFu;
            unsigned hi, lo;
            for (int spins = 0;; ++spins) {
                const unsigned long long w = ld(&comm->choice);
                hi = __builtin_amdgcn_readfirstlane((unsigned)(w >> 32));
                lo = __builtin_amdgcn_readfirstlane((unsigned)w);
                if ((hi >> 6) == want) break;
                if (spins > a.spin_limit || ld(&comm->abandoned) != 0) {
                    dead = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            if (dead) break;
            const int best = (int)(hi & 63u);
            double ttft, e2e;
            if (ENGINE)
                Q.template serve_engine<PROXY>(r, best, t, my_rtt, (int64_t)(int)lo, L, O, my_a_pf, my_a_dec, my_budget, a.eng_slowdown,
                               rec, lane, &ttft, &e2e);
            else
                Q.template serve<PROXY>(r, best, t, my_rtt, (int64_t)(int)lo, L, O, a.a_pf, a.a_dec, rec, lane, idle_now,
                                        &ttft, &e2e);
            o_ttft = lane == i ? ttft : o_ttft;
            o_e2e = lane == i ? e2e : o_e2e;
            if (ONLINE) {
                if (lane == 0) ring[ring_pos] = ttft;
                ring_pos = ring_pos + 1 == W ? 0 : ring_pos + 1;
                if (--until_step == 0) {
                    until_step = H;
                    wave_sync();
                    const double f = window_kth(ring, W, kth, lane);
                    if (!have_parent) {
                        f_par = f;                 // the first window measures the initial weights: the parent
                        have_parent = true;
                    } else {
                        const bool success = f < f_par;
                        if (success) {
                            for (int k = 0; k < 3; ++k) ln_par[k] = ln_cur[k];
                            f_par = f;
                            ++accepted;
                        }
                        sigma = sigma * (success ? a.tuner[13] : a.tuner[14]);
                    }
                    double th[3];
                    for (int k = 0; k < 3; ++k) {
                        const double zk = a.z[((size_t)p * a.steps + step) * 3 + k];
                        const double moved = ln_par[k] + sigma * zk;
                        ln_cur[k] = clip(moved, a.tuner[6 + k], a.tuner[9 + k]);
                        th[k] = clip(tuner_exp(ln_cur[k]), a.tuner[k], a.tuner[3 + k]);
                    }
                    if (lane == 0) {
                        for (int k = 0; k < 3; ++k) st(&comm->w[k], th[k]);    // published with the next load signals
                        if (a.fitness_step) a.fitness_step[(size_t)p * a.steps + step] = f;
                        if (a.theta_step)
                            for (int k = 0; k < 3; ++k) a.theta_step[((size_t)p * a.steps + step) * 3 + k] = th[k];
                    }
                    ++step;
                    wave_sync();
                }
            }
        }
        if (lane < nb && !dead) {
            const size_t o = (size_t)p * N + r0 + lane;
            if (a.ttft) a.ttft[o] = o_ttft;
            if (a.e2e) a.e2e[o] = o_e2e;
        }
    }
    if (ONLINE && lane == 0 && !dead) {
        if (a.theta_final)
            for (int k = 0; k < 3; ++k)
                a.theta_final[3 * (size_t)p + k] = clip(tuner_exp(ln_par[k]), a.tuner[k], a.tuner[3 + k]);
        if (a.sigma_final) a.sigma_final[p] = sigma;
        if (a.accepted) a.accepted[p] = accepted;
    }
    if (dead) {
        // the partner never answered (cannot happen unless the kernel is wrong): leave, and make sure nobody
        // mistakes this replay's latencies for results
        st(&comm->abandoned, 1);
        for (int64_t x = lane; x < N; x += WAVE) {
            if (a.ttft) a.ttft[(size_t)p * N + x] = NAN;
            if (a.e2e) a.e2e[(size_t)p * N + x] = NAN;
        }
    }
}

// Eviction cursor of one LRU over a replica's log of routed requests, held by lane = replica.
//   cursor: blocks last touched by a request before cur_r, or by cur_r at positions >= cur_k, are evicted;
//   cur_own is where cur_r's owned suffix starts.
//   nx_*, n2_*: the next two records of the replica's log that still own blocks (r < 0: empty).
//   fill_r: the record after the last one held here, or -1 when that one is the youngest of the log.
//   pend_*: a record being fetched (its load is only waited for one iteration later); changes made to it
//   meanwhile are kept in pend_own / pend_next and override the loaded fields.
// The kernel keeps the cursor of the replica's cache in plain local variables of the same names (the compiler
// does measurably better with them); this struct is the same machinery for the proxy's own index of the replica,
// an LRU of another capacity over the same log.
struct EvictCursor {
    int cur_r = -1, cur_k = 0, cur_own = 0;
    int nx_r = -1, nx_n = 0, nx_own = 0;
    int n2_r = -1, n2_n = 0, n2_own = 0;
    int fill_r = -1;
    int pend_r = -1, pend_own = -1, pend_next = -1;
    unsigned long long pend_raw = 0;
    int live = 0;             // blocks this LRU holds

    // the fetched record becomes usable: dropped if it owns nothing, else queued behind nx / n2
    __device__ __forceinline__ void take_pending(unsigned long long raw) {
        if (pend_r >= 0) {
            const int n = (int)(raw >> 48);
            const int own_mem = (int)((raw >> 32) & 0xFFFF);
            const int own = pend_own > own_mem ? pend_own : own_mem;
            const int next = pend_next >= 0 ? pend_next : (int)(unsigned int)raw;
            if (own < n) {
                if (nx_r < 0) {
                    nx_r = pend_r;
                    nx_n = n;
                    nx_own = own;
                } else {
                    n2_r = pend_r;
                    n2_n = n;
                    n2_own = own;
                }
            }
            fill_r = next;
            pend_r = -1;
        }
    }
    // fetch the next record of the log if there is room for it
    __device__ __forceinline__ void issue_fill(const unsigned long long* log64) {
        if (pend_r < 0 && fill_r >= 0 && n2_r < 0) {
            pend_r = fill_r;
            pend_own = -1;
            pend_next = -1;
            pend_raw = ld(&log64[fill_r]);
        }
    }
    // request `owner`'s owned suffix now starts at `end`
    __device__ __forceinline__ void disowned(int owner, int end) {
        cur_own = owner == cur_r ? end : cur_own;
        nx_own = owner == nx_r ? end : nx_own;
        n2_own = owner == n2_r ? end : n2_own;
        pend_own = owner == pend_r ? end : pend_own;
    }
    // request r (n blocks) has become the youngest record of the log of the replica whose lane has is_best set;
    // tail_r is the youngest before it
    __device__ __forceinline__ void appended(bool is_best, int r, int n, int tail_r) {
        const bool first = is_best && tail_r < 0;
        const bool to_pend = is_best && pend_r >= 0 && pend_r == tail_r;
        const bool to_fill = is_best && !first && !to_pend && pend_r < 0 && fill_r < 0;
        cur_r = first ? r : cur_r;
        cur_k = first ? n : cur_k;
        cur_own = first ? 0 : cur_own;
        pend_next = to_pend ? r : pend_next;
        fill_r = to_fill ? r : fill_r;
    }
    // `added` blocks have joined the LRU of the lane with `active` set; the cursor moves forward until the LRU
    // fits `cap` blocks again.  Up to two steps come from the records held in registers; more (rare) are
    // fetched on the spot.
    __device__ __forceinline__ void evict(bool active, int added, int cap, const unsigned long long* log64) {
        live += active ? added : 0;
        int E = active ? live - cap : 0;
        E = E > 0 ? E : 0;
        live -= E;
        if (__ballot(E > 0) != 0) {
            {
                int avail = cur_k - cur_own;
                avail = avail > 0 ? avail : 0;
                const int take = avail < E ? avail : E;
                cur_k -= take;
                E -= take;
            }
            while (E > 0) {       // only the chosen replica's lane can be here
                if (nx_r < 0) {
                    // fetch a record on the spot; pend_raw itself is only ever written by the look-ahead
                    // fetch, so that its load is never waited for in here
                    unsigned long long raw = pend_raw;
                    if (pend_r < 0) {
                        if (fill_r < 0) break;      // cannot happen while E > 0; bounds the loop
                        pend_r = fill_r;
                        pend_own = -1;
                        pend_next = -1;
                        raw = ld(&log64[fill_r]);
                    }
                    take_pending(raw);
                    continue;
                }
                cur_r = nx_r;
                cur_k = nx_n;
                cur_own = nx_own;
                nx_r = n2_r;
                nx_n = n2_n;
                nx_own = n2_own;
                n2_r = -1;
                int avail = cur_k - cur_own;
                avail = avail > 0 ? avail : 0;
                const int take = avail < E ? avail : E;
                cur_k -= take;
                E -= take;
            }
            live += E;            // nothing left to evict (unreachable, kept consistent)
        }
    }
};

template <int MODE, bool ENGINE, bool PROXY>
__global__ void __launch_bounds__(SEG_THREADS) replay_segments_kernel(SegArgs a) {
    constexpr bool ONLINE = MODE == MODE_ONLINE;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ SegRef stage[SEG_STAGE + SEG_CHUNK];    // padded: whole chunks are read unconditionally
    __shared__ SegComm comm;
    const int lane = threadIdx.x & (WAVE - 1);
    const int p = blockIdx.x;
    const int R = a.R;
    const int64_t N = a.N;
    const int C = (int)a.C;

    if (threadIdx.x == 0) {
        comm.seq_q = 0;
        comm.abandoned = 0;
        comm.choice = 0;
        for (int k = 0; k < 3; ++k) comm.w[k] = a.params[3 * (size_t)p + k];
    }
    __syncthreads();
    if (threadIdx.x >= WAVE) {
        queue_wave<MODE, ENGINE, PROXY>(a, p, lane, lds_raw, &comm);
        return;
    }
    __builtin_amdgcn_s_setprio(3);      // the cache wavefront has the longer loop: it goes first at issue
    bool dead = false;

    for (int x = lane; x < SEG_CHUNK; x += WAVE) stage[SEG_STAGE + x] = SegRef{0, 0};
    wave_sync();

    const uint64_t seed = MODE == MODE_RANDOM ? a.seeds[p] : 0;
    const uint32_t seed_lo = (uint32_t)seed, seed_hi = (uint32_t)(seed >> 32);
    // (with the online tuner the weights come with the load signals instead)
    const double w_rtt = a.params[3 * (size_t)p + 0];
    const double w_prefill = a.params[3 * (size_t)p + 1];
    const double w_queue = a.params[3 * (size_t)p + 2];
    const double my_rtt = !PROXY && lane < R ? a.rtt[lane] : 0.0;     // (proxy variants: comes with the load signals)
    // Proxy variants (Sec. 7: the proxy does not see replica-side eviction): the proxy keeps an index of its own
    // of what it dispatched to each replica, an LRU like the replica's cache but at least as large (or unbounded).
    // It sees the same touches, so it is the same rows read against a second eviction cursor (c2), which lags
    // the replica's; the match loop yields both prefixes, Eq. 3 scores with the index's.  Ownership is kept for
    // what the index holds, a superset of what is cached, which the replica's eviction walk does not mind:
    // records behind its cursor are never looked at again.  While the index never forgets (or is not used) its
    // cursor stays at the replica's first record and "in the index" means "ever dispatched here".
    const bool own_index = PROXY && a.index_blocks >= 0;
    const int index_cap = PROXY && a.index_blocks > 0 ? (int)a.index_blocks : 0;
    EvictCursor c2;                           // the index's cursor, as cur_* etc. below

    // Per-replica eviction state, held by lane = replica.
    //   cursor: blocks last touched by a request before cur_r, or by cur_r at positions >= cur_k, are
    //   evicted; cur_own is where cur_r's owned suffix starts.
    //   nx_*, n2_*: the next two records of the replica's log that still own blocks (r < 0: empty).
    //   fill_r: the record after the last one held here, or -1 when that one is the youngest of the log.
    //   pend_*: a record being fetched (its load is only waited for one iteration later); changes made to
    //   it meanwhile are kept in pend_own / pend_next and override the loaded fields.
    int cur_r = -1, cur_k = 0, cur_own = 0;
    int nx_r = -1, nx_n = 0, nx_own = 0;
    int n2_r = -1, n2_n = 0, n2_own = 0;
    int fill_r = -1;
    int pend_r = -1, pend_own = -1, pend_next = -1;
    unsigned long long pend_raw = 0;
    int tail_r = -1;          // youngest request routed to this replica
    int my_live = 0;          // blocks cached on this replica

    int32_t* const last = a.last + (size_t)p * a.nseg * R;
    // this lane's cell of a segment's row; rows of one replay span less than 4 GiB (checked by the host)
    const unsigned lane_off = (unsigned)(lane < R ? lane : 0) * 4u;
    const unsigned row_bytes = (unsigned)R * 4u;
    auto cell_at = [&](int seg_id) -> int32_t* {
        return reinterpret_cast<int32_t*>(reinterpret_cast<char*>(last) + ((unsigned)seg_id * row_bytes + lane_off));
    };
    LogRec* const log = a.log + (size_t)p * N;
    unsigned long long* const log64 = reinterpret_cast<unsigned long long*>(log);

    // the fetched record becomes usable: dropped if it owns nothing, else queued behind nx / n2
    auto take_pending = [&](unsigned long long raw) {
        if (pend_r >= 0) {
            const int n = (int)(raw >> 48);
            const int own_mem = (int)((raw >> 32) & 0xFFFF);
            const int own = pend_own > own_mem ? pend_own : own_mem;
            const int next = pend_next >= 0 ? pend_next : (int)(unsigned int)raw;
            if (own < n) {
                if (nx_r < 0) {
                    nx_r = pend_r;
                    nx_n = n;
                    nx_own = own;
                } else {
                    n2_r = pend_r;
                    n2_n = n;
                    n2_own = own;
                }
            }
            fill_r = next;
            pend_r = -1;
        }
    };
    // fetch the next record of the log if there is room for it
    auto issue_fill = [&]() {
        if (pend_r < 0 && fill_r >= 0 && n2_r < 0) {
            pend_r = fill_r;
            pend_own = -1;
            pend_next = -1;
            pend_raw = ld(&log64[fill_r]);
        }
    };

    int64_t r0 = 0;
    while (r0 < N && !dead) {
        // ---- stage a batch of up to 64 requests: per-request scalars in registers (lane = request), their
        // segment references in LDS.  The batch is cut where the references stop fitting; a single request
        // with more references than the stage holds is processed alone, reading them from global memory.
        const int nb0 = N - r0 < WAVE ? (int)(N - r0) : WAVE;
        const int64_t rr = r0 + (lane < nb0 ? lane : nb0 - 1);
        const int m_L = a.in_len[rr];
        const uint32_t m_hash = MODE == MODE_AFFINITY ? a.first_hash[rr] : 0u;
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
                m_n = stage[m_a0 + m_s - 1].end;
                m_root = stage[m_a0].id;
            }
        } else if (m_s > 0 && lane == 0) {
            m_n = gref[m_s - 1].end;
            m_root = gref[0].id;
        }

        int o_route = 0, o_hit = 0, o_believed = 0;

        // requests the rows of the first SEG_CHUNK segments of request i of the batch.  The references are
        // read four at a time (one LDS round trip), most requests having no more than four segments.
        auto request_rows = [&](int i, auto ref, RowSet& w) {
            const int a0 = __builtin_amdgcn_readlane(m_a0, i);
            const int s = __builtin_amdgcn_readlane(m_s, i);
            const int n = __builtin_amdgcn_readlane(m_n, i);
            w.of_lane = ref(a0 + (lane < SEG_CHUNK ? lane : 0), lane < s && lane < SEG_CHUNK);
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
                    w.end[h + k] = sr[k].end;
                    w.cell[h + k] = ld(cell_at(sr[k].id));           // lanes beyond R read a neighbouring cell, unused
                }
            }
        };

        // Processes request i of the batch.  `mine` holds the rows of its first segments; `other` receives
        // those of request i+1.
        auto process = [&](int i, auto ref, RowSet& mine, RowSet& other) {
            const int64_t r = r0 + i;
            const int L = __builtin_amdgcn_readlane(m_L, i);
            const int a0 = __builtin_amdgcn_readlane(m_a0, i);
            const int s = __builtin_amdgcn_readlane(m_s, i);
            const int n = __builtin_amdgcn_readlane(m_n, i);

            // ---- prefix match: lane = replica.  A request that touches a segment touches all its ancestors,
            // so along the path the cells never increase: first the segments touched after the cursor's
            // request (cached), then those it touched last itself (cached below the cursor position), then
            // older ones (evicted).  The match is max(e_gt, min(cur_k, e_ge)) with e_gt, e_ge the ends of the
            // last segment whose cell is above, respectively not below, the cursor's request.
            int e_gt = 0, e_ge = 0;
            int32_t own_gt = -1;        // previous owner of the last segment counted in e_gt
            int e_gt2 = 0, e_ge2 = 0;   // proxy variants: the same against the index's cursor
            int32_t own_gt2 = -1;
#pragma unroll
            for (int k = 0; k < SEG_CHUNK; ++k) {
                if (k >= s) break;
                const bool gt = mine.cell[k] > cur_r;
                const bool ge = mine.cell[k] >= cur_r;
                e_gt = gt ? mine.end[k] : e_gt;
                own_gt = gt ? mine.cell[k] : own_gt;
                e_ge = ge ? mine.end[k] : e_ge;
                if (PROXY) {
                    const bool gt2 = mine.cell[k] > c2.cur_r;
                    const bool ge2 = mine.cell[k] >= c2.cur_r;
                    e_gt2 = gt2 ? mine.end[k] : e_gt2;
                    own_gt2 = gt2 ? mine.cell[k] : own_gt2;
                    e_ge2 = ge2 ? mine.end[k] : e_ge2;
                }
            }
            const int below_cursor = cur_k < e_ge ? cur_k : e_ge;
            const bool some_eq = below_cursor > e_gt;       // blocks of the cursor's own request are matched
            int my_m = some_eq ? below_cursor : e_gt;
            const int below_cursor2 = c2.cur_k < e_ge2 ? c2.cur_k : e_ge2;
            const bool some_eq2 = below_cursor2 > e_gt2;
            int my_seen = PROXY ? (some_eq2 ? below_cursor2 : e_gt2) : 0;       // blocks in the proxy's index (>= my_m)
            // For the ownership update below: where the cached prefix ends on this replica (rounded up to the
            // end of a segment that the cursor's request owns: what lies beyond the cursor is evicted anyway)
            // and whether all cached segments had the same previous owner.  (Proxy variants: the same for the
            // prefix in the index.)
            const int k_end = PROXY ? (some_eq2 ? e_ge2 : e_gt2) : (some_eq ? e_ge : e_gt);
            const bool one_owner = PROXY ? (some_eq2 ? e_gt2 == 0 : own_gt2 == mine.cell[0])
                                         : (some_eq ? e_gt == 0 : own_gt == mine.cell[0]);
            int pos = mine.end[SEG_CHUNK - 1];
            bool open = my_m == pos;
            bool open_seen = PROXY && my_seen == pos;
            bool deep = false;          // the match went past the preloaded segments
            if (s > SEG_CHUNK && __ballot((PROXY ? open_seen : open) && lane < R) != 0) {      // (pos and open only matter in here)
                deep = true;
                for (int c0 = SEG_CHUNK; c0 < s; c0 += SEG_CHUNK) {
                    int32_t cell[SEG_CHUNK];
                    int send[SEG_CHUNK];
#pragma unroll
                    for (int k = 0; k < SEG_CHUNK; ++k) {
                        cell[k] = -1;
                        send[k] = pos;
                        if (c0 + k < s) {
                            const SegRef sr = ref(a0 + c0 + k, true);
                            send[k] = sr.end;
                            if ((PROXY ? open_seen : open) && lane < R) cell[k] = ld(cell_at(sr.id));
                        }
                    }
#pragma unroll
                    for (int k = 0; k < SEG_CHUNK; ++k) {
                        if (c0 + k < s) {
                            const int cnt = cached_in(cell[k], pos, send[k], cur_r, cur_k);
                            my_m += open ? cnt : 0;
                            open = open && cnt == send[k] - pos;
                            if (PROXY) {
                                const int cnt_seen = cached_in(cell[k], pos, send[k], c2.cur_r, c2.cur_k);
                                my_seen += open_seen ? cnt_seen : 0;
                                open_seen = open_seen && cnt_seen == send[k] - pos;
                            }
                            pos = send[k];
                        }
                    }
                    if (__ballot((PROXY ? open_seen : open) && lane < R) == 0) break;
                }
            }

            // ---- the single point of the iteration that waited for memory is behind us: the record fetched
            // during the previous iteration becomes usable, and the loads for the next iteration go out
            take_pending(pend_raw);
            if (PROXY && index_cap > 0) c2.take_pending(c2.pend_raw);
            if (i + 1 < nb) request_rows(i + 1, ref, other);
            issue_fill();
            if (PROXY && index_cap > 0) c2.issue_fill(log64);

            // ---- score (Eq. 3) and lowest-index minimum
            int hit_tok = a.block_tokens * my_m;           // block_tokens * blocks fits: both are below 2^16
            hit_tok = hit_tok > L ? L : hit_tok;
            int my_u = L - hit_tok;
            int my_u_seen = my_u;       // uncached tokens as Eq. 3 sees them
            if (PROXY) {
                int seen_tok = a.block_tokens * (own_index ? my_seen : my_m);
                seen_tok = seen_tok > L ? L : seen_tok;
                my_u_seen = L - seen_tok;
            }
            // the load signals of this request come from the queue wavefront (normally already there);
            // everything that does not need them is finished first, so that little is left between reading
            // them and announcing the choice
            const double score_rp = ONLINE || PROXY ? 0.0 : eq3_without_queue(w_rtt, w_prefill, my_rtt, a.a_pf, my_u);
            asm volatile("" : "+v"(my_u), "+v"(my_m));
            double score_rp_ready = score_rp;
            asm volatile("" : "+v"(score_rp_ready));
            double my_q;
            double now_rtt = 0.0, now_prefill = 0.0, now_queue = 0.0;
            double rtt_est = my_rtt;
            for (int spins = 0;; ++spins) {
                const unsigned seq = __builtin_amdgcn_readfirstlane(ld(&comm.seq_q));
                lds_acquire();
                my_q = ld(&comm.q[lane]);
                if (PROXY) rtt_est = ld(&comm.rtt[lane]);
                if (ONLINE) {
                    now_rtt = ld(&comm.w[0]);
                    now_prefill = ld(&comm.w[1]);
                    now_queue = ld(&comm.w[2]);
                }
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
            double my_score;
            if (MODE == MODE_COST_MODEL) {
                my_score = PROXY ? eq3_score(w_rtt, w_prefill, w_queue, rtt_est, a.a_pf, my_u_seen, my_q)
                                 : eq3_with_queue(score_rp_ready, w_queue, a.a_pf, my_q);
            } else if (MODE == MODE_ONLINE) {
                my_score = eq3_score(now_rtt, now_prefill, now_queue, rtt_est, a.a_pf, my_u_seen, my_q);
            } else if (MODE == MODE_LEAST_REQUEST) {
                my_score = my_q;                    // requests in flight
            } else {
                // the replica is dictated: by the hash of the first block, or by a counter-based draw
                const int target = MODE == MODE_AFFINITY ? (s > 0 ? spread((uint32_t)__builtin_amdgcn_readlane((int)m_hash, i), R) : 0)
                                                         : spread(philox4x32_10_first((uint32_t)r, (uint32_t)((uint64_t)r >> 32),
                                                                                      seed_lo, seed_hi), R);
                my_score = lane == target ? 0.0 : 1.0;
            }
            const int best = wave_argmin(my_score, lane, R);
            const bool is_best = lane == best;
            const int m_best = __builtin_amdgcn_readlane(my_m, best);
            const int seen_best = PROXY ? __builtin_amdgcn_readlane(my_seen, best) : m_best;
            if (lane == 0) {
                const unsigned u_best = (unsigned)__builtin_amdgcn_readlane(my_u, best);
                const unsigned tag = (((unsigned)(r + 1) & 0x3FFFFFFu) << 6) | (unsigned)best;
                st(&comm.choice, ((unsigned long long)tag << 32) | u_best);
            }

            // ---- ownership: the segments this request takes over on the chosen replica stop belonging to
            // their previous requests.  Along the path the previous owners form runs; each run moves its
            // owner's `own` to the end of the run.  Only cached segments matter (evicted ones belong to
            // requests the cursor has passed, or to the cursor request beyond its position).
            auto disown = [&](int owner, int end) {       // lane `best`: owner's owned suffix now starts at end
                st(&log[owner].own, (uint16_t)end);
                cur_own = owner == cur_r ? end : cur_own;
                nx_own = owner == nx_r ? end : nx_own;
                n2_own = owner == n2_r ? end : n2_own;
                pend_own = owner == pend_r ? end : pend_own;
                if (PROXY) c2.disowned(owner, end);
            };
            if (seen_best > 0) {
                const bool simple = !deep && __builtin_amdgcn_readlane((int)one_owner, best) != 0;
                if (simple) {
                    if (is_best) disown(mine.cell[0], k_end);
                } else {
                    // several previous owners, or a prefix longer than the preloaded rows: walk it
                    const int cb_r = __builtin_amdgcn_readlane(PROXY ? c2.cur_r : cur_r, best);
                    const int cb_k = __builtin_amdgcn_readlane(PROXY ? c2.cur_k : cur_k, best);
                    int run_owner = -1, run_end = 0, vpos = 0;
                    for (int j = 0; j < s; ++j) {
                        const SegRef sr = ref(a0 + j, true);
                        const int32_t rl = ld(&last[(size_t)sr.id * R + best]);
                        const int cnt = cached_in(rl, vpos, sr.end, cb_r, cb_k);
                        if (cnt > 0) {
                            if (rl != run_owner) {
                                if (run_owner >= 0 && is_best) disown(run_owner, run_end);
                                run_owner = rl;
                            }
                            run_end = sr.end;
                        }
                        if (cnt != sr.end - vpos) break;
                        vpos = sr.end;
                    }
                    if (run_owner >= 0 && is_best) disown(run_owner, run_end);
                }
            }

            // ---- cache update: every segment of the request is now last touched by r on the chosen replica
            // (lane k stores the cell of segment k)
            if (lane < s && lane < SEG_CHUNK) st(&last[(size_t)mine.of_lane.id * R + best], (int32_t)r);
            for (int j = SEG_CHUNK + lane; j < s; j += WAVE)
                st(&last[(size_t)ref(a0 + j, true).id * R + best], (int32_t)r);

            // ---- log and eviction, in the chosen replica's lane
            if (is_best) {
                st(&log64[r], 0xFFFFFFFFull | ((unsigned long long)n << 48));      // next -1, own 0, n
                if (tail_r >= 0) st(&log[tail_r].next, (int32_t)r);
            }
            {
                // r is now the youngest record of the chosen replica's log
                const bool first = is_best && tail_r < 0;
                const bool to_pend = is_best && pend_r >= 0 && pend_r == tail_r;
                const bool to_fill = is_best && !first && !to_pend && pend_r < 0 && fill_r < 0;
                cur_r = first ? (int)r : cur_r;
                cur_k = first ? n : cur_k;
                cur_own = first ? 0 : cur_own;
                if (PROXY) c2.appended(is_best, (int)r, n, tail_r);
                pend_next = to_pend ? (int)r : pend_next;
                fill_r = to_fill ? (int)r : fill_r;
                tail_r = is_best ? (int)r : tail_r;

                // eviction: move the cursor forward until the cache fits.  Up to two steps come from the
                // records held in registers; more (rare) are fetched on the spot.
                my_live += (is_best && C > 0) ? n - m_best : 0;
                int E = (is_best && C > 0) ? my_live - C : 0;
                E = E > 0 ? E : 0;
                my_live -= E;
                if (__ballot(E > 0) != 0) {
                    {
                        int avail = cur_k - cur_own;
                        avail = avail > 0 ? avail : 0;
                        const int take = avail < E ? avail : E;
                        cur_k -= take;
                        E -= take;
                    }
                    while (E > 0) {       // only the chosen replica's lane can be here
                        if (nx_r < 0) {
                            // fetch a record on the spot; pend_raw itself is only ever written by the
                            // look-ahead fetch, so that its load is never waited for in here
                            unsigned long long raw = pend_raw;
                            if (pend_r < 0) {
                                if (fill_r < 0) break;      // cannot happen while E > 0; bounds the loop
                                pend_r = fill_r;
                                pend_own = -1;
                                pend_next = -1;
                                raw = ld(&log64[fill_r]);
                            }
                            take_pending(raw);
                            continue;
                        }
                        cur_r = nx_r;
                        cur_k = nx_n;
                        cur_own = nx_own;
                        nx_r = n2_r;
                        nx_n = n2_n;
                        nx_own = n2_own;
                        n2_r = -1;
                        int avail = cur_k - cur_own;
                        avail = avail > 0 ? avail : 0;
                        const int take = avail < E ? avail : E;
                        cur_k -= take;
                        E -= take;
                    }
                    my_live += E;         // nothing left to evict (unreachable, kept consistent)
                }
                // the proxy's index evicts under its own capacity: its cursor walks the same log (whose memory
                // is up to date: ownership changes and links are stored as they happen)
                if (PROXY && index_cap > 0) c2.evict(is_best, n - seen_best, index_cap, log64);
            }

            // ---- the rows of request i+1 were requested before this request's stores: if it continues the
            // same tree, the cells this request just wrote are patched into them (common prefix of the paths)
            if (i + 1 < nb && s > 0 && __builtin_amdgcn_readlane(m_root, i + 1) == __builtin_amdgcn_readlane(m_root, i)) {
                const int s_next = __builtin_amdgcn_readlane(m_s, i + 1);
                const bool same = lane < s && lane < s_next && other.of_lane.id == mine.of_lane.id &&
                                  other.of_lane.end == mine.of_lane.end;
                const unsigned differ = ~(unsigned)__ballot(same && lane < SEG_CHUNK) | (1u << SEG_CHUNK);
                const int common = __ffs(differ) - 1;              // leading segments the two paths share
#pragma unroll
                for (int k = 0; k < SEG_CHUNK; ++k) other.cell[k] = (k < common && is_best) ? (int32_t)r : other.cell[k];
            }

            // ---- outputs of the cache side (kept in registers until the batch ends)
            if (a.route) o_route = lane == i ? best : o_route;
            if (a.hit) o_hit = lane == i ? m_best : o_hit;
            if (PROXY && a.believed) o_believed = lane == i ? (own_index ? seen_best : m_best) : o_believed;
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
            const size_t o = (size_t)p * N + r0 + lane;
            if (a.route) a.route[o] = (uint8_t)o_route;
            if (a.hit) a.hit[o] = (uint16_t)o_hit;
            if (PROXY && a.believed) a.believed[o] = (uint16_t)o_believed;
        }
        wave_sync();
        r0 += nb;
    }
}

}  // namespace gorgo

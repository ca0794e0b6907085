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
// every four to five cycles whatever its kind (a branch costs three to four times that), so the kernel is
// arranged around the instruction count of that chain, not around bandwidth.  A replay is run by two
// wavefronts of one workgroup that meet at two workgroup barriers per request.
//   The cache wavefront (lane = replica) holds the cache side in registers: eviction cursor, the next log
// records, the row cells of the current and the next request.  Per request it matches, scores, takes the
// minimum, announces the choice, then updates rows, log and cursor.  It does nothing else.
//   The queue wavefront (lane = replica) owns the service slots (LDS) and the load signal: before request r it
// retires what has completed by t_r and publishes every replica's queue term of Eq. 3; after the choice it
// serves the request and keeps the latencies and the per-request outputs.  It has the shorter chain, so it
// also is the trace's front end: three requests ahead it reads the request's segment references and leaves a
// descriptor in a small LDS ring -- row offsets, end positions, flags -- from which the cache wavefront
// issues its row loads without any address arithmetic or staging of its own.
//   Barrier A(r): the queue terms of r are published (and the descriptor of r + 1 is complete).  Barrier
// B(r): the choice of r is published.  Every wavefront executes exactly two barriers per request, whatever
// the data, so neither can wait for ever.
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
    unsigned long long* sections; // timed instantiation only: [P][3][SECTIONS] cycles per section (cache, queue, front-end wavefront)
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
constexpr int SEG_THREADS = 2 * WAVE;        // two replays per wavefront pair: cache wavefront + queue wavefront
constexpr int SEG3_THREADS = 3 * WAVE;       // cache, queue and front-end wavefront
constexpr int SEG_SPIN_LIMIT = 1 << 24;      // default: polls of a hand-over word before the replay is given up (~1 s)

// Fences between LDS data and the word that announces it (two replays per wavefront pair still hand over
// through polled words): the LDS executes the instructions of one wavefront in the order they were issued, so
// the fences only have to keep the compiler from changing that order, and cost no wait.
__device__ __forceinline__ void lds_release() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); }
__device__ __forceinline__ void lds_acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront"); }

// Orders the LDS accesses of one wavefront's lanes (the hardware executes them in program order).
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__host__ __device__ inline size_t replay_segments_lds_bytes(int R, int B, int window) {   // dynamic part
    // queues (in whichever layout is the larger: the launch picks one), then the tuner's TTFT window
    const size_t q = Queues::bytes(R, B) > SlotQueues::bytes() ? Queues::bytes(R, B) : SlotQueues::bytes();
    return q + (size_t)((window + 7) & ~7) * sizeof(double);
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

// k-th smallest (1-based) of the W values of `ring` (LDS, W <= 1024), by taking elements out from the nearer end: the
// largest W + 1 - k times, or the smallest k times (the tuner's k is the 95th percentile's: 7 rounds for a window
// of 128, against 128 comparisons for every element when the elements are ranked by counting).  Lane l looks after
// the elements l, l + 64, ...; a round takes this lane's best remaining element, finds the best over the wavefront
// (two 32-bit cross-lane reductions on the order-preserving integer image of the doubles, the second one only when
// the high words tie) and marks it as taken in the lowest lane that holds it.  Equal values are taken one by one, as
// a sorted list would have them.
__device__ __forceinline__ double window_kth(const double* ring, int W, int kth, int lane) {
    const bool from_top = W + 1 - kth <= kth;
    const int rounds = from_top ? W + 1 - kth : kth;
    unsigned taken = 0;                 // bit c: element c * 64 + lane is out
    unsigned last_hi = 0, last_lo = 0;
    // the wanted end is the largest key: the order-preserving integer image of the value, complemented from the bottom
    auto key_of = [&](int e) {
        const unsigned long long b = (unsigned long long)__double_as_longlong(ring[e]);
        const unsigned long long up = (b >> 63) ? ~b : (b | 0x8000000000000000ull);      // increasing with the value
        return from_top ? up : ~up;
    };
    // (this lane's first two elements stay in registers: windows of up to 128 values read LDS once)
    const bool has0 = lane < W, has1 = lane + WAVE < W;
    const unsigned long long key0 = has0 ? key_of(lane) : 0, key1 = has1 ? key_of(lane + WAVE) : 0;
    for (int round = 0; round < rounds; ++round) {
        const bool use0 = has0 && (taken & 1u) == 0;
        unsigned long long best = use0 ? key0 : 0;
        int best_c = use0 ? 0 : -1;
        const bool use1 = has1 && (taken & 2u) == 0 && (best_c < 0 || key1 > best);
        best = use1 ? key1 : best;
        best_c = use1 ? 1 : best_c;
        for (int c = 2, e = lane + 2 * WAVE; e < W; ++c, e += WAVE) {
            const unsigned long long key = key_of(e);
            const bool better = ((taken >> c) & 1u) == 0 && (best_c < 0 || key > best);
            best = better ? key : best;
            best_c = better ? c : best_c;
        }
        const bool have = best_c >= 0;
        const unsigned hi = (unsigned)(best >> 32), lo = (unsigned)best;
        const unsigned top_hi = ~wave_min_u32(~(have ? hi : 0u));
        const bool tie = have && hi == top_hi;
        unsigned long long who = __ballot(tie);
        if (__builtin_popcountll(who) > 1) {
            const unsigned top_lo = ~wave_min_u32(~(tie ? lo : 0u));
            who = __ballot(tie && lo == top_lo);
        }
        const int winner = __ffsll(who) - 1;
        last_hi = (unsigned)__builtin_amdgcn_readlane((int)hi, winner);
        last_lo = (unsigned)__builtin_amdgcn_readlane((int)lo, winner);
        taken |= lane == winner ? 1u << (best_c & 31) : 0u;
    }
    const unsigned long long key = ((unsigned long long)last_hi << 32) | last_lo;
    const unsigned long long up = from_top ? key : ~key;
    const unsigned long long b = (up >> 63) ? (up & 0x7FFFFFFFFFFFFFFFull) : ~up;
    return __longlong_as_double((long long)b);
}

// Rows of one request's first SEG_CHUNK segments as seen by this lane (= replica), with the segments' end
// positions (the same in every lane; entries past the request's last segment have end = n and no cell), and
// the reference of segment k in lane k.
struct RowSet {
    int32_t cell[SEG_CHUNK];
    int end[SEG_CHUNK];
    SegRef of_lane;
    int fresh;           // bit k: segment k's row slot starts over with this request (SEG_FRESH)
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


// ---------------------------------------------------------------------------------------------- hand-over
// Descriptor of one request, written by the queue wavefront's front end, read by the cache wavefront.
struct SegEnt {
    uint32_t rowoff;     // byte offset of the segment's row within the replay's rows
    int32_t end;         // blocks of the request up to and including this segment
};
struct SegDesc {
    SegEnt e[8];         // first eight segments, as the match reads them: where to load the row from and where the
                         // segment ends.  Past the last segment: the never-cached row, n.  Also the never-cached row for
                         // a segment whose row slot starts over with this request (SEG_FRESH: what the slot still holds
                         // belongs to a segment of the past), and for one whose slot started over with the previous
                         // request (this request's rows are loaded before that request's stores)
    int32_t L, n, s;     // input tokens, blocks, segments
    int32_t flags;       // DESC_MORE4 | DESC_DEEP | leading segments shared with the previous request << 8 |
                         // index of the first fresh segment among the first eight (8: none) << 16
    int64_t j0;          // index of the request's first segment reference (for requests of more than 8 segments)
    int32_t target;      // replica dictated by the session-affinity / random policy
    int32_t pad;
    uint32_t slot[8];    // where the rows of the first eight segments really are (past the last one: the spare row)
    uint32_t store[WAVE];   // per lane of the cache wavefront: the row its store after the decision goes to.  Lanes
                         // 0..31: the row of segment (lane mod 8), where this request's number is written into the
                         // chosen replica's cell.  Lanes 32..63, with at most 32 replicas: the row of the request's
                         // last segment if that one is fresh (replica lane - 32 of that row starts over), else, like
                         // every lane with nothing to store, the spare row
};
static_assert(sizeof(SegDesc) == 128 + 4 * WAVE, "descriptor layout");
constexpr int DESC_FRESH_TAIL = 4;   // the request's last segment is fresh and among the first eight (lanes 32..63 reset its row)
constexpr int DESC_FRESH_MORE = 8;   // further fresh segments among the first eight
constexpr int DESC_RING = 8;         // descriptors in flight (power of two)
constexpr int DESC_AHEAD = 3;        // the front end reads references this many requests ahead
constexpr int DESC_MORE4 = 1;        // more than four segments
constexpr int DESC_DEEP = 2;         // more than eight segments
constexpr int32_t NEVER_CACHED = INT32_MIN;      // cell value of the extra row: below any cursor

constexpr int LOOK_RING = 8;          // log records of look-ahead kept in LDS per replica, behind the two in registers
struct Handover {
    double sq[WAVE];                  // per replica: queue term of Eq. 3, w_queue * (a_pf * outstanding tokens)
                                      // (least-request policy: requests in flight)
    double rtt[WAVE];                 // proxy variants: estimated round trip time per replica
    double w[2];                      // online tuner: w_rtt, w_prefill in use
    unsigned long long choice;        // uncached tokens | (replica | cached blocks << 8) << 32
    unsigned long long unused[WAVE];  // where the lanes other than lane 0 write when the choice is announced
    int seen;                         // proxy variants: blocks the proxy believed cached on the chosen replica
    SegDesc ring[DESC_RING];
    // look-ahead of the eviction cursors (the cache's; the proxy's index's): per replica, log records fetched ahead
    // of the cursor, slot k of replica i at [k * WAVE + i]; the last slot is a spare that nothing reads
    unsigned long long look[2][(LOOK_RING + 1) * WAVE];
};

// Workgroup barrier that both wavefronts of a replay meet at; `after_lds`: this wavefront's LDS accesses have
// been performed before it arrives (what it wrote is there for the partner, what it read has been read).
// Global memory is not waited for: every global location is only ever touched by one of the two wavefronts.
__device__ __forceinline__ void meet(bool after_lds) {
    if (after_lds) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_barrier" ::: "memory");
}

// Section clock of the timed instantiation: cycles since the previous call are added to section k.  (Reading the
// clock waits for this wavefront's outstanding LDS and scalar-memory accesses, which the plain kernel does not.)
constexpr int SECTIONS = 12;
template <bool TIMED>
struct SectionClock {
    unsigned long long acc[SECTIONS] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    unsigned long long last = 0;
    __device__ __forceinline__ void start() {
        if (TIMED) last = __builtin_readcyclecounter();
    }
    __device__ __forceinline__ void tick(int k) {
        if (TIMED) {
            const unsigned long long now = __builtin_readcyclecounter();
            acc[k] += now - last;
            last = now;
        }
    }
    __device__ __forceinline__ void write(unsigned long long* out, int lane) {
        if (TIMED && out && lane == 0)
            for (int k = 0; k < SECTIONS; ++k) out[k] = acc[k];
    }
};


// Lowest-index minimum as wave_argmin, with the lane mask given.
__device__ __forceinline__ int argmin_lanes(double v, bool in) {
    const unsigned long long bits = (unsigned long long)__double_as_longlong(v + 0.0);
    const unsigned hi = (unsigned)(bits >> 32), lo = (unsigned)bits;
    const unsigned neg = (unsigned)((int)hi >> 31);
    const unsigned khi = in ? hi ^ (neg | 0x80000000u) : 0xffffffffu;
    const unsigned mhi = wave_min_u32(khi);
    const bool tie = khi == mhi;             // (lanes outside hold the all-ones key, which no score maps to)
    const unsigned long long ties = ballot(tie);
    if (__builtin_popcountll(ties) <= 1) return __builtin_ctzll(ties);      // one lane holds the smallest high word: done
    const unsigned klo = lo ^ neg;
    const unsigned mlo = wave_min_u32(tie ? klo : 0xffffffffu);
    return __builtin_ctzll(ballot(tie && klo == mlo));
}

// ---------------------------------------------------------------------------------------------- front end
// Front-end wavefront of a replay: walks the trace DESC_AHEAD requests ahead of the other two and leaves every
// request's descriptor in the ring.  Lane k < 8 holds segment reference k of the request in hand, lane 8 the last
// one (whose end position is the request's number of blocks).  It takes part in both meetings of every request
// (a workgroup barrier counts every wavefront) and is always early.
template <int MODE, bool TIMED>
__device__ __forceinline__ void front_wave(const SegArgs& a, int p, int lane, Handover* comm) {
    const int R = a.R;
    const int64_t N = a.N;
    const uint64_t seed = MODE == MODE_RANDOM ? a.seeds[p] : 0;
    const uint32_t seed_lo = (uint32_t)seed, seed_hi = (uint32_t)(seed >> 32);
    // the trace, 64 requests per lane-held batch (lane = request), two batches deep
    struct Batch {
        int L, s;        // input tokens, segment references
        int64_t j0;      // first segment reference
        uint32_t hash;   // session-affinity policy: hash of the first block
    };
    auto load_batch = [&](int64_t b0, Batch& b) {
        const int64_t x = b0 + lane;
        const bool in = x < N;
        const int64_t xx = in ? x : N - 1;
        b.L = in ? a.in_len[xx] : 0;
        const int64_t j0 = a.seg_off[xx], j1 = a.seg_off[xx + 1];
        b.j0 = j0;
        b.s = in ? (int)(j1 - j0) : 0;               // (requests past the end look empty)
        b.hash = MODE == MODE_AFFINITY ? a.first_hash[xx] : 0u;
    };
    Batch cur, nxt;
    int64_t b0 = 0;
    load_batch(0, cur);
    load_batch(WAVE, nxt);
    const uint32_t row_bytes = (uint32_t)R * 4u;
    const uint32_t never_off = (uint32_t)(a.nseg - 2) * row_bytes;      // the extra row that no request touches
    const uint32_t spare_off = (uint32_t)(a.nseg - 1) * row_bytes;      // the row that nothing reads
    int pend_id = 0, pend_end = 0, pend_s = 0, pend_L = 0, pend_target = 0;
    int64_t pend_j0 = 0;
    int prev_id = 0, prev_end = 0, prev_s = 0;
    bool prev_fresh = false;
    // request j's references are requested ... (j in this batch or the next)
    auto fe_issue = [&](int64_t j) {
        const int jj = (int)(j - b0);
        const bool here = jj < WAVE;
        const int jl = here ? jj : jj - WAVE;
        const int s = here ? __builtin_amdgcn_readlane(cur.s, jl) : __builtin_amdgcn_readlane(nxt.s, jl);
        pend_L = here ? __builtin_amdgcn_readlane(cur.L, jl) : __builtin_amdgcn_readlane(nxt.L, jl);
        pend_j0 = here ? readlane_i64(cur.j0, jl) : readlane_i64(nxt.j0, jl);
        pend_s = s;
        if (MODE == MODE_AFFINITY) {
            const uint32_t h = (uint32_t)(here ? __builtin_amdgcn_readlane((int)cur.hash, jl) : __builtin_amdgcn_readlane((int)nxt.hash, jl));
            pend_target = s > 0 ? spread(h, R) : 0;
        } else if (MODE == MODE_RANDOM) {
            pend_target = spread(philox4x32_10_first((uint32_t)j, (uint32_t)((uint64_t)j >> 32), seed_lo, seed_hi), R);
        }
        const int k = lane < 8 ? lane : s - 1;
        const bool on = lane < 8 ? lane < s : (lane == 8 && s > 0);
        SegRef ref{0, 0};
        if (on) ref = a.seg[pend_j0 + k];
        pend_id = ref.id;
        pend_end = ref.end;       // (with the SEG_FRESH mark)
    };
    // ... and one request later its descriptor is written
    auto fe_commit = [&](int64_t j) {
        const int s = pend_s;
        const bool fresh = (pend_end & SEG_FRESH) != 0;
        const int my_end = pend_end & SEG_END_MASK;
        const int n = s > 0 ? __builtin_amdgcn_readlane(my_end, 8) : 0;
        SegDesc* const d = &comm->ring[j & (DESC_RING - 1)];
        const bool real = lane < s;
        // leading segments shared with the previous request (same tree, same path so far): the cache wavefront
        // has requested this request's rows before the previous request's stores, and patches exactly these
        // (a fresh segment may sit in the slot that the previous request's segment at this place just gave up)
        const bool same = lane < 8 && lane < s && lane < prev_s && !fresh && pend_id == prev_id && my_end == prev_end;
        const unsigned differ = ~(unsigned)ballot(same) | 0x100u;
        const int common = __builtin_ctz(differ);
        // what the match loads: the segment's row, unless the row starts over now or did with the previous request
        const bool from_slot = real && !fresh && !(same && prev_fresh);
        const uint32_t slot_off = (uint32_t)pend_id * row_bytes;
        const int end = real ? my_end : n;
        if (lane < 8) {
            d->e[lane] = SegEnt{from_slot ? slot_off : never_off, end};
            d->slot[lane] = real ? slot_off : spare_off;
        }
        const unsigned fresh8 = (unsigned)ballot(lane < 8 && real && fresh);
        const int first_fresh = __builtin_ctz(fresh8 | 0x100u);
        // the store targets of the cache wavefront's lanes: lane 8 here holds the request's last segment
        const bool tail_fresh = s > 0 && s <= 8 && ((fresh8 >> (s - 1)) & 1u) != 0;
        const bool narrow = R <= 32;
        const uint32_t of_seg = (uint32_t)__builtin_amdgcn_ds_bpermute((lane & 7) << 2, (int)(real ? slot_off : spare_off));
        const uint32_t of_tail = (uint32_t)__builtin_amdgcn_readlane((int)slot_off, 8);
        d->store[lane] = lane < 32 || !narrow ? of_seg : (tail_fresh && lane - 32 < R ? of_tail : spare_off);
        const bool fresh_more = narrow ? (fresh8 & ~(tail_fresh ? 1u << (s - 1) : 0u)) != 0 : fresh8 != 0;
        if (lane == 0) {
            d->L = pend_L;
            d->n = n;
            d->s = s;
            d->flags = (s > 4 ? DESC_MORE4 : 0) | (s > 8 ? DESC_DEEP : 0) | (tail_fresh && narrow ? DESC_FRESH_TAIL : 0) |
                       (fresh_more ? DESC_FRESH_MORE : 0) | (common << 8) | (first_fresh << 16);
            d->j0 = pend_j0;
            d->target = pend_target;
        }
        prev_id = pend_id;
        prev_end = my_end;
        prev_s = s;
        prev_fresh = fresh;
    };
    fe_issue(0);
    fe_commit(0);
    fe_issue(1);
    fe_commit(1);
    fe_issue(2);
    meet(true);         // the first descriptors are there: the cache wavefront may start
    SectionClock<TIMED> clk;
    clk.start();
    for (int64_t r = 0; r < N; ++r) {
        // in the long stretch between B(r - 1) and A(r), where the cache wavefront reads the descriptor of r + 1:
        // the descriptor after that (first read by the cache wavefront after B(r))
        fe_commit(r + 2);
        clk.tick(0);                                                 // descriptors
        meet(true);                                                  // A(r)
        clk.tick(1);                                                 // waiting at A
        // in the short stretch where the cache wavefront decides: the references of the request after that
        fe_issue(r + 3);
        if (r + 1 - b0 == WAVE) {
            cur = nxt;
            b0 += WAVE;
            load_batch(b0 + WAVE, nxt);
        }
        clk.tick(3);                                                 // references
        meet(false);                                                 // B(r)
        clk.tick(2);                                                 // waiting at B
    }
    clk.write(a.sections ? a.sections + ((size_t)p * 3 + 2) * SECTIONS : nullptr, lane);
}

// ---------------------------------------------------------------------------------------------- queue side
// Queue wavefront of a replay.  Per request: retire what has completed by its arrival, publish the queue
// terms, meet (A); retire ahead to the next arrival and run the front end; meet (B); serve the request on
// the chosen replica.  Keeps and writes the latencies and the per-request outputs.
template <int MODE, bool ENGINE, bool PROXY, bool SLOTS, bool TIMED>
__device__ __forceinline__ void queue_wave(const SegArgs& a, int p, int lane, unsigned char* lds_raw, Handover* comm) {
    constexpr bool ONLINE = MODE == MODE_ONLINE;
    static_assert(!SLOTS || (!ENGINE && !PROXY), "one lane per slot exists for the linear replica model with fixed round trip times");
    const int R = a.R;
    const int64_t N = a.N;
    // the queue state: one lane per service slot where the model's shape allows it, else one lane per replica
    // with the slots in LDS
    // (the online tuner's instantiation does without the deferred fetch of deep lists: see SlotQueuesT)
    typename std::conditional<SLOTS, SlotQueuesT<MODE != MODE_ONLINE>, Queues>::type Q;
    if constexpr (SLOTS) {
        Q.init(lds_raw, R, a.B, lane);
    } else {
        Q.carve(lds_raw, R, a.B, lane);
        Q.init(lane);
    }
    // Online tuner (Sec. 2.3, Sec. 4), run here because this wavefront has the TTFTs: after every hop the p95
    // TTFT of the last `window` requests is the fitness of the weights in use; they replace the parent iff they
    // beat it; the step size follows the 1/5 rule; the next offspring is a log-space mutation of the parent.
    // The state is the same in every lane.
    double* const ring = reinterpret_cast<double*>(lds_raw + (SLOTS ? SlotQueues::bytes() : Queues::bytes(R, a.B)));
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
    }
    auto tuner_results = [&]() {
        if (ONLINE && lane == 0) {
            if (a.theta_final)
                for (int k = 0; k < 3; ++k)
                    a.theta_final[3 * (size_t)p + k] = clip(tuner_exp(ln_par[k]), a.tuner[k], a.tuner[3 + k]);
            if (a.sigma_final) a.sigma_final[p] = sigma;
            if (a.accepted) a.accepted[p] = accepted;
        }
    };
    if (N == 0) {           // (an empty trace still reports the tuner's initial state)
        tuner_results();
        return;
    }
    double w_queue = a.params[3 * (size_t)p + 2];      // (the online tuner replaces it at every step)
    const double sc = a.scale[p];
    double my_rtt = lane < R ? (PROXY ? a.rtt_true[lane] : a.rtt[lane]) : 0.0;
    // imperfect proxy knowledge (Sec. 2.2, Sec. 4 RTT figure): time is cut into probe epochs, the epoch of t being
    // the largest e with e * probe_ms <= t (capped at the last one given); a request experiences the true round
    // trip time of its epoch, the cost model scores with the proxy's moving average, handed to the cache wavefront
    // with the queue terms
    int epoch = 0;
    double next_probe = PROXY ? (double)a.probe_ms : 0.0;
    if (PROXY) comm->rtt[lane] = lane < R ? a.rtt_est[lane] : 0.0;
    // engine model: this lane's replica has its own rates and KV budget
    const double my_a_pf = ENGINE && lane < R ? a.eng_a_pf[lane] : 0.0;
    const double my_a_dec = ENGINE && lane < R ? a.eng_a_dec[lane] : 0.0;
    const double my_budget = ENGINE && lane < R ? a.eng_budget[lane] : 0.0;
    Rec* const rec = a.rec + (size_t)p * N;

    // ---- the trace, 64 requests per lane-held batch (lane = request), two batches deep so that a batch's loads
    // have a whole batch of time to arrive
    struct Batch {
        double t;        // arrival time, scaled
        int L, O;        // input tokens, output tokens
    };
    auto load_batch = [&](int64_t b0, Batch& b) {
        const int64_t x = b0 + lane;
        const int64_t xx = x < N ? x : N - 1;
        b.t = (double)a.ts[xx] * sc;                 // time scale: gaps scale linearly
        b.L = a.in_len[xx];
        b.O = a.out_len[xx];
    };
    Batch cur, nxt;
    load_batch(0, cur);
    load_batch(WAVE, nxt);
    meet(false);        // (the front end's first descriptors are there: the cache wavefront may start)

    double o_ttft = 0.0, o_e2e = 0.0;
    int o_route = 0, o_hit = 0, o_believed = 0;
    double own_done = INFINITY;               // (one lane per slot) when the previous request's completion reaches the proxy
    SectionClock<TIMED> clk;
    clk.start();
    // (a loop over the batches around a loop over a batch's requests: inside the inner one the batches do not change,
    // so nothing there has to wait for the loads of the batch after next, or, with them, for the stores of the
    // service step)
    for (int64_t b0 = 0; b0 < N; b0 += WAVE) {
        const int in_batch = N - b0 < WAVE ? (int)(N - b0) : WAVE;
        for (int i = 0; i < in_batch; ++i) {
            const int64_t r = b0 + i;
            const double t = readlane_f64(cur.t, i);
            const int L = __builtin_amdgcn_readlane(cur.L, i);
            const int O = __builtin_amdgcn_readlane(cur.O, i);
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
                    comm->rtt[lane] = a.rtt_est[at];
                }
            }
            // (one lane per slot: everything that completes by t was retired ahead, while the cache wavefront decided the
            // previous request -- except that request itself, whose completion time is known since it was served)
            if constexpr (SLOTS) {
                if (own_done <= t) Q.retire(t, rec, lane);
            } else {
                Q.retire(t, rec);
            }
            clk.tick(10);                                                // (finer: readlanes and retiring)
            // the queue term of Eq. 3, products rounded one by one (the least-request policy asks for the requests in
            // flight instead; the dictated policies ignore it)
            if (MODE == MODE_LEAST_REQUEST) comm->sq[lane] = Q.my_cnt;
            else if (MODE == MODE_COST_MODEL || MODE == MODE_ONLINE) {
                const double qd = a.a_pf * Q.my_q;
                comm->sq[lane] = w_queue * qd;
            }
            clk.tick(0);                                                 // retire, publish
            // The completions up to the next request's time do not depend on where this request goes (only this
            // request's own completion does, which is left for the retire above, next time round): they are retired
            // ahead, after the meeting, where this wavefront would otherwise wait while the cache wavefront decides.
            // The service step still has to see the slots that were idle at this request's time, so their set is
            // kept.
            unsigned long long idle_now = 0;
            SlotIdle idle_then{0, 0, 0, 0};
            if constexpr (SLOTS) {
                idle_then = Q.idle_slots();
            } else {
                idle_now = Q.idle;
            }
            clk.tick(2);                                                 // retire ahead
            clk.tick(3);                                                 // (nothing: what reading the clock costs)
            meet(true);                                                  // A(r)
            clk.tick(1);                                                 // waiting at A
            {
                const double t_ahead = i + 1 < WAVE ? readlane_f64(cur.t, i + 1) : readlane_f64(nxt.t, 0);
                if constexpr (SLOTS) {
                    if (r + 1 < N) Q.retire(t_ahead, rec, lane);
                } else {
                    if (r + 1 < N) Q.retire(t_ahead, rec);
                }
            }
            meet(false);                                                 // B(r)
            clk.tick(4);                                                 // waiting at B
            const unsigned long long w = comm->choice;
            const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(w >> 32));
            const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)w);
            const int best = (int)(hi & 63u);
            clk.tick(8);                                                 // (finer: the choice read)
            double ttft, e2e;
            if constexpr (SLOTS)
                Q.serve(r, best, t, readlane_f64(my_rtt, best), (int)lo, L, O, a.a_pf, a.a_dec, rec, lane, idle_then, &ttft, &e2e, &own_done);
            else if constexpr (ENGINE)
                Q.template serve_engine<PROXY>(r, best, t, my_rtt, (int64_t)(int)lo, L, O, my_a_pf, my_a_dec, my_budget, a.eng_slowdown,
                               rec, lane, &ttft, &e2e);
            else
                Q.template serve<PROXY>(r, best, t, my_rtt, (int64_t)(int)lo, L, O, a.a_pf, a.a_dec, rec, lane, idle_now,
                                        &ttft, &e2e);
            clk.tick(9);                                                 // (finer: service)
            o_ttft = lane == i ? ttft : o_ttft;
            o_e2e = lane == i ? e2e : o_e2e;
            o_route = lane == i ? best : o_route;
            o_hit = lane == i ? (int)(hi >> 8) : o_hit;
            if (PROXY && a.believed) o_believed = lane == i ? __builtin_amdgcn_readfirstlane(comm->seen) : o_believed;
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
                    w_queue = th[2];                                     // in use from the next request on
                    if (lane == 0) {
                        comm->w[0] = th[0];
                        comm->w[1] = th[1];
                        if (a.fitness_step) a.fitness_step[(size_t)p * a.steps + step] = f;
                        if (a.theta_step)
                            for (int k = 0; k < 3; ++k) a.theta_step[((size_t)p * a.steps + step) * 3 + k] = th[k];
                    }
                    ++step;
                    wave_sync();
                }
            }
            clk.tick(5);                                                 // serve, outputs, tuner
        }
        // the batch is done: its outputs go out, the next batch moves up and the one after it is requested
        if (lane < in_batch) {
            const size_t o = (size_t)p * N + b0 + lane;
            if (a.ttft) a.ttft[o] = o_ttft;
            if (a.e2e) a.e2e[o] = o_e2e;
            if (a.route) a.route[o] = (uint8_t)o_route;
            if (a.hit) a.hit[o] = (uint16_t)o_hit;
            if (PROXY && a.believed) a.believed[o] = (uint16_t)o_believed;
        }
        cur = nxt;
        load_batch(b0 + 2 * WAVE, nxt);
        clk.tick(6);                                                   // batch turnover
    }
    clk.write(a.sections ? a.sections + ((size_t)p * 3 + 1) * SECTIONS : nullptr, lane);
    tuner_results();
}

// ---------------------------------------------------------------------------------------------- cache side
// Eviction cursor of one LRU over a replica's log of routed requests, held by lane = replica.
//   cursor: blocks last touched by a request before cur_r, or by cur_r at positions >= cur_k, are evicted;
//   cur_own is where cur_r's owned suffix starts.
//   fill_r: the record after the last one held here, or -1 when that one is the youngest of the log.
//   pend_*: a record being fetched (its load is only waited for one iteration later); changes made to it
//   meanwhile are kept in pend_own / pend_next and override the loaded fields.
//   Records that have arrived wait in a ring in LDS until the cursor reaches them: the log is
//   read as far ahead of the cursor as the ring is long, so that a request which evicts several records' blocks at
//   once rarely has to wait for a record to come from memory.
// The same machinery serves the proxy's own index of the replica, an LRU of another capacity over the same log.
struct EvictCursor {
    int cur_r = -1, cur_k = 0, cur_own = 0;
    int fill_r = -1;
    int pend_r = -1, pend_own = -1, pend_next = -1;
    unsigned long long pend_raw = 0;
    // The look-ahead: a ring of records in LDS (slot k of this lane at ring[k * WAVE], packed r | own << 32 | n << 48),
    // ring_cnt of them from slot ring_head on, the youngest being request ring_hi.
    unsigned long long* ring = nullptr;
    int ring_head = 0, ring_cnt = 0, ring_hi = -1;
    int live = 0;             // blocks this LRU holds
    int n_spot = 0, n_adv = 0, n_dead = 0;       // statistics (only the timed instantiation reads them): records fetched
                                                 // on the spot, cursor advances, records dropped because they own nothing

    // In the lanes with `who` set, the record requested by the previous issue_fill becomes usable: dropped if it owns
    // nothing, else it joins the ring.  Straight-line code: lanes with nothing pending go through it unchanged
    // (every lane stores to LDS: those with nothing for the ring into its spare slot).
    __device__ __forceinline__ void take_pending(unsigned long long raw, bool who = true) {
        const bool have = who && pend_r >= 0;
        const unsigned hi = (unsigned)(raw >> 32);
        const int n = (int)(hi >> 16);
        const int own_mem = (int)(hi & 0xFFFFu);
        const int own = pend_own > own_mem ? pend_own : own_mem;
        const int next = pend_next >= 0 ? pend_next : (int)(unsigned)raw;
        const bool alive = have && own < n;
        const int slot = alive ? (ring_head + ring_cnt) & (LOOK_RING - 1) : LOOK_RING;
        ring[slot * WAVE] = (unsigned long long)(unsigned)pend_r | ((unsigned long long)((hi & 0xFFFF0000u) | (unsigned)own) << 32);
        ring_cnt += alive ? 1 : 0;
        ring_hi = alive ? pend_r : ring_hi;
        n_dead += have && !alive ? 1 : 0;
        fill_r = have ? next : fill_r;
        pend_r = have ? -1 : pend_r;
    }
    // Request the next record of the log where the ring has room for it.  Every lane loads (those with nothing to
    // fetch read the spare record behind the log, `spare`, and ignore it), so that the load is a plain instruction
    // of the request loop and not a branch around one.  Called right after take_pending: nothing is pending.
    __device__ __forceinline__ void issue_fill(const unsigned long long* log64, int spare) {
        const bool want = fill_r >= 0 && ring_cnt < LOOK_RING;
        pend_r = want ? fill_r : -1;
        pend_own = -1;
        pend_next = -1;
        pend_raw = ld(&log64[want ? fill_r : spare]);
    }
    // whether request `owner` may be one of the records in the ring (then disowned_anywhere is the call to make)
    __device__ __forceinline__ bool maybe_in_ring(int owner) const { return ring_cnt > 0 && owner <= ring_hi; }
    // request `owner`'s owned suffix now starts at `end` (owner = -2: nobody's); the owner is not in the ring
    __device__ __forceinline__ void disowned(int owner, int end) {
        cur_own = owner == cur_r ? end : cur_own;
        pend_own = owner == pend_r ? end : pend_own;
    }
    // the same where the owner may be a record in the ring (only called by the lanes it concerns)
    __device__ __forceinline__ void disowned_anywhere(int owner, int end) {
        disowned(owner, end);
        if (maybe_in_ring(owner)) {
#pragma nounroll
            for (int k = 0; k < LOOK_RING; ++k) {
                const unsigned long long e = ring[k * WAVE];
                if ((int)(unsigned)e == owner)
                    ring[k * WAVE] = (e & ~(0xFFFFull << 32)) | ((unsigned long long)(unsigned)end << 32);
            }
        }
    }
    // request r (n blocks) has become the youngest record of the log of the replica whose lane has is_best set;
    // tail_r is the youngest before it
    // (The replica's first record is not made the cursor's at once: it is the next one to fetch, like any record
    // appended after the look-ahead has caught up with the log, and the cursor, which starts before every request,
    // moves to it when something has to be evicted.)
    __device__ __forceinline__ void appended(bool is_best, int r, int n, int tail_r) {
        const bool to_pend = is_best && pend_r >= 0 && pend_r == tail_r;
        const bool to_fill = is_best && !to_pend && pend_r < 0 && fill_r < 0;
        pend_next = to_pend ? r : pend_next;
        fill_r = to_fill ? r : fill_r;
    }
    // takes up to E blocks from the owned suffix of the cursor's record
    __device__ __forceinline__ void take_from_cursor(int& E) {
        int avail = cur_k - cur_own;
        avail = avail > 0 ? avail : 0;
        const int take = avail < E ? avail : E;
        cur_k -= take;
        E -= take;
    }
    // The cursor moves on to further records until E blocks have been given up (all lanes together, those with
    // nothing to evict unchanged): records come from the ring, and from memory on the spot when the ring has run
    // out.  Works on a copy of the state, written back at the end: the request loop's common path, which does not
    // come here, then carries no register copies for this loop's sake.
    __device__ __forceinline__ void advance(int E_in, const unsigned long long* log64, int spare) {
        EvictCursor w = *this;
        int E = E_in;
        w.advance_loop(E, log64, spare);
        *this = w;
    }
    __device__ __forceinline__ void advance_loop(int& E, const unsigned long long* log64, int spare) {
        do {
            const bool empty = E > 0 && ring_cnt == 0;
            if (ballot(empty) != 0) {
                // fetch a record on the spot (the one being fetched, if any, is waited for instead)
                const bool fetch = empty && pend_r < 0 && fill_r >= 0;
                const bool stuck = empty && pend_r < 0 && fill_r < 0;      // cannot happen; bounds the loop
                live += stuck ? E : 0;
                E = stuck ? 0 : E;
                const unsigned long long got = ld(&log64[fetch ? fill_r : spare]);
                pend_r = fetch ? fill_r : pend_r;
                pend_own = fetch ? -1 : pend_own;
                pend_next = fetch ? -1 : pend_next;
                n_spot += fetch ? 1 : 0;
                take_pending(fetch ? got : pend_raw, empty && !stuck);
                continue;
            }
            const bool go = E > 0;
            const unsigned long long e = ring[(ring_head & (LOOK_RING - 1)) * WAVE];
            const unsigned hi = (unsigned)(e >> 32);
            n_adv += go ? 1 : 0;
            cur_r = go ? (int)(unsigned)e : cur_r;
            cur_k = go ? (int)(hi >> 16) : cur_k;
            cur_own = go ? (int)(hi & 0xFFFFu) : cur_own;
            ring_head += go ? 1 : 0;
            ring_cnt -= go ? 1 : 0;
            take_from_cursor(E);         // (lanes with E = 0 take nothing)
        } while (ballot(E > 0) != 0);
    }
    // `added` blocks have joined the LRU of the lane with `active` set; the cursor moves forward until the LRU
    // fits `cap` blocks again.  The cursor's own record is straight-line code; steps to further records loop (all
    // lanes together, those with nothing to evict unchanged), taking records from the ring, and from memory on the
    // spot when the ring has run out.
    __device__ __forceinline__ void evict(bool active, int added, int cap, const unsigned long long* log64, int spare) {
        live += active ? added : 0;
        int E = active ? live - cap : 0;
        E = E > 0 ? E : 0;
        live -= E;
        take_from_cursor(E);
        if (ballot(E > 0) != 0) advance(E, log64, spare);
    }
};

// Row cells of one request's first eight segments as seen by this lane (= replica), with the request's scalars
// (the same in every lane) and the row of segment (lane mod 8), whose cell that lane stores.
struct RowsOf {
    int32_t cell[8];
    int32_t end[8];
    int L, n, s, flags;
    uint32_t my_off;
};

// Cache wavefront of a replay.  Per request: meet (A); match the rows requested one request earlier, request the
// next request's rows, score, take the minimum, announce the choice; meet (B); update ownership, rows, log and
// eviction cursor on the chosen replica.
template <int MODE, bool ENGINE, bool PROXY, bool TIMED>
__device__ __forceinline__ void cache_wave(const SegArgs& a, int p, int lane, Handover* comm) {
    constexpr bool ONLINE = MODE == MODE_ONLINE;
    constexpr bool SCORED = MODE == MODE_COST_MODEL || MODE == MODE_ONLINE;
    constexpr bool DICTATED = MODE == MODE_AFFINITY || MODE == MODE_RANDOM;
    const int R = a.R;
    const int64_t N = a.N;
    const bool bounded = a.C > 0;
    // (kept in a vector register: under scalar-register pressure the compiler would otherwise re-read it from the
    // kernel arguments inside the request loop, a scalar-memory wait on the chain)
    int cap = (int)a.C;
    asm volatile("" : "+v"(cap));
    const bool in = lane < R;
    // (with the online tuner the weights come with the queue terms instead)
    const double w_rtt = a.params[3 * (size_t)p + 0];
    const double w_prefill = a.params[3 * (size_t)p + 1];
    const double my_rtt = !PROXY && in ? a.rtt[lane] : 0.0;     // (proxy variants: comes with the queue terms)
    const double rtt_term = w_rtt * my_rtt;                      // first product of Eq. 3, the same for every request
    // Proxy variants (Sec. 7: the proxy does not see replica-side eviction): the proxy keeps an index of its own
    // of what it dispatched to each replica, an LRU like the replica's cache but at least as large (or unbounded).
    // It sees the same touches, so it is the same rows read against a second eviction cursor (c2), which lags
    // the replica's; the match yields both prefixes, Eq. 3 scores with the index's.  Ownership is kept for
    // what the index holds, a superset of what is cached, which the replica's eviction walk does not mind:
    // records behind its cursor are never looked at again.  While the index never forgets (or is not used) its
    // cursor stays at the replica's first record and "in the index" means "ever dispatched here".
    const bool own_index = PROXY && a.index_blocks >= 0;
    const int index_cap = PROXY && a.index_blocks > 0 ? (int)a.index_blocks : 0;
    EvictCursor c1, c2;                       // the cache's cursor, the index's cursor
    c1.ring = &comm->look[0][lane];
    c2.ring = &comm->look[1][lane];
    for (int k = 0; k <= LOOK_RING; ++k) {
        c1.ring[k * WAVE] = ~0ull;
        c2.ring[k * WAVE] = ~0ull;
    }
    int tail_r = -1;                          // youngest request routed to this replica

    char* const rows = reinterpret_cast<char*>(a.last + (size_t)p * a.nseg * R);
    // this lane's cell of a row; the rows of one replay span less than 4 GiB (checked by the host)
    const unsigned lane_off = (unsigned)(in ? lane : 0) * 4u;
    const unsigned row_bytes = (unsigned)R * 4u;
    auto cell_at = [&](uint32_t rowoff) -> int32_t* { return reinterpret_cast<int32_t*>(rows + (rowoff + lane_off)); };
    auto cell_of = [&](uint32_t rowoff, int replica) -> int32_t* {
        return reinterpret_cast<int32_t*>(rows + (rowoff + (unsigned)replica * 4u));
    };
    // Stores and loads that only some lanes have use for are issued by every lane all the same, the others aimed
    // at a spare location (a row and a log record that nothing reads): a plain instruction of the request loop is
    // cheaper than a branch around it, and the number of memory operations in flight stays the same on every path.
    const unsigned spare_row = (unsigned)(a.nseg - 1) * row_bytes;
    const int spare = (int)N;                                   // the log record behind the last request's
    LogRec* const log = a.log + (size_t)p * (N + 1);
    unsigned long long* const log64 = reinterpret_cast<unsigned long long*>(log);
    unsigned long long* const choice_slot = lane == 0 ? &comm->choice : &comm->unused[lane];
    // the lanes that reset the row of a fresh last segment (see the store after the decision), and the replica of each
    const bool reset_lane = R <= 32 && lane >= 32;
    const int reset_rep = lane - 32 < R ? lane - 32 : R - 1;

    // the row loads of one request, from its descriptor: the descriptor is read (LDS) well before the loads go out
    struct DescCopy {
        int4 h, e01, e23, e45, e67;
        uint32_t my_off;
    };
    auto read_desc = [&](const SegDesc* d) {
        DescCopy c;
        c.h = *reinterpret_cast<const int4*>(&d->L);
        c.e01 = reinterpret_cast<const int4*>(d->e)[0];
        c.e23 = reinterpret_cast<const int4*>(d->e)[1];
        c.e45 = reinterpret_cast<const int4*>(d->e)[2];
        c.e67 = reinterpret_cast<const int4*>(d->e)[3];
        c.my_off = d->store[lane];
        return c;
    };
    auto request_rows = [&](const DescCopy& c, RowsOf& w) {
        w.my_off = c.my_off;
        w.L = c.h.x;
        w.n = c.h.y;
        w.s = c.h.z;
        w.flags = c.h.w;
        w.cell[0] = ld(cell_at((uint32_t)c.e01.x));
        w.cell[1] = ld(cell_at((uint32_t)c.e01.z));
        w.cell[2] = ld(cell_at((uint32_t)c.e23.x));
        w.cell[3] = ld(cell_at((uint32_t)c.e23.z));
        w.end[0] = c.e01.y;
        w.end[1] = c.e01.w;
        w.end[2] = c.e23.y;
        w.end[3] = c.e23.w;
        if (c.h.w & DESC_MORE4) {
            w.cell[4] = ld(cell_at((uint32_t)c.e45.x));
            w.cell[5] = ld(cell_at((uint32_t)c.e45.z));
            w.cell[6] = ld(cell_at((uint32_t)c.e67.x));
            w.cell[7] = ld(cell_at((uint32_t)c.e67.z));
            w.end[4] = c.e45.y;
            w.end[5] = c.e45.w;
            w.end[6] = c.e67.y;
            w.end[7] = c.e67.w;
        }
    };

    // Request r: `mine` holds its rows, `other` receives those of request r + 1.
    SectionClock<TIMED> clk;
    int n_walks = 0;          // statistics: ownership walks
    auto step = [&](int64_t r, RowsOf& mine, RowsOf& other, auto feeds) {
        const SegDesc* const dr = &comm->ring[r & (DESC_RING - 1)];
        const int target = DICTATED ? dr->target : 0;
        const DescCopy next = read_desc(&comm->ring[(r + 1) & (DESC_RING - 1)]);
        const int L = mine.L, n = mine.n, s = mine.s;
        int32_t rv = (int32_t)r;            // the request's number, once in a vector register for the stores below
        asm volatile("" : "+v"(rv));

        // ---- prefix match: lane = replica.  A request that touches a segment touches all its ancestors,
        // so along the path the cells never increase: first the segments touched after the cursor's
        // request (cached), then those it touched last itself (cached below the cursor position), then
        // older ones (evicted).  The match is max(e_gt, min(cur_k, e_ge)) with e_gt, e_ge the ends of the
        // last segment whose cell is above, respectively not below, the cursor's request.  (Entries past the
        // request's last segment hold the never-cached cell: they change nothing.)
        int e_gt = 0, e_ge = 0;
        int32_t own_gt = -1;        // previous owner of the last segment counted in e_gt
        int e_gt2 = 0, e_ge2 = 0;   // proxy variants: the same against the index's cursor
        int32_t own_gt2 = -1;
        auto compare = [&](int k) {
            const bool gt = mine.cell[k] > c1.cur_r;
            const bool ge = mine.cell[k] >= c1.cur_r;
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
        };
        compare(0);
        compare(1);
        compare(2);
        compare(3);
        if (mine.flags & DESC_MORE4) {
            compare(4);
            compare(5);
            compare(6);
            compare(7);
        }
        const int below_cursor = c1.cur_k < e_ge ? c1.cur_k : e_ge;
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
        bool deep = false;          // the match went past the preloaded segments
        if (mine.flags & DESC_DEEP) {
            // more than eight segments (rare): the rest of the path is read from the trace, eight references at a
            // time, as long as some replica's prefix is still open
            const int64_t j0 = dr->j0;
            int pos = mine.end[7];
            bool open = my_m == pos;
            bool open_seen = PROXY && my_seen == pos;
            if (ballot((PROXY ? open_seen : open) && in) != 0) {
                deep = true;
                for (int c0 = 8; c0 < s; c0 += 8) {
                    int32_t cell[8];
                    int send[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        cell[k] = NEVER_CACHED;
                        send[k] = pos;
                        if (c0 + k < s) {
                            const SegRef sr = a.seg[j0 + c0 + k];
                            send[k] = sr.end & SEG_END_MASK;
                            // (a fresh segment's row still holds what a segment of the past left there)
                            if ((PROXY ? open_seen : open) && in && !(sr.end & SEG_FRESH))
                                cell[k] = ld(cell_at((uint32_t)sr.id * row_bytes));
                        }
                    }
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        if (c0 + k < s) {
                            const int cnt = cached_in(cell[k], pos, send[k], c1.cur_r, c1.cur_k);
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
                    if (ballot((PROXY ? open_seen : open) && in) == 0) break;
                }
            }
        }

        clk.tick(1);                                                 // match (and the wait for the rows)
        // ---- the rows of this request have arrived: the loads for the next request go out
        request_rows(next, other);

        // ---- score (Eq. 3: rtt and prefill terms here, the queue term from the queue wavefront) and lowest-index
        // minimum.  block_tokens * blocks fits: below 2^15 and 2^16.
        int hit_tok = __mul24(a.block_tokens, my_m);
        hit_tok = hit_tok > L ? L : hit_tok;
        const int my_u = L - hit_tok;
        int my_u_seen = my_u;       // uncached tokens as Eq. 3 sees them
        if (PROXY) {
            int seen_tok = __mul24(a.block_tokens, own_index ? my_seen : my_m);
            seen_tok = seen_tok > L ? L : seen_tok;
            my_u_seen = L - seen_tok;
        }
        clk.tick(2);                                                 // log records, next rows, uncached tokens
        meet(false);                                                 // A(r): the queue terms of r are there
        clk.tick(0);                                                 // waiting at A
        const double sq = SCORED || MODE == MODE_LEAST_REQUEST ? comm->sq[lane] : 0.0;
        double rtt_now = my_rtt, now_rtt = w_rtt, now_prefill = w_prefill;
        if (PROXY) rtt_now = comm->rtt[lane];
        if (ONLINE) {
            now_rtt = comm->w[0];
            now_prefill = comm->w[1];
        }
        // (while those words come from LDS, every fourth request: the log record requested four requests ago has
        // arrived and becomes usable, and the next one is requested.  A replica's look-ahead needs a record every
        // thirty requests or so, and holds eight; feeding it in every fourth request costs a quarter.  Only the
        // second copy of the step has the code at all, so the other requests do not even branch around it.)
        if (decltype(feeds)::value && (r & 2)) {
            c1.take_pending(c1.pend_raw);
            if (PROXY && index_cap > 0) c2.take_pending(c2.pend_raw);
            c1.issue_fill(log64, spare);
            if (PROXY && index_cap > 0) c2.issue_fill(log64, spare);
        }
        double my_score;
        if (SCORED) {
            const double pf = a.a_pf * (double)my_u_seen;
            const double s_rtt = ONLINE || PROXY ? now_rtt * rtt_now : rtt_term;
            const double s_pf = now_prefill * pf;
            const double rtt_and_prefill = s_rtt + s_pf;
            my_score = rtt_and_prefill + sq;
        } else if (MODE == MODE_LEAST_REQUEST) {
            my_score = sq;                      // requests in flight
        } else {
            my_score = lane == target ? 0.0 : 1.0;      // the replica is dictated
        }
        const int best = argmin_lanes(my_score, in);
        const bool is_best = lane == best;
        const int m_best = __builtin_amdgcn_readlane(my_m, best);
        const int seen_best = PROXY ? __builtin_amdgcn_readlane(my_seen, best) : m_best;
        const unsigned u_best = (unsigned)__builtin_amdgcn_readlane(my_u, best);
        // (every lane writes: lane 0 the word that is read, the others a word of their own that is not)
        *choice_slot = ((unsigned long long)((unsigned)best | ((unsigned)m_best << 8)) << 32) | u_best;
        if (PROXY && lane == 0) comm->seen = own_index ? seen_best : m_best;
        clk.tick(3);                                                 // score, minimum, announcement
        // (the announcement is on its way through LDS; the second meeting comes after the ownership update below,
        // which does not depend on the queue side and gives it the time to arrive)

        // ---- ownership: the segments this request takes over on the chosen replica stop belonging to
        // their previous requests.  Along the path the previous owners form runs; each run moves its
        // owner's `own` to the end of the run.  Only cached segments matter (evicted ones belong to
        // requests the cursor has passed, or to the cursor request beyond its position).  One previous owner
        // (the usual case) is straight-line code: the chosen replica's lane names it, the others name nobody.
        const bool cached_some = seen_best > 0;
        // (a previous owner whose record waits in a cursor's look-ahead ring goes the long way too: rare, the ring
        // holds the oldest records of the replica and previous owners are mostly young)
        const bool plain_owner = one_owner && !c1.maybe_in_ring(mine.cell[0]) && !(PROXY && c2.maybe_in_ring(mine.cell[0]));
        const bool simple = cached_some && !deep && ((ballot(plain_owner) >> best) & 1ull) != 0;
        const int dis_owner = is_best && simple ? mine.cell[0] : -2;
        if (cached_some && !simple) {
            // several previous owners, or a prefix longer than the preloaded rows: walk it
            ++n_walks;
            auto disown = [&](int owner, int end) {       // lane `best`: owner's owned suffix now starts at end
                st(&log[owner].own, (uint16_t)end);
                c1.disowned_anywhere(owner, end);
                if (PROXY) c2.disowned_anywhere(owner, end);
            };
            const int64_t j0 = dr->j0;
            const int cb_r = __builtin_amdgcn_readlane(PROXY ? c2.cur_r : c1.cur_r, best);
            const int cb_k = __builtin_amdgcn_readlane(PROXY ? c2.cur_k : c1.cur_k, best);
            int run_owner = -1, run_end = 0, vpos = 0;
            for (int j = 0; j < s; ++j) {
                SegRef sr = a.seg[j0 + j];
                const int32_t rl = sr.end & SEG_FRESH ? NEVER_CACHED : ld(cell_of((uint32_t)sr.id * row_bytes, best));
                sr.end &= SEG_END_MASK;
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
        c1.disowned(dis_owner, k_end);
        if (PROXY) c2.disowned(dis_owner, k_end);
        st(&log[dis_owner >= 0 ? dis_owner : spare].own, (uint16_t)k_end);

        clk.tick(5);                                                 // ownership
        meet(true);                                                  // B(r): the choice is there (the stores below follow it:
                                                                     // the queue wavefront need not wait for them)
        clk.tick(4);                                                 // waiting at B
        // ---- cache update: every segment of the request is now last touched by r on the chosen replica
        // (lane k, and k + 8, ..., store the cell of segment k)
        // A segment that this request is the first to reference has taken over a row slot from a segment of the
        // past (the loader hands slots on): the row starts over, every replica's cell, never cached except on the
        // chosen one.  Fresh segments are the last ones of the path; mostly there is one, or none.  With at most 32
        // replicas the upper lanes do that in the same store: lane 32 + i writes replica i's cell of the row that the
        // front end names (the last segment's if it is fresh).  Further fresh segments, and any with more replicas,
        // take a loop of their own.
        {
            const int rep = reset_lane ? reset_rep : best;
            const int32_t val = reset_lane && rep != best ? NEVER_CACHED : rv;
            st(cell_of(mine.my_off, rep), val);
        }
        if (mine.flags & (DESC_FRESH_MORE | DESC_DEEP)) {      // (one test on the usual path for the two rare cases)
            if (mine.flags & DESC_FRESH_MORE) {
                const int first_fresh = (mine.flags >> 16) & 15;
                const int stop = (s < 8 ? s : 8) - ((mine.flags & DESC_FRESH_TAIL) ? 1 : 0);
                const int32_t fresh_cell = is_best ? (int32_t)r : NEVER_CACHED;
                for (int k = first_fresh; k < stop; ++k) {
                    const uint32_t off = ld(&dr->slot[k]);
                    st(cell_at(in ? off : spare_row), fresh_cell);
                }
            }
            if (mine.flags & DESC_DEEP) {
                const int64_t j0 = dr->j0;
                for (int j = 8; j < s; ++j) {
                    const SegRef sr = a.seg[j0 + j];
                    const uint32_t off = (uint32_t)sr.id * row_bytes;
                    if (sr.end & SEG_FRESH) st(cell_at(in ? off : spare_row), is_best ? (int32_t)r : NEVER_CACHED);
                    else if (is_best) st(cell_at(off), (int32_t)r);
                }
            }
        }

        // ---- log (every lane writes the same record; the chosen replica's lane links it) and eviction
        st(&log64[r], 0xFFFFFFFFull | ((unsigned long long)n << 48));      // next -1, own 0, n
        st(&log[is_best && tail_r >= 0 ? tail_r : spare].next, rv);
        clk.tick(6);                                                 // stores, log
        c1.appended(is_best, rv, n, tail_r);
        if (PROXY) c2.appended(is_best, (int)r, n, tail_r);
        tail_r = is_best ? rv : tail_r;
        c1.evict(is_best && bounded, n - m_best, cap, log64, spare);
        // the proxy's index evicts under its own capacity: its cursor walks the same log (whose memory is up to
        // date: ownership changes and links are stored as they happen)
        if (PROXY && index_cap > 0) c2.evict(is_best, n - seen_best, index_cap, log64, spare);

        // ---- the rows of request r + 1 were requested before this request's stores: the leading segments the two
        // paths share (none unless r + 1 continues the same tree) get the cells this request just wrote
        const int common = (other.flags >> 8) & 0xFF;
        if (common > 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) other.cell[k] = (k < common && is_best) ? rv : other.cell[k];
            if (other.flags & DESC_MORE4) {
#pragma unroll
                for (int k = 4; k < 8; ++k) other.cell[k] = (k < common && is_best) ? rv : other.cell[k];
            }
        }
        clk.tick(7);                                                 // eviction, patch, loop
    };

    RowsOf A, B;
    meet(false);                              // the first descriptors are there
    request_rows(read_desc(&comm->ring[0]), A);
    // (Where the loop is entered, as many memory operations are in flight behind the first request's row loads as a
    // pass through the loop leaves behind the next request's -- a log record load and five stores -- so that the
    // wait for the rows at the top of the loop is the same wait on both ways in, and not one for everything.)
    c1.issue_fill(log64, spare);
    for (int k = 0; k < 5; ++k) st(&log64[spare], 0ull);
    clk.start();
    for (int64_t r = 0; r < N; r += 2) {
        step(r, A, B, std::false_type{});
        if (r + 1 < N) step(r + 1, B, A, std::true_type{});
    }
    if (TIMED) {
        // statistics of the eviction walk, summed over the replicas
        clk.acc[8] = wave_sum_u32((unsigned)c1.n_spot);
        clk.acc[9] = wave_sum_u32((unsigned)c1.n_adv);
        clk.acc[10] = wave_sum_u32((unsigned)c1.n_dead);
        clk.acc[11] = (unsigned)__builtin_amdgcn_readfirstlane(n_walks);
    }
    clk.write(a.sections ? a.sections + (size_t)p * 3 * SECTIONS : nullptr, lane);
}

// (At most 128 vector registers: four wavefronts per SIMD.  The 1,024 replays of a population are 3,072 wavefronts,
// three per SIMD on 256 CUs; with registers for exactly three per SIMD a workgroup only fits where the wavefronts
// happen to be spread evenly, and part of the population waits for a second round.)
template <int MODE, bool ENGINE, bool PROXY, bool SLOTS = false, bool TIMED = false>
__global__ void __launch_bounds__(SEG3_THREADS, 4) replay_segments_kernel(SegArgs a) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ __align__(16) Handover comm;
    const int lane = threadIdx.x & (WAVE - 1);
    const int p = blockIdx.x;
    if (threadIdx.x == 0) {
        comm.w[0] = a.params[3 * (size_t)p + 0];
        comm.w[1] = a.params[3 * (size_t)p + 1];
    }
    __syncthreads();
    if (threadIdx.x >= 2 * WAVE) {
        if (a.N > 0) {
            __builtin_amdgcn_s_setprio(1);
            front_wave<MODE, TIMED>(a, p, lane, &comm);
        }
    } else if (threadIdx.x >= WAVE) {
        __builtin_amdgcn_s_setprio(3);
        queue_wave<MODE, ENGINE, PROXY, SLOTS, TIMED>(a, p, lane, lds_raw, &comm);
    } else if (a.N > 0) {
        __builtin_amdgcn_s_setprio(3);      // the two wavefronts on the chain go first at issue
        cache_wave<MODE, ENGINE, PROXY, TIMED>(a, p, lane, &comm);
    }
}

}  // namespace gorgo

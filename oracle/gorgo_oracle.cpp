// TEST INFRASTRUCTURE ONLY -- sequential CPU oracle for batched routing-fitness evaluation.
//
// This file is the reference that the GPU library is checked against.  It is deliberately plain and
// slow: one replay at a time, std::unordered_map / std::map / std::multiset, fp64 with every product and
// sum rounded separately (build with -ffp-contract=off), no blocking, no fusion, no shortcuts.  It shares no
// code with the GPU path and must never be called, linked or loaded by it.  Only tests, the smoke check and
// the benchmark's CPU-baseline leg may use it.
//
// What one replay computes (paper notation: replica i, request r, cached prefixes c_i, input x_r):
//   * TTFT decomposition, Eq. 1:   TTFT = T_network(i) + T_queue(i) + T_prefill(x_r \ c_i)
//   * proxy-observable load, Eq. 2: the queue term's input is the total number of tokens of requests that
//     have no completion event at the proxy yet
//   * weighted score, Eq. 3, routed to the replica of minimum score (Sec. 2.3 "GORGO Proxy Design")
//   * time_scale replay: timestamps scaled linearly (Sec. 3 "Dataset", Sec. 4 "Tuning and evaluation windows")
//   * objective: p95 TTFT (Sec. 2.3, Sec. 4); p95 E2E is reported beside it (Table 2)
// Readings taken where the paper is silent (functional forms of the three terms, the replica service model,
// LRU order, percentile definition) are stated next to the step that uses them.
//
// The online tuner (Sec. 2.3 "GORGO Proxy Design", Sec. 4 "Tuning and evaluation windows") runs inside one
// replay: after every `hop` requests the p95 TTFT of the last `window` requests is the fitness of the weights
// in use; a (1+1) evolution strategy keeps them if they beat the parent, adapts its step size by the 1/5
// rule and proposes the next offspring by the log-space mutation.
//
// Pinned by tests (tests/test_oracle_*.py): three hand-worked traces, brute force over every route sequence
// at R=2 N=10 against an independent forced-route evaluator, weight special cases (all-zero, rtt-only,
// prefix-only, queue-only, power-of-two rescaling), post-hoc recomputation of the load signal, Lindley /
// Kiefer-Wolfowitz recurrences for the service model, a list-based LRU model, sorted-array percentile.
// The engine model of a replica (continuous batching with a KV-token budget, decode slow-down under occupancy,
// per-replica rates; struct Engine below) is pinned by two hand-worked traces, a millisecond-stepped simulation
// of the admission rule on integer inputs, the serial-server and simultaneous-arrival closed forms, its
// reduction to the linear model, the independence of replicas under random routing, and its invariants rebuilt
// from the outputs.
// Imperfect proxy knowledge (round trip times per probe epoch scored through their moving average, a cache index
// of its own capacity; struct Proxy below) is pinned by a hand-worked trace, closed forms of the moving average,
// probe epochs recovered from latencies at and around the epoch boundaries, reductions to the plain replay, the
// forced-route model extended with the same knowledge, and the one-sidedness of the index's error.
// Parity unpinned by the paper (fixed by the readings stated here only): the service-model constants,
// the functional form of the engine model, the smoothing constant and the index's forgetting rule, and the
// root-newest stamp order inside one request.

#include <cstdint>
#include <cstddef>
#include <cstring>
#include <cmath>
#include <algorithm>
#include <map>
#include <set>
#include <unordered_map>
#include <unordered_set>
#include <utility>
#include <vector>

namespace {

// Stamps order cache entries by recency.  A later request is newer than an earlier one; inside one request
// the first (root) block is the newest and the last (deepest) block the oldest, so that eviction removes
// leaves before roots, as radix prefix caches do (Sec. 6 "Prefix caches and reuse").
constexpr int64_t STAMP_STRIDE = 65536;

struct Replica {
    std::unordered_map<int64_t, int64_t> cache;   // block id -> stamp
    std::map<int64_t, int64_t> by_stamp;          // stamp -> block id (stamps are unique per replica)
    std::vector<double> free_at;                  // per service slot: time the slot becomes free
    std::multiset<std::pair<double, int64_t>> inflight;   // (completion time at the proxy, input tokens)
    int64_t q = 0;                                // tokens of requests without a completion event (Eq. 2)
    // engine model only: the requests served here that may still be running at a later admission, as (time the
    // last token is produced, KV tokens held), and the time the latest request was admitted
    std::vector<std::pair<double, int64_t>> served;
    double last_start = 0.0;
    // imperfect proxy knowledge only: the proxy's own index of this replica's cache (same rules, own capacity)
    std::unordered_map<int64_t, int64_t> index_cache;
    std::map<int64_t, int64_t> index_by_stamp;
};

// The engine model of a replica (Sec. 2.2: continuous batching admits a request into the running batch while
// the batch is below its maximum number of concurrent requests and the KV-cache budget allows; Sec. 5
// "Exploiting Continuous Batching": once many requests decode together the replica's memory saturates and
// inter-token latency grows; Sec. 7: replicas may differ in prefill rate, queueing behaviour and KV capacity).
// The paper gives no formulas for any of this; the stated model is:
//   * replica i prefills at a_pf[i] ms per uncached token and decodes at a_dec[i] ms per output token;
//   * a request holds in_len + out_len KV tokens from its admission until its last token is produced;
//   * requests are admitted in arrival order (first come first served, no overtaking); a request is admitted at
//     the first time s, not before its arrival and not before the admission of its predecessor, at which the
//     requests running at s (admitted earlier, last token produced after s) number fewer than B and either
//     there are none or their KV tokens plus the request's own fit into kv_tokens[i] (0 = no budget);
//   * its decode takes (a_dec[i] * out_len) * (1 + slowdown * n), n being the number of requests running at its
//     admission (the slow-down is fixed at admission and not revised when the batch changes later).
// With slowdown = 0, no budget and equal rates this is the linear B-slot model.
struct Engine {
    const double* a_pf;        // [R]
    const double* a_dec;       // [R]
    const int64_t* kv_tokens;  // [R] or null
    double slowdown;
};

// exp(x) from additions and multiplications only, so that every build of it gives the same bits (the weights
// the tuner proposes decide routes, and the C library's exp is not the same everywhere).  Stated algorithm:
// k = floor(x / ln 2 + 1/2); r = (x - k * LN2_HI) - k * LN2_LO with ln 2 split so that k * LN2_HI is exact;
// exp(r) = sum_{j=0}^{13} r^j / j! by Horner's rule from the highest term down; result = that times 2^k.
// Valid for |x| <= 700 (the tuner's arguments are logarithms of weights in [1e-100, 1e100]).
double tuner_exp(double x) {
    const double INV_LN2 = 1.44269504088896338700e+00;
    const double LN2_HI = 6.93147180369123816490e-01;     // ln 2 with its low 21 bits zero
    const double LN2_LO = 1.90821492927058770002e-10;     // ln 2 - LN2_HI
    const double k = std::floor(x * INV_LN2 + 0.5);
    const double r = (x - k * LN2_HI) - k * LN2_LO;
    static const double inv_fact[14] = {1.0, 1.0, 1.0 / 2.0, 1.0 / 6.0, 1.0 / 24.0, 1.0 / 120.0, 1.0 / 720.0,
                                        1.0 / 5040.0, 1.0 / 40320.0, 1.0 / 362880.0, 1.0 / 3628800.0,
                                        1.0 / 39916800.0, 1.0 / 479001600.0, 1.0 / 6227020800.0};
    double p = inv_fact[13];
    for (int j = 12; j >= 0; --j) p = p * r + inv_fact[j];
    const uint64_t bits = (uint64_t)((int64_t)k + 1023) << 52;      // 2^k
    double two_k;
    std::memcpy(&two_k, &bits, sizeof two_k);
    return p * two_k;
}

double clip(double x, double lo, double hi) { return std::min(std::max(x, lo), hi); }

// Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11),
// written from the paper's definition: per round, two 32x32 -> 64 bit products of the counter words 0 and 2
// with the constants M0 and M1; the new counter is (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1,
// lo(M0 c0)); the key words advance by the Weyl constants between rounds.
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    uint32_t c[4] = {ctr[0], ctr[1], ctr[2], ctr[3]};
    uint32_t k[2] = {key[0], key[1]};
    for (int round = 0; round < 10; ++round) {
        const uint64_t a = M0 * c[0], b = M1 * c[2];
        const uint32_t n[4] = {(uint32_t)(b >> 32) ^ c[1] ^ k[0], (uint32_t)b, (uint32_t)(a >> 32) ^ c[3] ^ k[1],
                               (uint32_t)a};
        for (int j = 0; j < 4; ++j) c[j] = n[j];
        k[0] += 0x9E3779B9u;
        k[1] += 0xBB67AE85u;
    }
    for (int j = 0; j < 4; ++j) out[j] = c[j];
}

// SplitMix64 output function (Steele, Lea, Flood, "Fast splittable pseudorandom number generators", OOPSLA'14,
// in the form of Vigna's splitmix64.c): next value of a generator whose state is x.
uint64_t splitmix64_next(uint64_t x) {
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// A 32-bit value spread over R replicas: floor(h * R / 2^32).
int spread(uint32_t h, int R) { return (int)(((uint64_t)h * (uint64_t)R) >> 32); }

// What the proxy knows imperfectly (Sec. 2.2: T_network is the exponentially weighted moving average of a ping's
// round trip time; Sec. 4, RTT figure: measured every 30 s on a separate probe; Sec. 7: the proxy does not observe
// replica-side eviction, so its cache index may overestimate what is cached).  The paper gives neither the
// smoothing constant nor the index's own forgetting rule; the stated model is:
//   * time is cut into epochs of probe_ms: the epoch of time t is the largest e with e * probe_ms <= t, capped
//     at epochs - 1; during epoch e the true round trip time of replica i is rtt_true[e][i] (both legs of a
//     request dispatched in epoch e take half of it);
//   * the proxy probes at the start of every epoch and smooths: est[0] = rtt_true[0], est[e] = alpha *
//     rtt_true[e] + (1 - alpha) * est[e-1]; the cost model scores with est of the request's epoch;
//   * index_blocks >= 0: the proxy keeps an index of its own of what it dispatched to replica i (a prefix trie of
//     dispatched requests), updated like the replica's cache (least recently used block evicted first) but with
//     its own capacity: index_blocks per replica, 0 = it never forgets; the cost model takes its uncached tokens
//     from the longest prefix in that index, the replica prefills what its own cache really misses.
//     index_blocks < 0: the proxy sees the replicas' caches as they are.
struct Proxy {
    int32_t epochs;            // >= 1
    int32_t probe_ms;          // >= 1
    const double* rtt_true;    // [epochs][R]
    double alpha;              // in (0, 1]
    int64_t index_blocks;      // < 0 = the proxy sees the replicas' caches as they are
};

// Admission time of a request of `kv` KV tokens that arrives at `a` on replica X (see Engine), and the number
// of requests running then.  Written as the definition: the candidates are the earliest allowed time and every
// later time at which a running request ends, tried in increasing order.
double engine_admit(const Replica& X, int B, int64_t budget, double a, int64_t kv, int64_t* running_out) {
    const double s0 = std::max(a, X.last_start);
    std::vector<double> cand{s0};
    for (const auto& x : X.served)
        if (x.first > s0) cand.push_back(x.first);
    std::sort(cand.begin(), cand.end());
    for (double s : cand) {
        int64_t n = 0, held = 0;
        for (const auto& x : X.served)
            if (x.first > s) {
                ++n;
                held += x.second;
            }
        if (n < B && (n == 0 || budget == 0 || held + kv <= budget)) {
            *running_out = n;
            return s;
        }
    }
    return -1.0;   // not reached: after the last end nothing is running
}

}  // namespace

extern "C" {

// Exposed so that tests can pin the tuner's exp against the C library's, and the two generators against their
// published answers.
double gorgo_oracle_tuner_exp(double x) { return tuner_exp(x); }
void gorgo_oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) { philox4x32_10(ctr, key, out); }
uint64_t gorgo_oracle_splitmix64_next(uint64_t x) { return splitmix64_next(x); }

// Tuner steps a replay of N requests takes: one when the first window is full, then one every hop.
int64_t gorgo_oracle_online_steps(int64_t N, int32_t window, int32_t hop) {
    if (window < 1 || hop < 1) return 0;      // no tuner
    return N >= window ? (N - window) / hop + 1 : 0;
}

// Nearest-rank percentile: the k-th smallest element with k = ceil(0.95 n) (1-indexed), no interpolation.
// Objective of the tuner is the p95 of TTFT (Sec. 2.3, Sec. 4).
double gorgo_oracle_p95(const double* x, int64_t n) {
    if (n <= 0) return 0.0;
    std::vector<double> s(x, x + n);
    std::sort(s.begin(), s.end());
    int64_t k = (95 * n + 99) / 100;
    return s[k - 1];
}

// One replay of the trace under one weight vector w = (w_rtt, w_prefill, w_queue) and one time scale.
// Outputs (all host, caller-owned, each may be null): route[N], hit_blocks[N], ttft_ms[N], e2e_ms[N],
// p95[2] = {p95 ttft, p95 e2e}; debug outputs score_dbg[N*R] (score of every replica as seen by request r),
// q_dbg[N*R] (load signal after retirement, before dispatch), size_dbg[N] (blocks cached on the chosen
// replica after the update).  Returns 0, or -1 for bad arguments, -5 if a request has more distinct blocks
// than a bounded cache can hold.
//
// Weights: w is what the first request is scored with.  With window > 0 the weights change inside the replay,
// after requests window, window + hop, window + 2 hop, ... (counting from 1), step h = 0, 1, ...:
//   * schedule != null: the weights become schedule[h] (nothing else happens);
//   * otherwise the online tuner runs (z = standard normal draws [steps][3], lo/hi = clip range per weight,
//     sigma0 = initial step size; tuner outputs, each may be null: theta_step[steps][3] = weights in use after
//     each step, fitness_step[steps] = window p95 TTFT seen at each step, tuner_final[6] = parent weights (3),
//     step size, steps taken, offspring accepted).
//
// Policy (Sec. 4 "Baseline policies"; the cost model is policy 0, and two of the paper's baselines are
// special cases of it: prefix-cache = weights (0, 1, 0), proxy-only least-load = weights (0, 0, 1)):
//   1 least-request: the replica with the fewest in-flight requests (requests without a completion event at
//     the proxy), lowest index on ties;
//   2 session affinity: the replica that a hash of the request's first block selects (the paper hashes the
//     first 256 tokens; traces here carry one id per 512-token block): spread(high 32 bits of
//     splitmix64_next(first id)); a request without blocks goes to replica 0;
//   3 random: replica spread(first word of Philox-4x32-10(counter = (r mod 2^32, r div 2^32, 0, 0), key =
//     (seed mod 2^32, seed div 2^32))).
//
// Replica model: with engine == null the linear B-slot model; otherwise the engine model (see Engine), in which
// the cost model of Eq. 3 keeps the single prefill rate a_pf: the router does not know that replicas differ
// (Sec. 7, first limitation).
static int replay_impl(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len,
                       const int64_t* blk_off, const int64_t* hash_ids, int32_t block_tokens,
                       int32_t R, int32_t B, int64_t C, double a_pf, double a_dec,
                       const double* rtt_ms, const double* w, double scale,
                       int32_t window, int32_t hop, const double* schedule, const double* z,
                       const double* lo, const double* hi, double sigma0, int32_t policy, uint64_t seed,
                       const Engine* engine, const Proxy* proxy, double* rtt_est_out, uint16_t* believed_hit,
                       uint8_t* route, uint16_t* hit_blocks, double* ttft_ms, double* e2e_ms, double* p95,
                       double* score_dbg, int64_t* q_dbg, int64_t* size_dbg,
                       double* theta_step, double* fitness_step, double* tuner_final) {
    if (N < 0 || R < 1 || R > 255 || B < 1 || C < 0 || block_tokens < 1) return -1;
    if (N > 0 && (!ts_ms || !in_len || !out_len || !blk_off)) return -1;
    if (window < 0 || (window > 0 && hop < 1)) return -1;
    if (policy < 0 || policy > 3 || (policy != 0 && window > 0)) return -1;
    if (window > 0 && !schedule && (!z || !lo || !hi)) return -1;
    double w_rtt = w[0], w_prefill = w[1], w_queue = w[2];

    // Tuner state (Sec. 2.3): the parent in log space, its fitness once it has one, the offspring in use (in log
    // space, after clipping), the step size.  The paper's rule is x' = clip(exp(ln x_t + sigma z), [lo, hi]);
    // here ln x_t is carried along instead of being taken again from the clipped x_t.
    double ln_par[3] = {0, 0, 0}, ln_cur[3] = {0, 0, 0}, ln_lo[3] = {0, 0, 0}, ln_hi[3] = {0, 0, 0};
    double f_par = 0.0, sigma = sigma0;
    bool have_parent = false;
    int64_t steps = 0, accepted = 0;
    // Rechenberg's 1/5 rule in its damped form sigma * exp((s - 1/5) / 2), s = 1 after a success, else 0
    const double c_up = std::exp(0.4), c_down = std::exp(-0.1);
    if (window > 0 && !schedule)
        for (int k = 0; k < 3; ++k) {
            ln_par[k] = ln_cur[k] = std::log(w[k]);
            ln_lo[k] = std::log(lo[k]);
            ln_hi[k] = std::log(hi[k]);
        }

    // the proxy's smoothed round trip times, epoch by epoch
    std::vector<double> rtt_est;
    if (proxy) {
        rtt_est.assign((size_t)proxy->epochs * R, 0.0);
        for (int i = 0; i < R; ++i) rtt_est[i] = proxy->rtt_true[i];
        for (int64_t e = 1; e < proxy->epochs; ++e)
            for (int i = 0; i < R; ++i) {
                const double fresh = proxy->alpha * proxy->rtt_true[e * R + i];
                const double kept = (1.0 - proxy->alpha) * rtt_est[(e - 1) * R + i];
                rtt_est[e * R + i] = fresh + kept;
            }
        if (rtt_est_out) std::copy(rtt_est.begin(), rtt_est.end(), rtt_est_out);
    }
    int64_t epoch = 0;
    const double* rtt_score = rtt_ms;     // what the cost model believes ...
    const double* rtt_real = rtt_ms;      // ... and what a request experiences

    std::vector<Replica> rep(R);
    for (auto& x : rep) x.free_at.assign(B, 0.0);
    std::vector<double> ttft(N), e2e(N), score(R);
    std::vector<int64_t> m(R), u(R), m_seen(R), u_seen(R);

    for (int64_t r = 0; r < N; ++r) {
        const int64_t* ids = hash_ids + blk_off[r];
        const int64_t n = blk_off[r + 1] - blk_off[r];
        if (n < 0 || n >= STAMP_STRIDE) return -1;
        const int64_t L = in_len[r];

        // time scale: gaps between requests are scaled linearly (larger scale = lighter load, Table 3)
        const double t = (double)ts_ms[r] * scale;
        if (proxy) {
            // (timestamps do not decrease, so the epoch only moves forward)
            while (epoch + 1 < proxy->epochs && (double)(epoch + 1) * (double)proxy->probe_ms <= t) ++epoch;
            rtt_score = rtt_est.data() + epoch * R;
            rtt_real = proxy->rtt_true + epoch * R;
        }

        // retire: a request stops counting toward the load signal once its completion event has reached
        // the proxy (Eq. 2 and the sentence before it).  An event at exactly t counts as completed.
        for (int i = 0; i < R; ++i) {
            auto& f = rep[i].inflight;
            while (!f.empty() && f.begin()->first <= t) {
                rep[i].q -= f.begin()->second;
                f.erase(f.begin());
            }
        }

        // prefix match: tokens of x_r already cached on replica i are those of the longest prefix of the
        // request's blocks that is wholly present in c_i (Eq. 1: prefill depends on x_r \ c_i only).
        for (int i = 0; i < R; ++i) {
            int64_t k = 0;
            while (k < n && rep[i].cache.count(ids[k])) ++k;
            m[i] = k;
            int64_t hit_tok = std::min<int64_t>(L, (int64_t)block_tokens * k);   // partial last block
            u[i] = L - hit_tok;
        }
        // with an index of its own the cost model sees the longest prefix in that index instead
        u_seen = u;
        m_seen = m;
        if (proxy && proxy->index_blocks >= 0)
            for (int i = 0; i < R; ++i) {
                int64_t k = 0;
                while (k < n && rep[i].index_cache.count(ids[k])) ++k;
                m_seen[i] = k;
                u_seen[i] = L - std::min<int64_t>(L, (int64_t)block_tokens * k);
            }

        // score (Eq. 3) with all three terms in milliseconds: network = RTT_i; prefill = a_pf * uncached
        // tokens; queue = a_pf * outstanding tokens (time to prefill what is outstanding).  Association
        // is fixed: (w_rtt*rtt + w_prefill*pf) + w_queue*qd.
        for (int i = 0; i < R; ++i) {
            double pf = a_pf * (double)u_seen[i];
            double qd = a_pf * (double)rep[i].q;
            double s_rtt = w_rtt * rtt_score[i];
            double s_pf = w_prefill * pf;
            double s_q = w_queue * qd;
            double s = s_rtt + s_pf;
            s = s + s_q;
            score[i] = s;
            if (score_dbg) score_dbg[r * R + i] = s;
            if (q_dbg) q_dbg[r * R + i] = rep[i].q;
        }
        // route to the minimum calculated cost (Sec. 2.3); ties go to the lowest replica index
        int best = 0;
        for (int i = 1; i < R; ++i)
            if (score[i] < score[best]) best = i;
        // baseline policies route by their own rule instead (Sec. 4)
        if (policy == 1) {
            best = 0;
            for (int i = 1; i < R; ++i)
                if (rep[i].inflight.size() < rep[best].inflight.size()) best = i;
        } else if (policy == 2) {
            best = n > 0 ? spread((uint32_t)(splitmix64_next((uint64_t)ids[0]) >> 32), R) : 0;
        } else if (policy == 3) {
            const uint32_t ctr[4] = {(uint32_t)r, (uint32_t)((uint64_t)r >> 32), 0u, 0u};
            const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
            uint32_t x[4];
            philox4x32_10(ctr, key, x);
            best = spread(x[0], R);
        }
        Replica& X = rep[best];

        // cache update on the chosen replica: every block of the request becomes (or stays) cached with a
        // fresh stamp; if a bounded cache would overflow, the entries with the smallest stamps that do not
        // belong to this request are evicted first (least recently used).
        auto touch = [&](std::unordered_map<int64_t, int64_t>& cache, std::map<int64_t, int64_t>& by_stamp,
                         int64_t capacity) -> int {
            std::unordered_set<int64_t> mine(ids, ids + n);
            if (capacity > 0 && (int64_t)mine.size() > capacity) return -5;
            int64_t n_new = 0;
            for (int64_t id : mine) if (!cache.count(id)) ++n_new;
            if (capacity > 0) {
                int64_t excess = (int64_t)cache.size() + n_new - capacity;
                auto it = by_stamp.begin();
                while (excess > 0 && it != by_stamp.end()) {
                    if (mine.count(it->second)) { ++it; continue; }
                    cache.erase(it->second);
                    it = by_stamp.erase(it);
                    --excess;
                }
                if (excess > 0) return -5;
            }
            std::unordered_set<int64_t> seen;
            for (int64_t k = 0; k < n; ++k) {
                if (!seen.insert(ids[k]).second) continue;      // stamp comes from the first occurrence
                int64_t stamp = r * STAMP_STRIDE + (STAMP_STRIDE - 1 - k);
                auto f = cache.find(ids[k]);
                if (f != cache.end()) { by_stamp.erase(f->second); f->second = stamp; }
                else cache.emplace(ids[k], stamp);
                by_stamp.emplace(stamp, ids[k]);
            }
            return 0;
        };
        if (int rc = touch(X.cache, X.by_stamp, C)) return rc;
        if (size_dbg) size_dbg[r] = (int64_t)X.cache.size();
        // the proxy's index records the same dispatch under its own capacity
        if (proxy && proxy->index_blocks >= 0)
            if (int rc = touch(X.index_cache, X.index_by_stamp, proxy->index_blocks)) return rc;

        // service on the chosen replica (the paper leaves the replica model open; the one stated here is
        // linear): B slots, each serving one request at a time, first come first served on the
        // earliest-free slot (lowest index on ties); prefill a_pf ms per uncached token, then decode a_dec
        // ms per output token.  The request reaches the replica half an RTT after t and its first token /
        // completion event come back half an RTT after they are produced.  This reproduces Eq. 1:
        // ttft = rtt + (start - arrival) + prefill(x_r \ c_i).
        if (engine) {
            const double half = 0.5 * rtt_real[best];
            const double a = t + half;
            const int64_t kv = L + (int64_t)out_len[r];
            int64_t running = 0;
            const double s = engine_admit(X, B, engine->kv_tokens ? engine->kv_tokens[best] : 0, a, kv, &running);
            const double pf = engine->a_pf[best] * (double)u[best];
            const double f = s + pf;
            const double dec_alone = engine->a_dec[best] * (double)out_len[r];
            const double factor = 1.0 + engine->slowdown * (double)running;
            const double dec = dec_alone * factor;
            const double e = f + dec;
            // (requests whose last token is out by s are running at no later admission time: forget them)
            X.served.erase(std::remove_if(X.served.begin(), X.served.end(),
                                          [s](const std::pair<double, int64_t>& x) { return x.first <= s; }),
                           X.served.end());
            X.served.emplace_back(e, kv);
            X.last_start = s;
            const double done = e + half;
            ttft[r] = (f + half) - t;
            e2e[r] = done - t;
            X.inflight.emplace(done, L);
            X.q += L;
        } else {
            double half = 0.5 * rtt_real[best];
            double a = t + half;
            int ks = 0;
            for (int k = 1; k < B; ++k)
                if (X.free_at[k] < X.free_at[ks]) ks = k;
            double s = std::max(a, X.free_at[ks]);
            double pf = a_pf * (double)u[best];
            double f = s + pf;
            double dec = a_dec * (double)out_len[r];
            double e = f + dec;
            X.free_at[ks] = e;
            double done = e + half;
            ttft[r] = (f + half) - t;
            e2e[r] = done - t;
            X.inflight.emplace(done, L);
            X.q += L;
        }

        if (route) route[r] = (uint8_t)best;
        if (hit_blocks) hit_blocks[r] = (uint16_t)m[best];
        if (believed_hit) believed_hit[r] = (uint16_t)m_seen[best];
        if (ttft_ms) ttft_ms[r] = ttft[r];
        if (e2e_ms) e2e_ms[r] = e2e[r];

        // online tuning (Sec. 4, tuning window: p95 TTFT over a rolling window, taken every hop requests): a step
        // when the first window is full and then every hop requests; a request's TTFT enters the window when the
        // request is dispatched (the stated service model gives it at once), and the weights a step leaves are
        // used from request r+1 on
        if (window > 0 && r + 1 >= window && (r + 1 - window) % hop == 0) {
            const int64_t h = (r + 1 - window) / hop;
            if (schedule) {
                w_rtt = schedule[3 * h + 0];
                w_prefill = schedule[3 * h + 1];
                w_queue = schedule[3 * h + 2];
            } else {
                const double f = gorgo_oracle_p95(ttft.data() + (r + 1 - window), window);
                if (!have_parent) {
                    // the first window measures the initial weights: they are the parent
                    f_par = f;
                    have_parent = true;
                } else {
                    // the offspring replaces the parent iff it beats it on the objective; the step size
                    // follows the 1/5 success rule
                    const bool success = f < f_par;
                    if (success) {
                        for (int k = 0; k < 3; ++k) ln_par[k] = ln_cur[k];
                        f_par = f;
                        ++accepted;
                    }
                    sigma = sigma * (success ? c_up : c_down);
                }
                // next offspring: multiplicative perturbation in log space, clipped to the range
                double th[3];
                for (int k = 0; k < 3; ++k) {
                    const double y = clip(ln_par[k] + sigma * z[3 * h + k], ln_lo[k], ln_hi[k]);
                    ln_cur[k] = y;
                    th[k] = clip(tuner_exp(y), lo[k], hi[k]);
                }
                w_rtt = th[0];
                w_prefill = th[1];
                w_queue = th[2];
                if (fitness_step) fitness_step[h] = f;
                ++steps;
            }
            if (theta_step) {
                theta_step[3 * h + 0] = w_rtt;
                theta_step[3 * h + 1] = w_prefill;
                theta_step[3 * h + 2] = w_queue;
            }
        }
    }
    if (tuner_final && window > 0 && !schedule) {
        for (int k = 0; k < 3; ++k) tuner_final[k] = clip(tuner_exp(ln_par[k]), lo[k], hi[k]);
        tuner_final[3] = sigma;
        tuner_final[4] = (double)steps;
        tuner_final[5] = (double)accepted;
    }
    if (p95) {
        p95[0] = gorgo_oracle_p95(ttft.data(), N);
        p95[1] = gorgo_oracle_p95(e2e.data(), N);
    }
    return 0;
}

int gorgo_oracle_replay_ex(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len,
                           const int64_t* blk_off, const int64_t* hash_ids, int32_t block_tokens,
                           int32_t R, int32_t B, int64_t C, double a_pf, double a_dec,
                           const double* rtt_ms, const double* w, double scale,
                           int32_t window, int32_t hop, const double* schedule, const double* z,
                           const double* lo, const double* hi, double sigma0, int32_t policy, uint64_t seed,
                           uint8_t* route, uint16_t* hit_blocks, double* ttft_ms, double* e2e_ms, double* p95,
                           double* score_dbg, int64_t* q_dbg, int64_t* size_dbg,
                           double* theta_step, double* fitness_step, double* tuner_final) {
    return replay_impl(N, ts_ms, in_len, out_len, blk_off, hash_ids, block_tokens, R, B, C, a_pf, a_dec, rtt_ms, w,
                       scale, window, hop, schedule, z, lo, hi, sigma0, policy, seed, nullptr, nullptr, nullptr, nullptr, route,
                       hit_blocks, ttft_ms, e2e_ms, p95, score_dbg, q_dbg, size_dbg, theta_step, fitness_step,
                       tuner_final);
}

// The same replay with the engine model of a replica: a_pf_r[R], a_dec_r[R] = per-replica service rates,
// kv_tokens[R] = KV budgets in tokens (null or 0 = none), slowdown >= 0.  a_pf stays the cost model's rate.
int gorgo_oracle_replay_engine(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len,
                               const int64_t* blk_off, const int64_t* hash_ids, int32_t block_tokens,
                               int32_t R, int32_t B, int64_t C, double a_pf,
                               const double* a_pf_r, const double* a_dec_r, const int64_t* kv_tokens, double slowdown,
                               const double* rtt_ms, const double* w, double scale,
                               int32_t window, int32_t hop, const double* schedule, const double* z,
                               const double* lo, const double* hi, double sigma0, int32_t policy, uint64_t seed,
                               uint8_t* route, uint16_t* hit_blocks, double* ttft_ms, double* e2e_ms, double* p95,
                               double* theta_step, double* fitness_step, double* tuner_final) {
    if (!a_pf_r || !a_dec_r || !(slowdown >= 0.0)) return -1;
    if (kv_tokens)
        for (int i = 0; i < R; ++i)
            if (kv_tokens[i] < 0) return -1;
    const Engine engine{a_pf_r, a_dec_r, kv_tokens, slowdown};
    return replay_impl(N, ts_ms, in_len, out_len, blk_off, hash_ids, block_tokens, R, B, C, a_pf, 0.0, rtt_ms, w,
                       scale, window, hop, schedule, z, lo, hi, sigma0, policy, seed, &engine, nullptr, nullptr, nullptr, route,
                       hit_blocks, ttft_ms, e2e_ms, p95, nullptr, nullptr, nullptr, theta_step, fitness_step,
                       tuner_final);
}

// The same replay with imperfect proxy knowledge (see Proxy): rtt_true[epochs][R] replaces rtt_ms; the engine
// model is used when a_pf_r is not null (then a_dec is ignored), else the linear model.  Extra outputs, each may
// be null: rtt_est[epochs][R] = the proxy's smoothed round trip times, believed_hit[N] = blocks the proxy's
// index matched on the chosen replica (hit_blocks stays what the replica's cache really held).
int gorgo_oracle_replay_proxy(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len,
                              const int64_t* blk_off, const int64_t* hash_ids, int32_t block_tokens,
                              int32_t R, int32_t B, int64_t C, double a_pf, double a_dec,
                              const double* a_pf_r, const double* a_dec_r, const int64_t* kv_tokens, double slowdown,
                              int32_t epochs, int32_t probe_ms, const double* rtt_true, double alpha, int64_t index_blocks,
                              const double* w, double scale,
                              int32_t window, int32_t hop, const double* z,
                              const double* lo, const double* hi, double sigma0,
                              uint8_t* route, uint16_t* hit_blocks, double* ttft_ms, double* e2e_ms, double* p95,
                              double* score_dbg, double* rtt_est, uint16_t* believed_hit,
                              double* theta_step, double* fitness_step, double* tuner_final) {
    if (epochs < 1 || probe_ms < 1 || !rtt_true || !(alpha > 0.0) || !(alpha <= 1.0)) return -1;
    if (a_pf_r && (!a_dec_r || !(slowdown >= 0.0))) return -1;
    const Engine engine{a_pf_r, a_dec_r, kv_tokens, slowdown};
    const Proxy proxy{epochs, probe_ms, rtt_true, alpha, index_blocks};
    return replay_impl(N, ts_ms, in_len, out_len, blk_off, hash_ids, block_tokens, R, B, C, a_pf, a_dec, rtt_true, w,
                       scale, window, hop, nullptr, z, lo, hi, sigma0, 0, 0, a_pf_r ? &engine : nullptr, &proxy, rtt_est,
                       believed_hit, route, hit_blocks, ttft_ms, e2e_ms, p95, score_dbg, nullptr, nullptr, theta_step,
                       fitness_step, tuner_final);
}

// One replay under one fixed weight vector.
int gorgo_oracle_replay(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len,
                        const int64_t* blk_off, const int64_t* hash_ids, int32_t block_tokens,
                        int32_t R, int32_t B, int64_t C, double a_pf, double a_dec,
                        const double* rtt_ms, const double* w, double scale,
                        uint8_t* route, uint16_t* hit_blocks, double* ttft_ms, double* e2e_ms, double* p95,
                        double* score_dbg, int64_t* q_dbg, int64_t* size_dbg) {
    return gorgo_oracle_replay_ex(N, ts_ms, in_len, out_len, blk_off, hash_ids, block_tokens, R, B, C, a_pf, a_dec,
                                  rtt_ms, w, scale, 0, 0, nullptr, nullptr, nullptr, nullptr, 0.0, 0, 0, route,
                                  hit_blocks, ttft_ms, e2e_ms, p95, score_dbg, q_dbg, size_dbg, nullptr, nullptr,
                                  nullptr);
}

}  // extern "C"

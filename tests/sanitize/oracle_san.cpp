// The CPU oracle (oracle/gorgo_oracle.cpp) under AddressSanitizer and UndefinedBehaviorSanitizer: seeded small
// traces in the shapes that stress its bookkeeping (empty trace, one replica, one slot, unbounded and tiny caches,
// repeated blocks inside a request, equal timestamps), replayed through every entry point.  usage: oracle_san SEED ROUNDS
// (tests/test_sanitized_host.py compiles and runs it).  Checks only what holds for any replay: statuses, ranges,
// hit <= blocks, ttft <= e2e, finite latencies.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
int gorgo_oracle_replay(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len, const int64_t* blk_off,
                        const int64_t* hash_ids, int32_t block_tokens, int32_t R, int32_t B, int64_t C, double a_pf, double a_dec,
                        const double* rtt_ms, const double* w, double scale, uint8_t* route, uint16_t* hit_blocks,
                        double* ttft_ms, double* e2e_ms, double* p95, double* score_dbg, int64_t* q_dbg, int64_t* size_dbg);
int gorgo_oracle_replay_ex(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len, const int64_t* blk_off,
                           const int64_t* hash_ids, int32_t block_tokens, int32_t R, int32_t B, int64_t C, double a_pf,
                           double a_dec, const double* rtt_ms, const double* w, double scale, int32_t window, int32_t hop,
                           const double* schedule, const double* z, const double* lo, const double* hi, double sigma0,
                           int32_t policy, uint64_t seed, uint8_t* route, uint16_t* hit_blocks, double* ttft_ms,
                           double* e2e_ms, double* p95, double* score_dbg, int64_t* q_dbg, int64_t* size_dbg,
                           double* theta_step, double* fitness_step, double* tuner_final);
int gorgo_oracle_replay_engine(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len,
                               const int64_t* blk_off, const int64_t* hash_ids, int32_t block_tokens, int32_t R, int32_t B,
                               int64_t C, double a_pf, const double* a_pf_r, const double* a_dec_r, const int64_t* kv_tokens,
                               double slowdown, const double* rtt_ms, const double* w, double scale, int32_t window,
                               int32_t hop, const double* schedule, const double* z, const double* lo, const double* hi,
                               double sigma0, int32_t policy, uint64_t seed, uint8_t* route, uint16_t* hit_blocks,
                               double* ttft_ms, double* e2e_ms, double* p95, double* theta_step, double* fitness_step,
                               double* tuner_final);
int gorgo_oracle_replay_proxy(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len,
                              const int64_t* blk_off, const int64_t* hash_ids, int32_t block_tokens, int32_t R, int32_t B,
                              int64_t C, double a_pf, double a_dec, const double* a_pf_r, const double* a_dec_r,
                              const int64_t* kv_tokens, double slowdown, int32_t epochs, int32_t probe_ms,
                              const double* rtt_true, double alpha, int64_t index_blocks, const double* w, double scale,
                              int32_t window, int32_t hop, const double* z, const double* lo, const double* hi, double sigma0,
                              uint8_t* route, uint16_t* hit_blocks, double* ttft_ms, double* e2e_ms, double* p95,
                              double* score_dbg, double* rtt_est, uint16_t* believed_hit, double* theta_step,
                              double* fitness_step, double* tuner_final);
int64_t gorgo_oracle_online_steps(int64_t N, int32_t window, int32_t hop);
}

static uint64_t rng_state;
static uint64_t rnd() {
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static uint64_t below(uint64_t n) { return n ? rnd() % n : 0; }
static double unit() { return (double)(rnd() >> 11) / 9007199254740992.0; }

#define CHECK(cond)                                                                          \
    do {                                                                                     \
        if (!(cond)) {                                                                       \
            std::fprintf(stderr, "oracle_san: check failed at line %d: %s\n", __LINE__, #cond); \
            std::exit(3);                                                                    \
        }                                                                                    \
    } while (0)

struct Trace {
    std::vector<int64_t> ts, off, ids;
    std::vector<int32_t> in_len, out_len;
    int64_t N = 0;
    int max_distinct = 0;
};

static Trace make_trace(int n) {
    Trace t;
    t.N = n;
    t.off.push_back(0);
    int64_t ts = 0;
    std::vector<int64_t> session;
    for (int r = 0; r < n; ++r) {
        ts += below(3) ? (int64_t)below(40) : 0;        // equal timestamps happen
        if (below(3) == 0) session.clear();
        const int add = (int)below(5);
        for (int k = 0; k < add; ++k) session.push_back(below(5) ? (int64_t)below(1u << 16) : (session.empty() ? 7 : session[below(session.size())]));
        t.ts.push_back(ts);
        t.in_len.push_back((int32_t)(session.size() * 16 + below(16)));
        t.out_len.push_back(1 + (int32_t)below(50));
        for (int64_t id : session) t.ids.push_back(id);
        t.off.push_back((int64_t)t.ids.size());
        std::vector<int64_t> d(session);
        int distinct = 0;
        for (size_t a = 0; a < d.size(); ++a) {
            bool seen = false;
            for (size_t b = 0; b < a; ++b) seen = seen || d[b] == d[a];
            distinct += seen ? 0 : 1;
        }
        t.max_distinct = distinct > t.max_distinct ? distinct : t.max_distinct;
    }
    return t;
}

static void check_outputs(const Trace& t, int R, const std::vector<uint8_t>& route, const std::vector<uint16_t>& hit,
                          const std::vector<double>& ttft, const std::vector<double>& e2e) {
    for (int64_t r = 0; r < t.N; ++r) {
        CHECK(route[r] < R);
        CHECK((int64_t)hit[r] <= t.off[r + 1] - t.off[r]);
        CHECK(std::isfinite(ttft[r]) && std::isfinite(e2e[r]) && ttft[r] >= 0.0 && ttft[r] <= e2e[r]);
    }
}

int main(int argc, char** argv) {
    if (argc != 3) {
        std::fprintf(stderr, "usage: oracle_san SEED ROUNDS\n");
        return 2;
    }
    rng_state = std::strtoull(argv[1], nullptr, 10);
    const long rounds = std::strtol(argv[2], nullptr, 10);
    for (long it = 0; it < rounds; ++it) {
        const int n = it == 0 ? 0 : (int)below(400);
        const Trace t = make_trace(n);
        const int R = 1 + (int)below(below(4) ? 8 : 64), B = 1 + (int)below(below(4) ? 4 : 64);
        const int64_t C = below(3) == 0 ? 0 : t.max_distinct + (int64_t)below(40);
        std::vector<double> rtt(R), w = {unit() * 2, unit() * 2, unit()};
        for (auto& x : rtt) x = unit() * 200.0;
        const double scale = 0.25 + unit() * 4;
        const size_t N = (size_t)t.N;
        std::vector<uint8_t> route(N + 1);
        std::vector<uint16_t> hit(N + 1), believed(N + 1);
        std::vector<double> ttft(N + 1), e2e(N + 1), score(N * R + 1);
        std::vector<int64_t> qd(N * R + 1), sz(N * R + 1);
        double p95[2] = {0, 0};
        CHECK(gorgo_oracle_replay(t.N, t.ts.data(), t.in_len.data(), t.out_len.data(), t.off.data(), t.ids.data(), 16, R, B, C, 0.05,
                                  20.0, rtt.data(), w.data(), scale, route.data(), hit.data(), ttft.data(), e2e.data(), p95,
                                  score.data(), qd.data(), sz.data()) == 0);
        check_outputs(t, R, route, hit, ttft, e2e);
        // policies
        for (int policy = 1; policy <= 3; ++policy) {
            CHECK(gorgo_oracle_replay_ex(t.N, t.ts.data(), t.in_len.data(), t.out_len.data(), t.off.data(), t.ids.data(), 16, R, B, C,
                                         0.05, 20.0, rtt.data(), w.data(), scale, 0, 0, nullptr, nullptr, nullptr, nullptr, 0.0,
                                         policy, rnd(), route.data(), hit.data(), ttft.data(), e2e.data(), p95, nullptr, nullptr,
                                         nullptr, nullptr, nullptr, nullptr) == 0);
            check_outputs(t, R, route, hit, ttft, e2e);
        }
        // online tuner
        const int window = 8 + (int)below(24), hop = 1 + (int)below(8);
        const int64_t steps = gorgo_oracle_online_steps(t.N, window, hop);
        CHECK(steps >= 0);
        std::vector<double> z((size_t)steps * 3 + 3), th((size_t)steps * 3 + 3), fs((size_t)steps + 1);
        for (auto& x : z) x = (unit() - 0.5) * 4;
        const double lo[3] = {0.05, 1.0, 0.05}, hi[3] = {2.0, 1.0, 0.5};
        double fin[6] = {0, 0, 0, 0, 0, 0};      // weights, step size, steps, accepted
        const double th0[3] = {0.5, 1.0, 0.1};
        CHECK(gorgo_oracle_replay_ex(t.N, t.ts.data(), t.in_len.data(), t.out_len.data(), t.off.data(), t.ids.data(), 16, R, B, C, 0.05,
                                     20.0, rtt.data(), th0, scale, window, hop, nullptr, z.data(), lo, hi, 0.5, 0, 0, route.data(),
                                     hit.data(), ttft.data(), e2e.data(), p95, nullptr, nullptr, nullptr, th.data(), fs.data(),
                                     fin) == 0);
        check_outputs(t, R, route, hit, ttft, e2e);
        // engine model and imperfect proxy knowledge
        std::vector<double> apf(R), adec(R);
        std::vector<int64_t> kv(R);
        for (int i = 0; i < R; ++i) {
            apf[i] = 0.02 + unit() * 0.1;
            adec[i] = 5 + unit() * 30;
            kv[i] = below(3) ? (int64_t)(2000 + below(20000)) : 0;
        }
        CHECK(gorgo_oracle_replay_engine(t.N, t.ts.data(), t.in_len.data(), t.out_len.data(), t.off.data(), t.ids.data(), 16, R, B, C,
                                         0.05, apf.data(), adec.data(), kv.data(), unit() * 0.1, rtt.data(), w.data(), scale, 0, 0,
                                         nullptr, nullptr, nullptr, nullptr, 0.0, 0, 0, route.data(), hit.data(), ttft.data(),
                                         e2e.data(), p95, nullptr, nullptr, nullptr) == 0);
        check_outputs(t, R, route, hit, ttft, e2e);
        const int epochs = 1 + (int)below(6), probe = 1 + (int)below(500);
        std::vector<double> rt((size_t)epochs * R), est((size_t)epochs * R);
        for (auto& x : rt) x = 1 + unit() * 200;
        const int64_t index_blocks = below(3) == 0 ? -1 : (below(2) ? 0 : t.max_distinct + C + (int64_t)below(50));
        CHECK(gorgo_oracle_replay_proxy(t.N, t.ts.data(), t.in_len.data(), t.out_len.data(), t.off.data(), t.ids.data(), 16, R, B, C,
                                        0.05, 20.0, below(2) ? apf.data() : nullptr, adec.data(), kv.data(), 0.05, epochs, probe,
                                        rt.data(), 0.05 + unit() * 0.95, index_blocks, w.data(), scale, 0, 0, nullptr, nullptr,
                                        nullptr, 0.0, route.data(), hit.data(), ttft.data(), e2e.data(), p95, nullptr, est.data(),
                                        believed.data(), nullptr, nullptr, nullptr) == 0);
        check_outputs(t, R, route, hit, ttft, e2e);
    }
    std::printf("oracle_san: %ld rounds\n", rounds);
    return 0;
}

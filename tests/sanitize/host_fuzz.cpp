// Seeded mutation fuzz of libgorgo's host side, built with AddressSanitizer and UndefinedBehaviorSanitizer
// (tests/test_sanitized_host.py compiles and runs it).  usage: host_fuzz SEED ITERATIONS SCRATCH_FILE
// Each iteration writes a small valid JSON-lines trace (Sec. 3 layout: timestamp, input_length, output_length,
// hash_ids), damages it in one of several ways (or not at all), loads it, and on success walks the host-side entry
// points with ordinary and hostile arguments.  Nothing here has an expected value beyond "returns a documented
// status and the sanitizers stay silent"; valid files must load, and what they report must match what was written.
#include <cinttypes>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <string>
#include <vector>

#include "gorgo.h"

static uint64_t rng_state;
static uint64_t rnd() {       // SplitMix64
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static uint64_t below(uint64_t n) { return n ? rnd() % n : 0; }

#define CHECK(cond)                                                                                   \
    do {                                                                                              \
        if (!(cond)) {                                                                                \
            std::fprintf(stderr, "host_fuzz: check failed at line %d: %s (last error: %s)\n", __LINE__, #cond, \
                         gorgo_last_error());                                                         \
            std::exit(3);                                                                             \
        }                                                                                             \
    } while (0)

static bool documented(int rc) { return rc <= 0 && rc >= -9; }

struct Written {
    int64_t n = 0, blocks = 0;
};

static std::string valid_trace(Written* w) {
    std::string s;
    const int n = 1 + (int)below(24);
    int64_t ts = (int64_t)below(1000);
    std::vector<int64_t> session;       // a growing prefix, so that the trace is chain-consistent most of the time
    for (int r = 0; r < n; ++r) {
        ts += (int64_t)below(50);
        if (below(4) == 0) session.clear();
        const int add = (int)below(6);
        for (int k = 0; k < add; ++k) session.push_back((int64_t)below(1u << 20));
        char buf[256];
        std::snprintf(buf, sizeof buf, "{\"timestamp\": %" PRId64 ", \"input_length\": %d, \"output_length\": %d, \"hash_ids\": [",
                      ts, (int)(session.size() * 512 + below(512)), 1 + (int)below(300));
        s += buf;
        for (size_t k = 0; k < session.size(); ++k) {
            std::snprintf(buf, sizeof buf, "%s%" PRId64, k ? ", " : "", session[k]);
            s += buf;
        }
        s += "]}\n";
        w->blocks += (int64_t)session.size();
    }
    w->n = n;
    return s;
}

static void damage(std::string& s) {
    static const char* const fragments[] = {"{", "}", "[", "]", "\"", ",", ":", "-", "e308", "1e999", "99999999999999999999999",
                                            "-1", "null", "\"timestamp\"", "\"hash_ids\": [", "\\u0000", "\n", "\n\n", " ", "0x10",
                                            "\"input_length\": -5", "\"output_length\": 4294967296", "\t", "\r\n", "nan", "1.5",
                                            "\xEF\xBB\xBF", "[[1, 2], [3]]", "[1, [2, [3, [4]]]]", "1e", "-", "1.", "00012", "+7"};
    const int kind = (int)below(9);
    if (s.empty()) return;
    const size_t at = (size_t)below(s.size());
    switch (kind) {
        case 0: s[at] = (char)below(256); break;                                     // one byte
        case 1: s.erase(at, (size_t)below(1 + s.size() - at)); break;               // cut a tail or a middle
        case 2: s.insert(at, fragments[below(sizeof fragments / sizeof *fragments)]); break;
        case 3: s.insert(at, s.substr((size_t)below(s.size()), (size_t)below(64))); break;      // duplicate a piece
        case 4: s.resize(at); break;                                                 // truncate
        case 5: for (int k = 0; k < 8; ++k) s[(size_t)below(s.size())] = (char)below(256); break;
        case 6:
            if (below(4) == 0) {
                // a request with more ids than a request may have (65,535), as one well-formed line
                std::string line = "{\"timestamp\": 999999999, \"input_length\": 1, \"output_length\": 1, \"hash_ids\": [";
                const int n = 65530 + (int)below(5000);
                for (int k = 0; k < n; ++k) line += k ? ",1" : "1";
                s += line + "]}\n";
            } else {
                s.insert(at, std::string((size_t)below(5000), "0123456789[,"[below(12)]));     // a long run
            }
            break;
        case 7: s.insert(0, "\xEF\xBB\xBF"); break;                                   // a byte-order mark in front
        default: {                                                                   // swap two lines (timestamps may decrease)
            const size_t a = s.find('\n', at);
            if (a != std::string::npos && a + 1 < s.size()) {
                const std::string head = s.substr(0, a + 1), tail = s.substr(a + 1);
                s = tail + head;
            }
        }
    }
}

static void walk(const gorgo_trace* t, bool pristine, const Written& w) {
    int64_t N = 0, total = 0, unique = 0;
    int32_t maxb = 0, chain = 0;
    CHECK(gorgo_trace_info(t, &N, &total, &maxb, &unique, &chain) == 0);
    CHECK(N >= 0 && total >= 0 && maxb >= 0 && unique >= 0 && unique <= total && (chain == 0 || chain == 1));
    if (pristine) CHECK(N == w.n && total == w.blocks);
    CHECK(gorgo_trace_info(t, nullptr, nullptr, nullptr, nullptr, nullptr) == 0);
    int32_t path = 0;
    int64_t nseg = 0, refs = 0;
    CHECK(gorgo_query_replay_path(t, nullptr, &path, &nseg, &refs) == 0 && (path == 1 || path == 2) && nseg >= 0 && refs >= 0);
    for (int k = 0; k < 6; ++k) {
        gorgo_model m;
        m.R = (int32_t)below(70) - 2;
        m.batch = (int32_t)below(70) - 2;
        m.block_tokens = below(3) ? 512 : (int32_t)below(70000);
        m._pad = 0;
        m.cache_blocks = below(3) ? (int64_t)below(64) : (int64_t)rnd();
        m.prefill_ms_per_token = below(5) ? 0.05 : (below(2) ? std::numeric_limits<double>::quiet_NaN() : -1.0);
        m.decode_ms_per_token = below(5) ? 20.0 : 1e300;
        gorgo_options o;
        gorgo_options_default(&o);
        if (below(2)) {
            o.replay_path = (int32_t)below(5) - 1;
            o.replay_packing = (int32_t)below(5) - 1;
            o.handover_poll_limit = (int32_t)rnd();
            o.table_factor_percent = (int32_t)below(2000);
        }
        const int32_t P = below(4) ? 1 + (int32_t)below(64) : (int32_t)rnd();
        gorgo_outputs out;
        std::memset(&out, 0, sizeof out);
        if (below(2)) out.p95_ttft_ms = reinterpret_cast<double*>(256);
        if (below(2)) out.route = reinterpret_cast<uint8_t*>(256);
        size_t bytes = 0;
        const int rc = gorgo_workspace_bytes(t, &m, below(2) ? &o : nullptr, P, below(2) ? &out : nullptr, &bytes);
        CHECK(documented(rc));
        if (rc == 0) CHECK(bytes > 0 && bytes % 256 == 0);
        size_t es_bytes = 0;
        CHECK(documented(gorgo_es_workspace_bytes(t, &m, &o, P, &es_bytes)));
        int32_t packed = -1;
        CHECK(documented(gorgo_query_replay_packing(t, &m, &o, P, &packed)));
        // an evaluation gets as far as the first device operation at most (this build has none)
        std::vector<double> rtt(64, 10.0), par(3 * 64, 1.0), sc(64, 1.0);
        const int32_t Pe = P >= 1 && P <= 64 ? P : 2;
        const int erc = gorgo_eval_population(t, &m, &o, rtt.data(), par.data(), sc.data(), Pe, &out, reinterpret_cast<void*>(256),
                                              (size_t)1 << 40, nullptr);
        CHECK(erc < 0 && documented(erc));
    }
}

static void es_walk() {
    gorgo_es_state s;
    CHECK(gorgo_es_init(&s, rnd()) == 0);
    CHECK(gorgo_es_init(nullptr, 1) == GORGO_ERR_INVALID_ARG);
    const int32_t P = 1 + (int32_t)below(40);
    std::vector<double> z(3 * (size_t)P), par(3 * (size_t)P), fit((size_t)P);
    CHECK(gorgo_es_sample(rnd(), (int64_t)below(1000), P, z.data()) == 0);
    for (double v : z) CHECK(std::isfinite(v));
    CHECK(gorgo_es_propose(&s, z.data(), P, par.data()) == 0);
    for (size_t k = 0; k < par.size(); ++k) CHECK(par[k] >= s.lo[k % 3] && par[k] <= s.hi[k % 3]);
    for (auto& f : fit) f = (double)below(100000) / 7.0;
    if (below(3) == 0) fit[below((uint64_t)P)] = std::numeric_limits<double>::quiet_NaN();
    if (below(3) == 0) z[below(z.size())] = std::numeric_limits<double>::infinity();
    CHECK(documented(gorgo_es_propose(&s, z.data(), P, par.data())));
    const int rc = gorgo_es_update(par.data(), fit.data(), P, &s);
    CHECK(documented(rc));
    if (rc == 0) CHECK(std::isfinite(s.sigma) && s.sigma > 0.0);
    CHECK(documented(gorgo_es_sample(1, -1, P, z.data())));
    CHECK(documented(gorgo_es_sample(1, 0, 0, z.data())));
    CHECK(documented(gorgo_es_update(par.data(), fit.data(), -3, &s)));
    uint32_t ctr[4] = {(uint32_t)rnd(), (uint32_t)rnd(), (uint32_t)rnd(), (uint32_t)rnd()}, key[2] = {(uint32_t)rnd(), (uint32_t)rnd()}, out4[4];
    gorgo_philox4x32_10(ctr, key, out4);
    CHECK(gorgo_online_steps(-1, 128, 32) < 0 && gorgo_online_steps(1000, 128, 32) == 28);
}

int main(int argc, char** argv) {
    if (argc != 4) {
        std::fprintf(stderr, "usage: host_fuzz SEED ITERATIONS SCRATCH_FILE\n");
        return 2;
    }
    rng_state = std::strtoull(argv[1], nullptr, 10);
    const long iterations = std::strtol(argv[2], nullptr, 10);
    const char* path = argv[3];
    long loaded = 0, refused = 0;
    for (long it = 0; it < iterations; ++it) {
        Written w;
        std::string text = valid_trace(&w);
        const int hits = (int)below(4);              // 0: left as written
        for (int k = 0; k < hits; ++k) damage(text);
        FILE* f = std::fopen(path, "wb");
        CHECK(f != nullptr);
        CHECK(std::fwrite(text.data(), 1, text.size(), f) == text.size());
        std::fclose(f);
        gorgo_trace* t = nullptr;
        const int32_t bt = below(8) ? 512 : (int32_t)below(70000) - 10;
        const int rc = gorgo_load_trace(path, bt, &t);
        CHECK(documented(rc));
        if (hits == 0 && bt == 512) CHECK(rc == 0);
        if (rc == 0) {
            CHECK(t != nullptr);
            ++loaded;
            walk(t, hits == 0, w);
            gorgo_free_trace(t);
        } else {
            CHECK(t == nullptr && gorgo_last_error()[0] != 0);
            ++refused;
        }
        if (it % 16 == 0) es_walk();
    }
    gorgo_trace* t = nullptr;
    CHECK(gorgo_load_trace("/nonexistent/trace.jsonl", 512, &t) == GORGO_ERR_IO);
    CHECK(gorgo_load_trace(nullptr, 512, &t) == GORGO_ERR_INVALID_ARG);
    CHECK(gorgo_load_trace(path, 512, nullptr) == GORGO_ERR_INVALID_ARG);
    gorgo_free_trace(nullptr);
    std::printf("host_fuzz: %ld iterations, %ld files loaded, %ld refused\n", iterations, loaded, refused);
    return loaded > 0 && refused > 0 ? 0 : 4;
}

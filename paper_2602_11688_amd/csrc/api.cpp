// Evaluation entry points of the C ABI: argument validation, workspace layout, launches, ES generation.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <limits>
#include <string>
#include <vector>

#include "internal.h"

namespace gorgo {
namespace {


size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

constexpr gorgo_options DEFAULT_OPTIONS = {PATH_AUTO, 2, 1 << 24, 200};

// The caller's options (NULL: the defaults), checked.
int take_options(const gorgo_options* given, gorgo_options* out) {
    *out = given ? *given : DEFAULT_OPTIONS;
    if (out->replay_path != PATH_AUTO && out->replay_path != PATH_BLOCKS && out->replay_path != PATH_SEGMENTS)
        return fail(GORGO_ERR_INVALID_ARG, "options.replay_path must be 0 (auto), 1 (block tables) or 2 (segment rows)");
    if (out->replay_packing < 0 || out->replay_packing > 2)
        return fail(GORGO_ERR_INVALID_ARG, "options.replay_packing must be 0 (never), 1 (whenever possible) or 2 (automatic)");
    if (out->handover_poll_limit < 0) return fail(GORGO_ERR_INVALID_ARG, "options.handover_poll_limit must be >= 0");
    if (out->table_factor_percent < 110 || out->table_factor_percent > 1600)
        return fail(GORGO_ERR_INVALID_ARG, "options.table_factor_percent must be in 110..1600");
    return GORGO_OK;
}

// which formulation a trace gets under a replay_path setting
int32_t path_for(const gorgo_trace* t, int32_t mode) {
    const bool few = (int64_t)t->seg.size() <= 16 * (t->N > 0 ? t->N : 1);
    return mode == PATH_SEGMENTS || (mode == PATH_AUTO && t->chain_consistent && few) ? PATH_SEGMENTS : PATH_BLOCKS;
}

int check_model(const gorgo_trace* t, const gorgo_model* m) {
    if (!t) return fail(GORGO_ERR_INVALID_ARG, "trace is NULL");
    if (!m) return fail(GORGO_ERR_INVALID_ARG, "model is NULL");
    if (m->R < 1 || m->R > 64) return fail(GORGO_ERR_INVALID_ARG, "R must be in 1..64");
    if (m->batch < 1 || m->batch > 64) return fail(GORGO_ERR_INVALID_ARG, "batch must be in 1..64");
    if ((int64_t)m->R * m->batch > 1024) return fail(GORGO_ERR_INVALID_ARG, "R * batch must not exceed 1024");
    if (m->block_tokens < 1 || m->block_tokens > 32767)      // (tokens of a cached prefix are counted in 32 bits)
        return fail(GORGO_ERR_INVALID_ARG, "block_tokens must be in 1..32767");
    if (m->block_tokens != t->block_tokens)
        return fail(GORGO_ERR_INVALID_ARG, "model.block_tokens differs from the trace's");
    if (m->cache_blocks < 0 || m->cache_blocks > ((int64_t)1 << 30))
        return fail(GORGO_ERR_INVALID_ARG, "cache_blocks must be in 0..2^30");
    if (!std::isfinite(m->prefill_ms_per_token) || !std::isfinite(m->decode_ms_per_token))
        return fail(GORGO_ERR_NONFINITE, "service constants must be finite");
    if (m->prefill_ms_per_token < 0 || m->prefill_ms_per_token > 1e6 || m->decode_ms_per_token < 0 ||
        m->decode_ms_per_token > 1e6)
        return fail(GORGO_ERR_NONFINITE, "service constants must be in 0..1e6 ms per token");
    if (m->cache_blocks > 0 && t->max_distinct > m->cache_blocks)
        return fail(GORGO_ERR_CAPACITY, "a request has " + std::to_string(t->max_distinct) +
                                            " distinct blocks but the cache holds " + std::to_string(m->cache_blocks));
    return GORGO_OK;
}

// Fewest slots of a block table that holds `resident` entries while a request of up to d distinct blocks is being
// inserted, given that the replay compacts a table once 7/8 of its slots have been used.
int64_t least_table_slots(int64_t resident, int64_t d) { return ((resident + d) * 8 + 6) / 7 + 64; }

// Table geometry and workspace carve-up.
int make_plan(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, int32_t P, const gorgo_outputs* o,
              Plan* pl) {
    if (P < 1 || P > (1 << 20)) return fail(GORGO_ERR_INVALID_ARG, "P must be in 1..2^20");
    gorgo_options opt;
    int orc = take_options(options, &opt);
    if (orc) return orc;
    pl->packing = opt.replay_packing;
    pl->poll_limit = opt.handover_poll_limit;
    pl->P = P;
    pl->R = m->R;
    pl->B = m->batch;
    pl->N = t->N;
    pl->C = m->cache_blocks;
    pl->block_tokens = m->block_tokens;
    pl->a_pf = m->prefill_ms_per_token;
    pl->a_dec = m->decode_ms_per_token;
    // Formulation: dense segment rows when the trace is chain-consistent and its requests are few segments
    // long (every request then costs a handful of row reads); hashed block tables otherwise.
    if (opt.replay_path == PATH_SEGMENTS && !t->chain_consistent)
        return fail(GORGO_ERR_INVALID_ARG, "the segment formulation needs a chain-consistent trace");
    pl->path = path_for(t, opt.replay_path);
    pl->nseg = t->n_slots;           // rows: segments share them, see the loader
    if (pl->path == PATH_SEGMENTS && (uint64_t)(pl->nseg + 2) * (uint64_t)m->R * 4u >= (1ull << 32))
        return fail(GORGO_ERR_INVALID_ARG, "segment rows of one replay exceed 4 GiB; use the block-table formulation");
    // A table must hold the cached blocks plus the blocks of the request being inserted, with room to
    // spare: the replay compacts a table once 7/8 of its slots have been used.
    const int64_t d = t->max_distinct;
    const int64_t resident = (pl->C > 0 ? pl->C : t->unique_ids) + d;
    const int64_t factor = opt.table_factor_percent;
    int64_t need = (resident * factor + 99) / 100;
    const int64_t floor_need = least_table_slots(resident, d);
    if (need < floor_need) need = floor_need;
    int64_t cap = 128;
    while (cap < need) cap <<= 1;
    pl->cap = cap;
    const size_t N = (size_t)t->N;
    size_t off = 0;
    pl->off_tables = off;
    if (pl->path == PATH_SEGMENTS) {
        off += up256((size_t)P * (size_t)(pl->nseg + 2) * pl->R * 4);   // a row per segment, one that no request touches, a spare
        pl->off_spare = off;                              // per-request log records of the segment kernel
        off += up256((size_t)P * ((size_t)t->N + 1) * 8);            // (and a spare record per replay)
    } else {
        off += up256((size_t)P * pl->R * (size_t)cap * 16);
        pl->off_spare = off;
        off += up256((size_t)P * (size_t)cap * 16);
    }
    pl->off_rec = off;
    off += up256((size_t)P * N * 16);
    const bool want_p95_t = !o || o->p95_ttft_ms, want_p95_e = !o || o->p95_e2e_ms;
    pl->off_route = off;
    if (pl->path == PATH_BLOCKS) off += up256((size_t)P * N);   // the block kernel's log of choices (its eviction walks it)
    pl->off_ttft = off;
    if (!o || (!o->ttft_ms && want_p95_t)) off += up256((size_t)P * N * 8);
    pl->off_e2e = off;
    if (!o || (!o->e2e_ms && want_p95_e)) off += up256((size_t)P * N * 8);
    pl->off_small = off;
    // rtt, params, scale; tuner constants, ln theta0; seeds of the random policy; rates and budgets of the engine model
    off += up256((4 * (size_t)pl->R + 8 * (size_t)P + TUNER_CONSTS) * 8);
    pl->total = off;
    return GORGO_OK;
}

}  // namespace
}  // namespace gorgo

using namespace gorgo;

extern "C" {

void gorgo_options_default(gorgo_options* options) {
    if (options) *options = DEFAULT_OPTIONS;
}

int gorgo_query_replay_packing(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, int32_t P,
                               int32_t* packed) {
    clear_error();
    if (!packed) return fail(GORGO_ERR_INVALID_ARG, "packed is NULL");
    int rc = check_model(t, m);
    if (rc) return rc;
    Plan pl;
    rc = make_plan(t, m, options, P, nullptr, &pl);
    if (rc) return rc;
    *packed = pl.path == PATH_SEGMENTS && pack_replays(pl, pl.nseg + 2) ? 1 : 0;
    return GORGO_OK;
}

int gorgo_query_row_slots(const gorgo_trace* t, int64_t* slots) {
    clear_error();
    if (!t) return fail(GORGO_ERR_INVALID_ARG, "trace is NULL");
    if (!slots) return fail(GORGO_ERR_INVALID_ARG, "slots is NULL");
    *slots = t->n_slots;
    return GORGO_OK;
}

int gorgo_query_replay_path(const gorgo_trace* t, const gorgo_options* options, int32_t* path, int64_t* n_segments,
                            int64_t* segment_refs) {
    clear_error();
    if (!t) return fail(GORGO_ERR_INVALID_ARG, "trace is NULL");
    gorgo_options opt;
    const int orc = take_options(options, &opt);
    if (orc) return orc;
    if (path) *path = path_for(t, opt.replay_path);
    if (n_segments) *n_segments = t->n_segments;
    if (segment_refs) *segment_refs = (int64_t)t->seg.size();
    return GORGO_OK;
}

int gorgo_workspace_bytes(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, int32_t P,
                          const gorgo_outputs* outputs,
                          size_t* bytes) {
    clear_error();
    if (!bytes) return fail(GORGO_ERR_INVALID_ARG, "bytes is NULL");
    int rc = check_model(t, m);
    if (rc) return rc;
    Plan pl;
    rc = make_plan(t, m, options, P, outputs, &pl);
    if (rc) return rc;
    *bytes = pl.total;
    return GORGO_OK;
}

}  // extern "C"

namespace {

// Validation, small copies and launches common to the fixed-weight and the online evaluation.
int evaluate(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, const double* rtt_ms,
             const double* params,
             const double* scale, int32_t P, const gorgo_online* online, int32_t policy, const uint64_t* seeds,
             const gorgo_outputs* outputs, void* workspace, size_t workspace_bytes, void* hip_stream,
             const gorgo_engine* engine = nullptr, const gorgo_proxy* proxy = nullptr,
             unsigned long long* sections = nullptr) {
    int rc = check_model(t, m);
    if (rc) return rc;
    if (proxy) {
        if (proxy->epochs < 1 || proxy->epochs > 65536) return fail(GORGO_ERR_INVALID_ARG, "epochs must be in 1..65536");
        if (proxy->probe_interval_ms < 1) return fail(GORGO_ERR_INVALID_ARG, "probe_interval_ms must be >= 1");
        if (!proxy->rtt_true_ms || !proxy->rtt_tables) return fail(GORGO_ERR_INVALID_ARG, "the proxy's round trip time tables are NULL");
        if (!(proxy->ewma_alpha > 0.0) || !(proxy->ewma_alpha <= 1.0))
            return fail(GORGO_ERR_NONFINITE, "ewma_alpha must be in (0, 1]");
        if (proxy->index_blocks < -1 || proxy->index_blocks > ((int64_t)1 << 30))
            return fail(GORGO_ERR_INVALID_ARG, "index_blocks must be -1 (none), 0 (never forgets) or a capacity up to 2^30");
        if (proxy->index_blocks > 0 && (m->cache_blocks == 0 || proxy->index_blocks < m->cache_blocks))
            return fail(GORGO_ERR_INVALID_ARG, "an index of its own must hold at least cache_blocks (the replicas' caches are " +
                                                   std::string(m->cache_blocks == 0 ? "unbounded" : "larger") + ")");
        for (int64_t j = 0; j < (int64_t)proxy->epochs * m->R; ++j)
            if (!std::isfinite(proxy->rtt_true_ms[j]) || proxy->rtt_true_ms[j] < 0 || proxy->rtt_true_ms[j] > 1e9)
                return fail(GORGO_ERR_NONFINITE, "rtt_true_ms[" + std::to_string(j / m->R) + "][" + std::to_string(j % m->R) +
                                                     "] must be finite and in 0..1e9");
        rtt_ms = proxy->rtt_true_ms;      // (its first row stands in where a single row is copied below)
    }
    std::vector<double> eng;        // a_pf[R], a_dec[R], budget[R]
    if (engine) {
        if (!engine->prefill_ms_per_token || !engine->decode_ms_per_token)
            return fail(GORGO_ERR_INVALID_ARG, "engine rates are NULL");
        if (!std::isfinite(engine->decode_slowdown) || engine->decode_slowdown < 0 || engine->decode_slowdown > 1e3)
            return fail(GORGO_ERR_NONFINITE, "decode_slowdown must be finite and in 0..1e3");
        eng.assign(3 * (size_t)m->R, 0.0);
        for (int i = 0; i < m->R; ++i) {
            const double pf = engine->prefill_ms_per_token[i], dec = engine->decode_ms_per_token[i];
            if (!std::isfinite(pf) || pf < 0 || pf > 1e6 || !std::isfinite(dec) || dec < 0 || dec > 1e6)
                return fail(GORGO_ERR_NONFINITE, "engine rates of replica " + std::to_string(i) +
                                                     " must be finite and in 0..1e6");
            const int64_t kv = engine->kv_tokens ? engine->kv_tokens[i] : 0;
            if (kv < 0 || kv > (1ll << 52))
                return fail(GORGO_ERR_INVALID_ARG, "kv_tokens[" + std::to_string(i) + "] must be in 0..2^52");
            eng[i] = pf;
            eng[m->R + i] = dec;
            eng[2 * (size_t)m->R + i] = (double)kv;
        }
    }
    if (!rtt_ms || !params || !scale || !outputs) return fail(GORGO_ERR_INVALID_ARG, "a required pointer is NULL");
    Plan pl;
    rc = make_plan(t, m, options, P, outputs, &pl);
    if (rc) return rc;
    for (int i = 0; i < m->R; ++i)
        if (!std::isfinite(rtt_ms[i]) || rtt_ms[i] < 0 || rtt_ms[i] > 1e9)
            return fail(GORGO_ERR_NONFINITE, "rtt_ms[" + std::to_string(i) + "] must be finite and in 0..1e9");
    for (int64_t j = 0; j < 3 * (int64_t)P; ++j)
        if (!std::isfinite(params[j]) || std::fabs(params[j]) > 1e100)
            return fail(GORGO_ERR_NONFINITE, "params[" + std::to_string(j / 3) + "][" + std::to_string(j % 3) +
                                                 "] must be finite with magnitude <= 1e100");
    for (int32_t p = 0; p < P; ++p)
        if (!std::isfinite(scale[p]) || scale[p] < 0 || scale[p] > 1e6)
            return fail(GORGO_ERR_NONFINITE, "scale[" + std::to_string(p) + "] must be finite and in 0..1e6");
    if (proxy && proxy->index_blocks >= 0 && pl.path == PATH_BLOCKS && pl.C > 0) {
        // the tables also hold what only the proxy's index still holds: more entries than the cache's, all the
        // trace's when the index never forgets
        const int64_t held = proxy->index_blocks > 0 ? std::max<int64_t>(pl.C, proxy->index_blocks) : t->unique_ids;
        const int64_t least = least_table_slots(held + t->max_distinct, t->max_distinct);
        if (pl.cap < least)
            return fail(GORGO_ERR_CAPACITY,
                        "the block tables have " + std::to_string(pl.cap) + " slots, the proxy's index needs " +
                            std::to_string(least) + ": raise options.table_factor_percent to at least " +
                            std::to_string((least * 100 + pl.C + t->max_distinct - 1) / (pl.C + t->max_distinct) + 1) +
                            " (for the workspace size and for this call)");
    }
    std::vector<double> tuner;      // constants, then ln theta0[P][3]
    int64_t steps = 0;
    if (online) {
        steps = gorgo_online_steps(pl.N, online->window, online->hop);
        if (steps < 0 || online->window > 1024) return fail(GORGO_ERR_INVALID_ARG, "window must be in 1..1024 and hop >= 1");
        if (steps > 0 && !online->z) return fail(GORGO_ERR_INVALID_ARG, "online->z is NULL");
        if (!std::isfinite(online->sigma0) || online->sigma0 < 0 || online->sigma0 > 1e3)
            return fail(GORGO_ERR_NONFINITE, "sigma0 must be finite and in 0..1e3");
        for (int k = 0; k < 3; ++k) {
            const double lo = online->lo[k], hi = online->hi[k];
            if (!std::isfinite(lo) || !std::isfinite(hi) || lo < 1e-100 || hi > 1e100 || lo > hi)
                return fail(GORGO_ERR_NONFINITE, "lo and hi must satisfy 1e-100 <= lo <= hi <= 1e100");
            for (int32_t p = 0; p < P; ++p)
                if (params[3 * (size_t)p + k] < lo || params[3 * (size_t)p + k] > hi)
                    return fail(GORGO_ERR_INVALID_ARG, "theta0[" + std::to_string(p) + "][" + std::to_string(k) +
                                                           "] is outside [lo, hi]");
        }
        tuner.assign(TUNER_CONSTS + 3 * (size_t)P, 0.0);
        for (int k = 0; k < 3; ++k) {
            tuner[k] = online->lo[k];
            tuner[3 + k] = online->hi[k];
            tuner[6 + k] = std::log(online->lo[k]);
            tuner[9 + k] = std::log(online->hi[k]);
        }
        tuner[12] = online->sigma0;
        tuner[13] = std::exp(0.4);       // 1/5 rule: sigma * exp((s - 1/5) / 2) with s = 1 ...
        tuner[14] = std::exp(-0.1);      // ... and s = 0
        for (size_t j = 0; j < 3 * (size_t)P; ++j) tuner[TUNER_CONSTS + j] = std::log(params[j]);
    }
    if (!workspace) return fail(GORGO_ERR_WORKSPACE, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(GORGO_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < pl.total)
        return fail(GORGO_ERR_WORKSPACE, "workspace has " + std::to_string(workspace_bytes) + " bytes, needs " +
                                             std::to_string(pl.total));
    rc = upload_trace(t);
    if (rc) return rc;

    char* ws = static_cast<char*>(workspace);
    double* d_rtt = reinterpret_cast<double*>(ws + pl.off_small);
    double* d_params = d_rtt + pl.R;
    double* d_scale = d_params + 3 * (size_t)P;
    double* d_tuner = d_scale + P;
    uint64_t* d_seeds = reinterpret_cast<uint64_t*>(d_tuner + TUNER_CONSTS + 3 * (size_t)P);
    double* d_eng = reinterpret_cast<double*>(d_seeds + P);
    EngineLaunch el;
    if (engine) {
        // (the host vector goes away when this function returns: the copy must have been taken by then)
        if ((rc = copy_small_to_device(d_eng, eng.data(), sizeof(double) * eng.size(), hip_stream))) return rc;
        if ((rc = wait_for_copies(hip_stream))) return rc;
        el.a_pf = d_eng;
        el.a_dec = d_eng + pl.R;
        el.budget = d_eng + 2 * (size_t)pl.R;
        el.slowdown = engine->decode_slowdown;
    }
    ProxyLaunch xl;
    if (proxy) {
        const size_t cells = (size_t)proxy->epochs * pl.R;
        if ((rc = copy_small_to_device(proxy->rtt_tables, proxy->rtt_true_ms, sizeof(double) * cells, hip_stream))) return rc;
        if ((rc = wait_for_copies(hip_stream))) return rc;       // (the caller's host table may go away)
        xl.epochs = proxy->epochs;
        xl.probe_ms = proxy->probe_interval_ms;
        xl.rtt_true = proxy->rtt_tables;
        xl.rtt_est = proxy->rtt_tables + cells;
        xl.alpha = proxy->ewma_alpha;
        xl.index_blocks = proxy->index_blocks;
        xl.believed = proxy->believed_hit_blocks;
    }
    PolicyLaunch pol;
    pol.policy = policy;
    if (policy == GORGO_POLICY_RANDOM) {
        if ((rc = copy_small_to_device(d_seeds, seeds, sizeof(uint64_t) * (size_t)P, hip_stream))) return rc;
        pol.seeds = d_seeds;
    }
    if ((rc = copy_small_to_device(d_rtt, rtt_ms, sizeof(double) * pl.R, hip_stream))) return rc;
    if ((rc = copy_small_to_device(d_params, params, sizeof(double) * 3 * (size_t)P, hip_stream))) return rc;
    if ((rc = copy_small_to_device(d_scale, scale, sizeof(double) * (size_t)P, hip_stream))) return rc;
    // (the library's own stand-in weights go away when its entry point returns: every copy must have been taken by then)
    if (policy != 0 && (rc = wait_for_copies(hip_stream))) return rc;
    OnlineLaunch ol;
    if (online) {
        // (the host vector may go away when this function returns: the copy must have been taken by then)
        if ((rc = copy_small_to_device(d_tuner, tuner.data(), sizeof(double) * tuner.size(), hip_stream))) return rc;
        if ((rc = wait_for_copies(hip_stream))) return rc;
        ol.window = online->window;
        ol.hop = online->hop;
        ol.steps = steps;
        ol.tuner = d_tuner;
        ol.ln_theta0 = d_tuner + TUNER_CONSTS;
        ol.z = online->z;
        ol.theta_step = online->theta_step;
        ol.fitness_step = online->fitness_step;
        ol.theta_final = online->theta_final;
        ol.sigma_final = online->sigma_final;
        ol.accepted = online->accepted;
    }

    uint8_t* route = outputs->route;
    double* ttft = outputs->ttft_ms;
    if (!ttft && outputs->p95_ttft_ms) ttft = reinterpret_cast<double*>(ws + pl.off_ttft);
    double* e2e = outputs->e2e_ms;
    if (!e2e && outputs->p95_e2e_ms) e2e = reinterpret_cast<double*>(ws + pl.off_e2e);
    rc = launch_replay(t, pl, d_rtt, d_params, d_scale, route, outputs->hit_blocks, ttft, e2e, workspace, hip_stream,
                       online ? &ol : nullptr, policy != 0 ? &pol : nullptr, engine ? &el : nullptr, proxy ? &xl : nullptr,
                       sections);
    if (rc) return rc;
    if (outputs->p95_ttft_ms && (rc = launch_p95(ttft, pl.N, P, outputs->p95_ttft_ms, hip_stream))) return rc;
    if (outputs->p95_e2e_ms && (rc = launch_p95(e2e, pl.N, P, outputs->p95_e2e_ms, hip_stream))) return rc;
    return GORGO_OK;
}

}  // namespace

extern "C" {

int gorgo_eval_population(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options,
        const double* rtt_ms, const double* params,
                          const double* scale, int32_t P, const gorgo_outputs* outputs, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    clear_error();
    return evaluate(t, m, options, rtt_ms, params, scale, P, nullptr, 0, nullptr, outputs, workspace, workspace_bytes, hip_stream);
}

int gorgo_eval_population_sections(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options,
        const double* rtt_ms, const double* params,
                                   const double* scale, int32_t P, const gorgo_outputs* outputs, void* workspace,
                                   size_t workspace_bytes, void* hip_stream, uint64_t* sections) {
    clear_error();
    if (!sections) return fail(GORGO_ERR_INVALID_ARG, "sections is NULL");
    return evaluate(t, m, options, rtt_ms, params, scale, P, nullptr, 0, nullptr, outputs, workspace, workspace_bytes, hip_stream,
                    nullptr, nullptr, reinterpret_cast<unsigned long long*>(sections));
}

int gorgo_trace_to_device(const gorgo_trace* t) {
    clear_error();
    if (!t) return fail(GORGO_ERR_INVALID_ARG, "trace is NULL");
    return upload_trace(t);
}

int gorgo_eval_population_static(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options,
        const double* rtt_ms, const double* params,
                                 const double* scale, int32_t P, const gorgo_outputs* outputs, void* hip_stream) {
    clear_error();
    int rc = check_model(t, m);
    if (rc) return rc;
    if (!trace_is_resident(t))
        return fail(GORGO_ERR_INVALID_ARG, "the trace is not resident on the current device: call gorgo_trace_to_device "
                                           "(which allocates) once beforehand");
    Plan pl;
    if ((rc = make_plan(t, m, options, P, outputs, &pl))) return rc;
    void* scratch = nullptr;
    size_t have = 0;
    if ((rc = static_scratch(&scratch, &have))) return rc;
    if (pl.total > have)
        return fail(GORGO_ERR_WORKSPACE, "this evaluation needs " + std::to_string(pl.total) + " bytes of workspace, the "
                                         "library's static scratch holds " + std::to_string(have) +
                                         " (GORGO_STATIC_SCRATCH_BYTES): use gorgo_eval_population with a caller workspace");
    set_event_marks(false);       // no event is created or recorded on this path
    rc = evaluate(t, m, options, rtt_ms, params, scale, P, nullptr, 0, nullptr, outputs, scratch, have, hip_stream);
    set_event_marks(true);
    return rc;
}

int64_t gorgo_online_steps(int64_t N, int32_t window, int32_t hop) {
    if (N < 0 || window < 1 || hop < 1) return -1;
    return N >= window ? (N - window) / hop + 1 : 0;
}

int gorgo_eval_online(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options,
        const double* rtt_ms, const double* theta0,
                      const double* scale, int32_t P, const gorgo_online* online, const gorgo_outputs* outputs,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
    clear_error();
    if (!online) return fail(GORGO_ERR_INVALID_ARG, "online is NULL");
    return evaluate(t, m, options, rtt_ms, theta0, scale, P, online, 0, nullptr, outputs, workspace, workspace_bytes, hip_stream);
}

int gorgo_eval_policy(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options,
        const double* rtt_ms, int32_t policy,
                      const uint64_t* seeds, const double* scale, int32_t P, const gorgo_outputs* outputs,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
    clear_error();
    if (policy != GORGO_POLICY_LEAST_REQUEST && policy != GORGO_POLICY_SESSION_AFFINITY && policy != GORGO_POLICY_RANDOM)
        return fail(GORGO_ERR_INVALID_ARG, "policy must be least-request (1), session-affinity (2) or random (3); "
                                           "prefix-cache and least-load are gorgo_eval_population with weights "
                                           "(0,1,0) and (0,0,1)");
    if (policy == GORGO_POLICY_RANDOM && !seeds) return fail(GORGO_ERR_INVALID_ARG, "seeds is NULL");
    if (P < 1 || P > (1 << 20)) return fail(GORGO_ERR_INVALID_ARG, "P must be in 1..2^20");
    const std::vector<double> zero(3 * (size_t)P, 0.0);       // the weights play no part
    return evaluate(t, m, options, rtt_ms, zero.data(), scale, P, nullptr, policy, seeds, outputs, workspace, workspace_bytes,
                    hip_stream);
}

int gorgo_eval_engine(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options,
        const gorgo_engine* engine, const double* rtt_ms,
                      int32_t policy, const double* params, const uint64_t* seeds, const gorgo_online* online,
                      const double* scale, int32_t P, const gorgo_outputs* outputs, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
    clear_error();
    if (!engine) return fail(GORGO_ERR_INVALID_ARG, "engine is NULL");
    if (policy < GORGO_POLICY_COST_MODEL || policy > GORGO_POLICY_RANDOM)
        return fail(GORGO_ERR_INVALID_ARG, "policy must be 0 (cost model) .. 3 (random)");
    if (policy == GORGO_POLICY_COST_MODEL)
        return evaluate(t, m, options, rtt_ms, params, scale, P, online, 0, nullptr, outputs, workspace, workspace_bytes,
                        hip_stream, engine);
    if (online) return fail(GORGO_ERR_INVALID_ARG, "the online tuner tunes the cost model: policy must be 0");
    if (policy == GORGO_POLICY_RANDOM && !seeds) return fail(GORGO_ERR_INVALID_ARG, "seeds is NULL");
    if (P < 1 || P > (1 << 20)) return fail(GORGO_ERR_INVALID_ARG, "P must be in 1..2^20");
    const std::vector<double> zero(3 * (size_t)P, 0.0);       // the weights play no part
    return evaluate(t, m, options, rtt_ms, zero.data(), scale, P, nullptr, policy, seeds, outputs, workspace, workspace_bytes,
                    hip_stream, engine);
}

int gorgo_eval_proxy(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options,
        const gorgo_proxy* proxy, const gorgo_engine* engine,
                     const double* params, const gorgo_online* online, const double* scale, int32_t P,
                     const gorgo_outputs* outputs, void* workspace, size_t workspace_bytes, void* hip_stream) {
    clear_error();
    if (!proxy) return fail(GORGO_ERR_INVALID_ARG, "proxy is NULL");
    if (!m) return fail(GORGO_ERR_INVALID_ARG, "model is NULL");
    return evaluate(t, m, options, proxy->rtt_true_ms, params, scale, P, online, 0, nullptr, outputs, workspace, workspace_bytes,
                    hip_stream, engine, proxy);
}

int gorgo_last_eval_kernel_ms(double* fill_ms, double* replay_ms, double* select_ms) {
    clear_error();
    return last_eval_kernel_ms(fill_ms, replay_ms, select_ms);
}

int gorgo_es_workspace_bytes(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, int32_t P,
                             size_t* bytes) {
    clear_error();
    if (!bytes) return fail(GORGO_ERR_INVALID_ARG, "bytes is NULL");
    int rc = check_model(t, m);
    if (rc) return rc;
    gorgo_outputs o;
    std::memset(&o, 0, sizeof o);
    o.p95_ttft_ms = reinterpret_cast<double*>(256);   // only which outputs are wanted matters for sizing
    Plan pl;
    rc = make_plan(t, m, options, P, &o, &pl);
    if (rc) return rc;
    *bytes = pl.total + up256(sizeof(double) * (size_t)P);
    return GORGO_OK;
}

int gorgo_es_step(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options,
        const double* rtt_ms, double scale, int32_t P,
                  gorgo_es_state* inout, double* params_out, double* fitness_out, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
    clear_error();
    if (!inout) return fail(GORGO_ERR_INVALID_ARG, "state is NULL");
    size_t need = 0;
    int rc = gorgo_es_workspace_bytes(t, m, options, P, &need);
    if (rc) return rc;
    if (!workspace) return fail(GORGO_ERR_WORKSPACE, "workspace is NULL");
    if (workspace_bytes < need)
        return fail(GORGO_ERR_WORKSPACE, "workspace has " + std::to_string(workspace_bytes) + " bytes, needs " +
                                             std::to_string(need));
    std::vector<double> z((size_t)P * 3), params((size_t)P * 3), fit((size_t)P), sc((size_t)P, scale);
    if ((rc = gorgo_es_sample(inout->seed, inout->generation, P, z.data()))) return rc;
    if ((rc = gorgo_es_propose(inout, z.data(), P, params.data()))) return rc;
    const size_t fit_bytes = up256(sizeof(double) * (size_t)P);
    double* d_fit = reinterpret_cast<double*>(static_cast<char*>(workspace) + (need - fit_bytes));
    gorgo_outputs o;
    std::memset(&o, 0, sizeof o);
    o.p95_ttft_ms = d_fit;
    rc = gorgo_eval_population(t, m, options, rtt_ms, params.data(), sc.data(), P, &o, workspace, need - fit_bytes, hip_stream);
    if (rc) return rc;
    if ((rc = copy_small_to_host_sync(fit.data(), d_fit, sizeof(double) * (size_t)P, hip_stream))) return rc;
    if ((rc = gorgo_es_update(params.data(), fit.data(), P, inout))) return rc;
    if (params_out) std::memcpy(params_out, params.data(), sizeof(double) * params.size());
    if (fitness_out) std::memcpy(fitness_out, fit.data(), sizeof(double) * fit.size());
    return GORGO_OK;
}

}  // extern "C"

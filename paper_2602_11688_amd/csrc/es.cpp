// Host side of the evolution-strategy tuner (Sec. 2.3 "GORGO Proxy Design"): counter-based normal draws,
// log-space mutation with clipping, rank-based parent update and the 1/5 step-size rule.
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

#include "internal.h"

namespace {

// Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
// SC'11): a keyed bijection of a 128-bit counter built from two 32x32->64 multiplications per round.
void philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4]) {
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;   // Weyl sequence: golden ratio
            k1 += 0xBB67AE85u;   // sqrt(3) - 1
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// 52 random bits -> uniform in the open interval (0, 1)
double open_unit(uint32_t hi, uint32_t lo) {
    uint64_t bits = ((uint64_t)hi << 20) | (lo >> 12);
    return ((double)bits + 0.5) * (1.0 / 4503599627370496.0);
}

bool finite_pos(double x) { return std::isfinite(x) && x > 0.0; }

int check_state(const gorgo_es_state* s) {
    if (!s) return gorgo::fail(GORGO_ERR_INVALID_ARG, "state is NULL");
    for (int k = 0; k < 3; ++k) {
        if (!finite_pos(s->theta[k]) || !finite_pos(s->lo[k]) || !finite_pos(s->hi[k]))
            return gorgo::fail(GORGO_ERR_NONFINITE, "theta, lo and hi must be finite and > 0");
        if (s->lo[k] > s->hi[k]) return gorgo::fail(GORGO_ERR_INVALID_ARG, "lo > hi");
    }
    if (!std::isfinite(s->sigma) || s->sigma < 0.0) return gorgo::fail(GORGO_ERR_NONFINITE, "sigma must be finite and >= 0");
    return GORGO_OK;
}

}  // namespace

extern "C" {

// Exposed for known-answer tests of the generator.
void gorgo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    philox4x32_10(ctr, key, out);
}

int gorgo_es_init(gorgo_es_state* s, uint64_t seed) {
    gorgo::clear_error();
    if (!s) return gorgo::fail(GORGO_ERR_INVALID_ARG, "state is NULL");
    const double theta[3] = {0.5, 1.0, 0.1}, lo[3] = {0.05, 1.0, 0.05}, hi[3] = {2.0, 1.0, 0.5};
    for (int k = 0; k < 3; ++k) {
        s->theta[k] = theta[k];
        s->lo[k] = lo[k];
        s->hi[k] = hi[k];
        s->best_theta[k] = theta[k];
    }
    s->sigma = 0.5;
    s->seed = seed;
    s->generation = 0;
    s->best_fitness = std::numeric_limits<double>::infinity();
    return GORGO_OK;
}

int gorgo_es_sample(uint64_t seed, int64_t generation, int32_t P, double* z) {
    gorgo::clear_error();
    if (P < 1 || !z) return gorgo::fail(GORGO_ERR_INVALID_ARG, "P < 1 or z is NULL");
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int32_t p = 0; p < P; ++p) {
        for (uint32_t k = 0; k < 3; ++k) {
            const uint32_t ctr[4] = {(uint32_t)generation, (uint32_t)((uint64_t)generation >> 32), (uint32_t)p, k};
            uint32_t x[4];
            philox4x32_10(ctr, key, x);
            double u1 = open_unit(x[0], x[1]), u2 = open_unit(x[2], x[3]);
            z[3 * (size_t)p + k] = std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586476925 * u2);
        }
    }
    return GORGO_OK;
}

int gorgo_es_propose(const gorgo_es_state* s, const double* z, int32_t P, double* params) {
    gorgo::clear_error();
    int rc = check_state(s);
    if (rc) return rc;
    if (P < 1 || !z || !params) return gorgo::fail(GORGO_ERR_INVALID_ARG, "P < 1 or a NULL array");
    for (int k = 0; k < 3; ++k) params[k] = s->theta[k];
    for (int32_t p = 1; p < P; ++p) {
        for (int k = 0; k < 3; ++k) {
            double zk = z[3 * (size_t)p + k];
            if (!std::isfinite(zk)) return gorgo::fail(GORGO_ERR_NONFINITE, "z is not finite");
            double x = std::exp(std::log(s->theta[k]) + s->sigma * zk);
            params[3 * (size_t)p + k] = std::min(std::max(x, s->lo[k]), s->hi[k]);
        }
    }
    return GORGO_OK;
}

int gorgo_es_update(const double* params, const double* fitness, int32_t P, gorgo_es_state* st) {
    gorgo::clear_error();
    int rc = check_state(st);
    if (rc) return rc;
    if (P < 1 || !params || !fitness) return gorgo::fail(GORGO_ERR_INVALID_ARG, "P < 1 or a NULL array");
    for (int32_t p = 0; p < P; ++p) {
        if (std::isnan(fitness[p])) return gorgo::fail(GORGO_ERR_NONFINITE, "fitness is NaN");
        for (int k = 0; k < 3; ++k)
            if (!finite_pos(params[3 * (size_t)p + k]))
                return gorgo::fail(GORGO_ERR_NONFINITE, "params must be finite and > 0");
    }
    std::vector<int32_t> order((size_t)P);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return fitness[a] < fitness[b]; });
    const int32_t mu = std::max(1, P / 4);
    double nt[3];
    if (mu == 1) {
        for (int k = 0; k < 3; ++k) nt[k] = params[3 * (size_t)order[0] + k];
    } else {
        for (int k = 0; k < 3; ++k) {
            double acc = 0.0;
            for (int32_t j = 0; j < mu; ++j) acc += std::log(params[3 * (size_t)order[(size_t)j] + k]);
            nt[k] = std::exp(acc / (double)mu);
        }
    }
    int32_t succ = 0;
    for (int32_t p = 1; p < P; ++p)
        if (fitness[p] < fitness[0]) ++succ;
    const double s = P > 1 ? (double)succ / (double)(P - 1) : 0.0;
    for (int k = 0; k < 3; ++k) st->theta[k] = std::min(std::max(nt[k], st->lo[k]), st->hi[k]);
    st->sigma = st->sigma * std::exp((s - 0.2) / 2.0);
    const int32_t b = order[0];
    if (fitness[b] < st->best_fitness) {
        st->best_fitness = fitness[b];
        for (int k = 0; k < 3; ++k) st->best_theta[k] = params[3 * (size_t)b + k];
    }
    st->generation += 1;
    return GORGO_OK;
}

}  // extern "C"

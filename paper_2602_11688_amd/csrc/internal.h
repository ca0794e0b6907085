// Internal declarations shared by the host-side translation units of libgorgo.
#pragma once
#include <cstdint>
#include <cstddef>
#include <string>
#include <vector>

#include "gorgo.h"

namespace gorgo {

// thread-local error text behind gorgo_last_error()
int fail(int code, const std::string& msg);
void clear_error();

// One segment of a request's block list: segment id and the number of the request's blocks up to and
// including this segment.
struct SegRef {
    int32_t id;       // in the loaded trace: the row slot the segment occupies while it is referenced
    int32_t end;      // | SEG_FRESH where this is the segment's first reference (its row slot starts over there)
};
constexpr int32_t SEG_FRESH = 1 << 30;
constexpr int32_t SEG_END_MASK = 0xFFFF;     // (a request has fewer than 2^16 blocks)

// Device-resident copy of a trace (filled lazily by the first evaluation).
struct DeviceTrace {
    int device = -1;
    void* base = nullptr;          // one allocation holding every array below
    const int64_t* ts = nullptr;   // [N]
    const int32_t* in_len = nullptr;
    const int32_t* out_len = nullptr;
    const int64_t* blk_off = nullptr;   // [N+1]
    const uint32_t* key = nullptr;      // [total] dense block key (1-based)
    const uint8_t* first = nullptr;     // [total] 1 = first occurrence of its key inside the request
    const int64_t* seg_off = nullptr;   // [N+1] (chain-consistent traces only)
    const SegRef* seg = nullptr;        // [seg_off[N]]
    const uint32_t* first_hash = nullptr;   // [N] hash of the request's first block (session-affinity policy)
};

}  // namespace gorgo

// The opaque handle of the C ABI.
struct gorgo_trace {
    int64_t N = 0;
    int32_t block_tokens = 0;
    std::vector<int64_t> ts;
    std::vector<int32_t> in_len, out_len;
    std::vector<int64_t> blk_off;
    std::vector<uint32_t> key;       // dense remap of hash ids: 1 + order of first appearance in the file
    std::vector<uint8_t> first;
    std::vector<uint32_t> first_hash;   // per request: high word of SplitMix64's output for its first block id
    int64_t total_blocks = 0;
    int32_t max_blocks = 0;          // largest n_r
    int32_t max_distinct = 0;        // largest number of distinct ids in one request
    int64_t unique_ids = 0;
    bool chain_consistent = true;
    std::vector<int64_t> seg_off;    // chain-consistent traces: request -> its segments
    std::vector<gorgo::SegRef> seg;
    int64_t n_segments = 0;
    int64_t n_slots = 0;             // rows a replay needs: the most segments in use at one time
    gorgo::DeviceTrace dev;
};

namespace gorgo {

// Geometry of one evaluation, computed on the host and handed to the launchers.
enum ReplayPath { PATH_AUTO = 0, PATH_BLOCKS = 1, PATH_SEGMENTS = 2 };

struct Plan {
    int32_t path = PATH_BLOCKS;      // PATH_BLOCKS: hashed block tables; PATH_SEGMENTS: dense segment rows
    int64_t nseg = 0;
    int32_t P = 0, R = 0, B = 0;
    int64_t N = 0, C = 0;
    int64_t cap = 0;                 // slots per (replay, replica) table, power of two
    int32_t block_tokens = 0;
    double a_pf = 0, a_dec = 0;
    int32_t packing = 2;             // gorgo_options::replay_packing of the call
    int32_t poll_limit = 1 << 24;    // gorgo_options::handover_poll_limit of the call
    // workspace carve-up (byte offsets from the workspace base)
    size_t off_tables = 0, off_spare = 0, off_rec = 0, off_route = 0, off_ttft = 0, off_e2e = 0, off_small = 0;
    size_t total = 0;
};

// Online tuner of one launch (device pointers; see gorgo_online in gorgo.h).
struct OnlineLaunch {
    int32_t window = 0, hop = 0;
    int64_t steps = 0;
    const double* tuner = nullptr;       // lo[3], hi[3], ln lo[3], ln hi[3], sigma0, exp(0.4), exp(-0.1)
    const double* ln_theta0 = nullptr;   // [P][3]
    const double* z = nullptr;
    double* theta_step = nullptr;
    double* fitness_step = nullptr;
    double* theta_final = nullptr;
    double* sigma_final = nullptr;
    int32_t* accepted = nullptr;
};
constexpr int TUNER_CONSTS = 16;         // doubles reserved for OnlineLaunch::tuner

// How a replay picks replicas (gorgo_policy in gorgo.h) and, for the random policy, the seeds of the replays.
struct PolicyLaunch {
    int32_t policy = 0;
    const uint64_t* seeds = nullptr;     // device [P]
};

// Engine model of a replica of one launch (device pointers; see gorgo_engine in gorgo.h).
struct EngineLaunch {
    const double* a_pf = nullptr;        // [R]
    const double* a_dec = nullptr;       // [R]
    const double* budget = nullptr;      // [R] KV tokens as doubles, 0 = none
    double slowdown = 0.0;
};

// Imperfect proxy knowledge of one launch (device pointers; see gorgo_proxy in gorgo.h).
struct ProxyLaunch {
    int32_t epochs = 0, probe_ms = 0;
    const double* rtt_true = nullptr;    // [epochs][R]
    double* rtt_est = nullptr;           // [epochs][R], written by the launch before the replay
    double alpha = 1.0;
    int64_t index_blocks = -1;
    uint16_t* believed = nullptr;        // [P][N], nullable
};

// kernels.hip
bool pack_replays(const Plan& pl, int64_t rows);     // rows of one replay: its segments + 2
int launch_replay(const gorgo_trace* t, const Plan& pl, const double* d_rtt, const double* d_params,
                  const double* d_scale, uint8_t* route, uint16_t* hit, double* ttft, double* e2e,
                  void* workspace, void* stream, const OnlineLaunch* online = nullptr,
                  const PolicyLaunch* policy = nullptr, const EngineLaunch* engine = nullptr,
                  const ProxyLaunch* proxy = nullptr, unsigned long long* sections = nullptr);
int launch_p95(const double* x, int64_t N, int32_t P, double* out, void* stream);
int last_eval_kernel_ms(double* fill_ms, double* replay_ms, double* select_ms);
int upload_trace(const gorgo_trace* t);
bool trace_is_resident(const gorgo_trace* t);          // on the current device
int static_scratch(void** ptr, size_t* bytes);         // device address and size of the library's static scratch array
void set_event_marks(bool on);                         // whether this thread's evaluations record timing events
void release_device_trace(gorgo_trace* t);
int copy_small_to_device(void* dst, const void* src, size_t bytes, void* stream);
int wait_for_copies(void* stream);
int copy_small_to_host_sync(void* dst, const void* src, size_t bytes, void* stream);

}  // namespace gorgo

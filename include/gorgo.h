/* gorgo.h -- C ABI of the batched routing-fitness evaluator (MI355X / gfx950).
 *
 * The library replays a Mooncake-style request trace under a whole population of cost-model weight
 * vectors at once.  For every request, every candidate scores every replica with the three TTFT terms of
 * the paper's cost model (Eq. 1-3: weighted RTT + prefill cost of the uncached suffix + weighted queueing
 * term from proxy-recorded load), routes to the replica of minimum score, updates that replica's cache and
 * queue state, and the replay is reduced to p95 TTFT / p95 E2E -- the objective of the tuner of Sec. 2.3.
 *
 * Conventions
 *   - every function returns an int: GORGO_OK (0) or a negative gorgo_status; nothing throws, aborts or
 *     prints.  gorgo_last_error() gives a human-readable message for the last failure on this thread.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory of the current
 *     device.  All arrays are caller-owned; handles (gorgo_trace*) are library-owned and released with the
 *     matching free function.
 *   - all argument validation happens before anything is enqueued: an error return means that no output
 *     byte was written and no kernel was launched.
 *   - no routine falls back to the CPU: evaluation entry points fail with GORGO_ERR_DEVICE when no GPU is
 *     usable.
 */
#ifndef GORGO_H
#define GORGO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gorgo_status {
    GORGO_OK = 0,
    GORGO_ERR_INVALID_ARG = -1, /* null pointer, size out of range, model limits exceeded                */
    GORGO_ERR_IO = -2,          /* file cannot be opened / read                                          */
    GORGO_ERR_PARSE = -3,       /* malformed trace record                                                */
    GORGO_ERR_UNSORTED = -4,    /* timestamps decrease                                                   */
    GORGO_ERR_CAPACITY = -5,    /* a request has more distinct blocks than the bounded cache can hold    */
    GORGO_ERR_NONFINITE = -6,   /* NaN / Inf / out-of-range value among weights, RTTs, scales, constants */
    GORGO_ERR_WORKSPACE = -7,   /* caller workspace too small or misaligned                              */
    GORGO_ERR_OOM = -8,         /* host or device allocation failed                                      */
    GORGO_ERR_DEVICE = -9       /* HIP error or no device                                                */
} gorgo_status;

/* Message for the most recent failure on the calling thread ("" if none).  Library-owned, valid until the
 * next library call on this thread. */
const char* gorgo_last_error(void);

/* ------------------------------------------------------------------------------------------------ trace
 * A trace is the replay input of Sec. 3 ("Dataset"): per-request timestamps that can be scaled linearly,
 * request metadata, and one integer hash id per fixed-size prompt block (Mooncake FAST'25 layout).  It is
 * immutable after load and can be shared by any number of evaluations. */
typedef struct gorgo_trace gorgo_trace;

/* Parse a JSON-lines file (host path).  One object per line with integer members "timestamp" (ms),
 * "input_length", "output_length" (tokens) and "hash_ids" (array of integers, one per block of
 * `block_tokens` tokens); other members are ignored.  Timestamps must be non-decreasing (equal timestamps
 * keep file order).  On success *out receives a new handle. */
int gorgo_load_trace(const char* jsonl_path, int32_t block_tokens, gorgo_trace** out);

/* Same, from host arrays (copied; the caller keeps its arrays).  blk_off has N+1 entries, blk_off[0] = 0,
 * request r owns hash_ids[blk_off[r] .. blk_off[r+1]).  Limits: 0 <= N < 2^31-1, at most 65535 blocks per
 * request, lengths >= 0. */
int gorgo_load_trace_arrays(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len,
                            const int64_t* blk_off, const int64_t* hash_ids, int32_t block_tokens,
                            gorgo_trace** out);

/* Trace statistics (each out pointer may be NULL): request count, total blocks, largest block count of one
 * request, number of distinct hash ids, and whether the trace is chain-consistent (every id always appears
 * at one position with one predecessor, never twice in a request -- true for prefix hashes). */
int gorgo_trace_info(const gorgo_trace* t, int64_t* N, int64_t* total_blocks, int32_t* max_blocks,
                     int64_t* unique_ids, int32_t* chain_consistent);

/* Releases host and device storage of the handle (NULL is allowed). */
void gorgo_free_trace(gorgo_trace* t);

/* ------------------------------------------------------------------------------------------------ model
 * The replica side.  The paper leaves the replica service model open (Sec. 2.1-2.2); this library fixes a
 * linear one: each replica has `batch` service slots, a request takes the earliest-free slot (lowest index
 * on ties), prefill costs prefill_ms_per_token per uncached token, decode costs decode_ms_per_token per
 * output token, and every message between proxy and replica takes half the replica's RTT.  Each replica
 * caches blocks with least-recently-used eviction at block granularity (cache_blocks = 0: unbounded).
 * Limits: 1 <= R <= 64, 1 <= batch <= 64, R * batch <= 1024. */
typedef struct gorgo_model {
    int32_t R;             /* replicas                                        */
    int32_t batch;         /* concurrent service slots per replica            */
    int32_t block_tokens;  /* must equal the trace's                          */
    int32_t _pad;          /* set to 0                                        */
    int64_t cache_blocks;  /* per-replica cache capacity in blocks, 0 = unbounded */
    double prefill_ms_per_token;
    double decode_ms_per_token;
} gorgo_model;

/* How an evaluation is carried out.  None of it changes a result; all of it is per call: every entry point that
 * evaluates, sizes a workspace or answers a question about an evaluation takes a `const gorgo_options*`, and NULL
 * stands for the defaults (the library keeps no settings between calls).  gorgo_options_default fills in the
 * defaults; out-of-range values make the call fail with GORGO_ERR_INVALID_ARG.
 *   replay_path: formulation of the cache state.  0 = automatic (default), 1 = hashed block tables (any trace),
 *     2 = dense segment rows (chain-consistent traces only; the call fails otherwise).  Both compute identical
 *     results; they differ in workspace size and speed.  Automatic picks segment rows when the trace is
 *     chain-consistent and its requests average at most 16 segments.  Size the workspace with the same options
 *     as the evaluation.
 *   replay_packing: with at most 32 replicas, at most 16 slots per replica and an even number of replays,
 *     gorgo_eval_population and gorgo_es_step can run two replays per pair of wavefronts of the segment-row kernel
 *     (a replay keeps one lane per replica, so half of a 64-lane wavefront idles otherwise).  A replay is a serial
 *     chain, so this only pays when the replays would not all be resident on the GPU at once (more than about
 *     1,024 of them) but the pairs would: 2 (default) packs exactly then, 1 whenever the shape allows, 0 never.
 *   handover_poll_limit: how many times a wavefront of the packed segment-row replay polls for its partner's
 *     word before the replay is given up (default 2^24, about a second; a replay that is given up ends at once,
 *     every latency of it becomes NaN, so does its p95, and gorgo_es_step fails with GORGO_ERR_NONFINITE).  It
 *     never happens unless the library is wrong; the setting exists so that this path can be exercised: with 0
 *     every replay whose partner is not ready at the first poll is given up.  (The unpacked kernel's wavefronts
 *     meet at workgroup barriers and do not poll.)
 *   table_factor_percent: the open-addressed cache tables of the block-table formulation get at least
 *     ceil(factor/100 * (cache_blocks + max blocks of a request)) slots, rounded up to a power of two
 *     (default 200, 110..1600). */
typedef struct gorgo_options {
    int32_t replay_path;
    int32_t replay_packing;
    int32_t handover_poll_limit;
    int32_t table_factor_percent;
} gorgo_options;
void gorgo_options_default(gorgo_options* options);

/* Per-replay outputs.  Every pointer is a DEVICE pointer owned by the caller, or NULL to skip that output.
 * P = number of replays, N = requests in the trace; [P][N] arrays are row-major (replay-major). */
typedef struct gorgo_outputs {
    uint8_t* route;        /* [P][N] chosen replica                                           */
    uint16_t* hit_blocks;  /* [P][N] blocks of the request found cached on the chosen replica */
    double* ttft_ms;       /* [P][N] time to first token                                      */
    double* e2e_ms;        /* [P][N] end-to-end latency                                       */
    double* p95_ttft_ms;   /* [P]    nearest-rank 95th percentile of ttft_ms[p][.]            */
    double* p95_e2e_ms;    /* [P]    nearest-rank 95th percentile of e2e_ms[p][.]             */
} gorgo_outputs;

/* Device workspace needed by gorgo_eval_population for P replays with this set of outputs (`outputs` may
 * be NULL: the size then covers any combination).  The workspace holds the per-replay cache tables, the
 * in-flight request records and stand-ins for per-request outputs that were not requested but are needed
 * by the percentile reduction. */
int gorgo_workspace_bytes(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, int32_t P, const gorgo_outputs* outputs,
                          size_t* bytes);

/* Evaluate P replays of the trace (Eq. 1-3, Sec. 2.2-2.3; one replay per candidate weight vector and time
 * scale).  Replay p uses weights params[3p..3p+2] = (w_rtt, w_prefill, w_queue) and scales every timestamp
 * by scale[p] (Sec. 3: time between requests is scaled linearly to control replica load).
 *   rtt_ms  host [R]     round-trip time proxy <-> replica, finite, 0 <= rtt <= 1e9
 *   params  host [P][3]  finite, |w| <= 1e100 (negative weights are legal)
 *   scale   host [P]     finite, 0 <= scale <= 1e6
 *   workspace            device, 256-byte aligned, at least gorgo_workspace_bytes(); contents are scratch
 *   hip_stream           hipStream_t (NULL = default stream)
 * The call copies the small host arrays, enqueues its kernels on the stream and returns without waiting
 * for them; outputs are valid once the stream has reached that point.  The first evaluation of a trace on
 * a device uploads the trace (one allocation and one synchronous copy).  Calls that share a workspace must
 * be ordered on one stream. */
int gorgo_eval_population(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, const double* rtt_ms,
                          const double* params, const double* scale, int32_t P, const gorgo_outputs* outputs,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* Uploads the trace to the current device now (one allocation, one synchronous copy) instead of at its first
 * evaluation there.  Does nothing if it is already resident on this device. */
int gorgo_trace_to_device(const gorgo_trace* t);

/* gorgo_eval_population for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid it.  Same arguments, results and errors, except that there is no workspace
 * argument: the cache rows, logs, in-flight records and the copies of the small host arrays live in an array of
 * GORGO_STATIC_SCRATCH_BYTES that is part of the library's device code (each GPU the library runs on holds it
 * until the process ends).  The call allocates nothing on the device and creates no event or stream
 * (gorgo_last_eval_kernel_ms does not cover it); the trace must already be resident on the current device
 * (gorgo_trace_to_device, or any earlier evaluation there), else GORGO_ERR_INVALID_ARG.  An evaluation whose
 * gorgo_workspace_bytes exceeds GORGO_STATIC_SCRATCH_BYTES is refused with GORGO_ERR_WORKSPACE before anything
 * is enqueued.  Every call on a GPU uses that GPU's one array: what must start clean is cleared by the call's
 * own kernels, and two such calls that overlap in time on one GPU (different streams or threads) race. */
#define GORGO_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int gorgo_eval_population_static(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, const double* rtt_ms,
                                 const double* params, const double* scale, int32_t P,
                                 const gorgo_outputs* outputs, void* hip_stream);

/* ------------------------------------------------------------------------------------------------ tuner
 * Evolution-strategy state (Sec. 2.3): parent weights theta, step size sigma, per-weight ranges, the
 * generation counter and the best candidate seen so far.  Plain data, caller-owned; serialise it to
 * checkpoint a tuning run.  A weight with lo == hi is pinned (the paper pins the prefill weight to 1). */
typedef struct gorgo_es_state {
    double theta[3];
    double sigma;
    double lo[3];
    double hi[3];
    uint64_t seed;
    int64_t generation;
    double best_fitness;   /* +inf before the first update */
    double best_theta[3];
} gorgo_es_state;

/* Paper defaults: theta = (0.5, 1, 0.1), ranges [0.05, 2] / [1, 1] / [0.05, 0.5], sigma = 0.5 (Sec. 4). */
int gorgo_es_init(gorgo_es_state* s, uint64_t seed);

/* Standard-normal draws z[P][3] (host) of one generation: a counter-based generator (Philox-4x32-10 keyed
 * by the seed, counter = (generation, candidate), Box-Muller transform), so that a generation can be
 * reproduced from (seed, generation) alone. */
int gorgo_es_sample(uint64_t seed, int64_t generation, int32_t P, double* z);

/* The generator's block function alone (for known-answer tests): out = Philox-4x32-10(counter, key). */
void gorgo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Candidates of one generation from given draws (host arrays): params[0] = theta (the parent itself),
 * params[p][k] = clip(exp(ln theta[k] + sigma * z[p][k]), lo[k], hi[k]) for p >= 1 (mutation rule of
 * Sec. 2.3).  Requires theta, lo, hi > 0. */
int gorgo_es_propose(const gorgo_es_state* s, const double* z, int32_t P, double* params);

/* Selection and step-size update from evaluated candidates (host arrays; fitness is minimised).  Rank by
 * (fitness, index); the new parent is the geometric mean of the best max(1, P/4) candidates, clipped (for
 * P < 8 this is the best candidate itself, so P = 2 is the paper's accept-if-better step); sigma is
 * multiplied by exp((s - 1/5) / 2) with s the fraction of offspring that strictly beat the parent
 * (Rechenberg's 1/5 rule); generation is incremented; the best candidate so far is recorded. */
int gorgo_es_update(const double* params, const double* fitness, int32_t P, gorgo_es_state* inout);

/* One full generation: sample, propose, evaluate all P candidates at one time scale with
 * gorgo_eval_population (fitness = p95 TTFT in ms), synchronise the stream once, update the state.
 * params_out [P][3] and fitness_out [P] are optional host arrays.  The workspace must be sized with
 * gorgo_es_workspace_bytes. */
int gorgo_es_workspace_bytes(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, int32_t P, size_t* bytes);
int gorgo_es_step(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, const double* rtt_ms, double scale, int32_t P,
                  gorgo_es_state* inout, double* params_out, double* fitness_out, void* workspace,
                  size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------- online tuner
 * The tuner as the paper runs it (Sec. 2.3 "GORGO Proxy Design"; Sec. 4 "Tuning and evaluation windows"):
 * inside ONE replay, the p95 TTFT of a rolling window of `window` requests (paper: 128) is taken every `hop`
 * requests (paper: 32), first when the first window is full.  It is the fitness of the weights then in use.
 * The first window measures the initial weights, which become the parent.  Afterwards the weights in use
 * (the offspring) replace the parent iff their fitness is strictly lower than the parent's, and sigma is
 * multiplied by exp(0.4) after a success and exp(-0.1) otherwise (the 1/5 rule of gorgo_es_update at P = 2).
 * Every step ends by proposing the next offspring from the parent by the log-space mutation of Sec. 2.3,
 *   theta[k] = clip(exp(clip(ln parent[k] + sigma * z[step][k], ln lo[k], ln hi[k])), lo[k], hi[k]),
 * used from the next request on (ln of the parent is carried along, not retaken from the clipped value; exp
 * is evaluated by a fixed sequence of additions and multiplications, so that it has the same bits on every
 * processor).  A request's TTFT enters the window when the request is dispatched: the stated service model gives
 * it at once, whereas the paper's proxy only sees a TTFT when the first token has come back, so the tuner here is
 * fed a little earlier than a live one would be (a reading of this library, see the design notes).
 * P replays run P independent tuners (different draws, initial weights or time scales).
 * Runs in either formulation of the cache state (gorgo_options.replay_path), like everything below. */
typedef struct gorgo_online {
    int32_t window;        /* 1..1024 requests per fitness window                                     */
    int32_t hop;           /* >= 1 requests between tuner steps                                        */
    double lo[3], hi[3];   /* clip range per weight, 0 < lo <= hi, finite; lo == hi pins the weight    */
    double sigma0;         /* initial step size, finite, >= 0                                          */
    const double* z;       /* DEVICE [P][steps][3] standard normal draws, steps = gorgo_online_steps() */
    /* outputs, DEVICE, caller-owned, each may be NULL */
    double* theta_step;    /* [P][steps][3] weights in use after each step                             */
    double* fitness_step;  /* [P][steps]    window p95 TTFT (ms) seen at each step                     */
    double* theta_final;   /* [P][3]        parent weights after the last step                         */
    double* sigma_final;   /* [P]                                                                      */
    int32_t* accepted;     /* [P]           offspring that replaced their parent                       */
} gorgo_online;

/* Tuner steps of a replay of N requests: (N - window) / hop + 1 if N >= window, else 0 (at the paper's 128 /
 * 32, request 672 ends step 18).  Negative on invalid arguments. */
int64_t gorgo_online_steps(int64_t N, int32_t window, int32_t hop);

/* Evaluate P replays, each with its own online tuner.  As gorgo_eval_population, except that
 * theta0 (host [P][3], each within [lo, hi]) are the weights of the first window.  Same workspace size. */
int gorgo_eval_online(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, const double* rtt_ms, const double* theta0,
                      const double* scale, int32_t P, const gorgo_online* online, const gorgo_outputs* outputs,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* -------------------------------------------------------------------------------- baseline policies
 * The routing policies that the paper compares the cost model with (Sec. 4 "Baseline policies"), replayed on
 * the same trace with the same replica model.  Two of them are the cost model itself with special weights and
 * need no entry point of their own: prefix-cache (highest prefix overlap) is gorgo_eval_population with
 * weights (0, 1, 0), and least-load restricted to what the proxy itself tracks (tokens of requests without a
 * completion event) is weights (0, 0, 1).  The others:
 *   GORGO_POLICY_LEAST_REQUEST     fewest in-flight requests (no completion event at the proxy yet), lowest
 *                                  replica index on ties
 *   GORGO_POLICY_SESSION_AFFINITY  the replica selected by a hash of the request's first block (the paper hashes
 *                                  the first 256 tokens; a trace carries one id per block): replica =
 *                                  floor(h * R / 2^32) with h the high 32 bits of the value that a SplitMix64
 *                                  generator in state `id` returns next; a request without blocks goes to replica 0
 *   GORGO_POLICY_RANDOM            replica = floor(x * R / 2^32) with x the first output word of Philox-4x32-10
 *                                  for counter (request index, 0, 0) and key seeds[p] */
typedef enum gorgo_policy {
    GORGO_POLICY_COST_MODEL = 0,   /* accepted by gorgo_eval_policy only with weights, i.e. not at all: use gorgo_eval_population */
    GORGO_POLICY_LEAST_REQUEST = 1,
    GORGO_POLICY_SESSION_AFFINITY = 2,
    GORGO_POLICY_RANDOM = 3
} gorgo_policy;

/* Evaluate P replays routed by `policy`, replay p at time scale scale[p] (and, for the random policy, with
 * seed seeds[p]; seeds is a host array [P], may be NULL for the other policies).  Everything else as
 * gorgo_eval_population, same workspace size. */
int gorgo_eval_policy(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, const double* rtt_ms, int32_t policy,
                      const uint64_t* seeds, const double* scale, int32_t P, const gorgo_outputs* outputs,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------- engine model of a replica
 * A richer replica than the linear B-slot model of gorgo_model, for the effects the paper reports but gives no
 * formulas for: continuous batching admits a request into the running batch while the batch is below its
 * maximum number of concurrent requests and the KV-cache budget allows (Sec. 2.2); when many requests decode
 * together the replica's memory saturates and inter-token latency grows, so a router can buy a low TTFT with a
 * high E2E latency by concentrating load (Sec. 5 "Exploiting Continuous Batching"); replicas may differ in
 * prefill rate, queueing behaviour and KV capacity, which the cost model does not know (Sec. 7).  Stated model:
 *   - replica i prefills at prefill_ms_per_token[i] per uncached token and decodes at decode_ms_per_token[i]
 *     per output token; the cost model of Eq. 3 keeps the single rate of gorgo_model;
 *   - a request holds input_length + output_length KV tokens from its admission until its last token;
 *   - requests are admitted in arrival order: a request is admitted at the first time s, not before its
 *     arrival at the replica nor the admission of its predecessor there, at which the requests running at s
 *     (admitted earlier, last token after s) number fewer than gorgo_model.batch and either there are none or
 *     their KV tokens plus its own do not exceed kv_tokens[i] (0 or a NULL array: no budget);
 *   - its decode takes (decode_ms_per_token[i] * output_length) * (1 + decode_slowdown * n), n = the number of
 *     requests running at its admission; the factor is fixed at admission.
 * With decode_slowdown = 0, no budget and rates equal to gorgo_model's the results equal the linear model's bit
 * for bit.  gorgo_model.decode_ms_per_token is not used. */
typedef struct gorgo_engine {
    const double* prefill_ms_per_token;   /* host [R], finite, 0..1e6          */
    const double* decode_ms_per_token;    /* host [R], finite, 0..1e6          */
    const int64_t* kv_tokens;             /* host [R], 0..2^52, or NULL        */
    double decode_slowdown;               /* finite, 0..1e3                    */
} gorgo_engine;

/* Evaluate P replays under the engine model.  What routes is chosen by `policy`:
 *   GORGO_POLICY_COST_MODEL with online == NULL: fixed weights params (host [P][3]), as gorgo_eval_population;
 *   GORGO_POLICY_COST_MODEL with online != NULL: the online tuner from weights params, as gorgo_eval_online;
 *   the other policies: as gorgo_eval_policy (params may be NULL; seeds as there; online must be NULL).
 * Everything else (outputs, workspace and its size, stream, errors) as gorgo_eval_population. */
int gorgo_eval_engine(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, const gorgo_engine* engine, const double* rtt_ms,
                      int32_t policy, const double* params, const uint64_t* seeds, const gorgo_online* online,
                      const double* scale, int32_t P, const gorgo_outputs* outputs, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------- imperfect proxy knowledge
 * What the proxy of the paper knows only approximately.  (1) Round trip times: T_network is the exponentially
 * weighted moving average of a ping's round trip time (Sec. 2.2), measured at fixed intervals on a separate probe
 * (Sec. 4, RTT figure: every 30 s).  (2) Cached prefixes: the proxy does not observe replica-side eviction, so its
 * cache index may overestimate what a replica holds (Sec. 7).  The paper gives neither the smoothing constant nor
 * the index's own forgetting rule.  Stated model:
 *   - time is cut into epochs of probe_interval_ms: the epoch of time t (= timestamp * scale) is the largest e with
 *     e * probe_interval_ms <= t, capped at epochs - 1; a request dispatched in epoch e experiences the round trip
 *     time rtt_true_ms[e][i] on replica i (half of it each way);
 *   - the proxy probes at the start of every epoch: est[0] = rtt_true_ms[0], est[e] = ewma_alpha * rtt_true_ms[e]
 *     + (1 - ewma_alpha) * est[e-1]; Eq. 3 scores with est of the request's epoch;
 *   - index_blocks >= 0: the proxy keeps an index of its own of what it dispatched to replica i (a prefix trie of
 *     dispatched requests), updated like the replica's cache (least recently used block first) but with its own
 *     capacity: index_blocks per replica (at least gorgo_model.cache_blocks), 0 = it never forgets.  Eq. 3 takes
 *     the uncached tokens of replica i from the longest prefix of the request in that index, while the replica
 *     prefills what its own cache really misses; hit_blocks stays the real count.  index_blocks = -1: the proxy
 *     sees the replicas' caches as they are.
 * With one epoch (or equal rows) and index_blocks = -1 or = cache_blocks the results equal
 * gorgo_eval_population's bit for bit.
 * In the block-table formulation the index lives in the replica's table (the same entries read against a second
 * eviction threshold), so a bounded cache's tables must also hold what only the index still holds: the call fails
 * with GORGO_ERR_CAPACITY, naming the options.table_factor_percent that is enough, when the tables of the
 * workspace are too small for index_blocks (or, with index_blocks = 0, for every id of the trace). */
typedef struct gorgo_proxy {
    int32_t epochs;               /* 1..65536 probe epochs given                                              */
    int32_t probe_interval_ms;    /* >= 1                                                                     */
    const double* rtt_true_ms;    /* host [epochs][R], finite, 0..1e9                                         */
    double ewma_alpha;            /* in (0, 1]                                                                */
    int64_t index_blocks;         /* -1, 0, or cache_blocks..2^30 (only 0 or -1 when cache_blocks is 0)       */
    double* rtt_tables;           /* DEVICE [2][epochs][R], caller-owned, written: [0] a copy of rtt_true_ms,
                                     [1] the proxy's estimates; must stay valid until the stream has run      */
    uint16_t* believed_hit_blocks;/* DEVICE [P][N] or NULL: blocks Eq. 3 took for cached on the chosen replica */
} gorgo_proxy;

/* Evaluate P replays with imperfect proxy knowledge.  engine may be NULL (linear model) or an engine model as in
 * gorgo_eval_engine; online may be NULL (fixed weights params, host [P][3]) or an online tuner as in
 * gorgo_eval_online (params are then the initial weights).  The round trip times come from proxy->rtt_true_ms.
 * Everything else (outputs, workspace and its size, stream, errors) as gorgo_eval_population. */
int gorgo_eval_proxy(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, const gorgo_proxy* proxy, const gorgo_engine* engine,
                     const double* params, const gorgo_online* online, const double* scale, int32_t P,
                     const gorgo_outputs* outputs, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------ misc
 * Device time (ms, HIP events recorded on the evaluation's stream) of the three stages of the most recent
 * gorgo_eval_population / gorgo_es_step issued by the calling thread: state initialisation, the replay
 * kernel, and the percentile selection.  Waits for that evaluation to finish.  Each pointer may be NULL. */
int gorgo_last_eval_kernel_ms(double* fill_ms, double* replay_ms, double* select_ms);

/* Measurement aid: gorgo_eval_population run by an instantiation of the segment-row kernel that reads the GPU's
 * cycle counter between the sections of its request loop and adds up, per replay and wavefront, the cycles each
 * section took (same results; slower by the clock reads, each of which also waits for the wavefront's
 * outstanding LDS accesses).  sections: DEVICE [P][3][GORGO_SECTIONS] uint64, [p][0] the cache wavefront
 * (0 waiting for the queue terms, 1 match incl. the wait for its rows, 2 log records and the next rows, 3 score,
 * minimum and announcement, 4 waiting at the second meeting point, 5 ownership, 6 stores, log and eviction,
 * 7 patch and loop; then counts, not cycles: 8 log records fetched on the spot by the eviction walk, 9 cursor
 * advances, 10 log records dropped because they own nothing, 11 ownership walks), [p][1] the queue wavefront (0 retire and publish, 1 waiting at the first meeting point,
 * 2 retiring ahead, 3 nothing, 4 waiting for the choice, 5 service and outputs, 6 batch turnover), [p][2] the
 * front-end wavefront (0 the descriptor of the request after next, 1 and 2 waiting at the two meeting points, 3 the
 * references of the request after that, loaded between the meeting points).  Needs the
 * segment formulation without packing; everything else as gorgo_eval_population. */
#define GORGO_SECTIONS 12
int gorgo_eval_population_sections(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, const double* rtt_ms,
                                   const double* params, const double* scale, int32_t P,
                                   const gorgo_outputs* outputs, void* workspace, size_t workspace_bytes,
                                   void* hip_stream, uint64_t* sections);

/* Whether gorgo_eval_population with P replays of this trace and model would pack them under these options
 * (*packed = 1) or not (0).  Asks the current device how many workgroups it holds at once. */
int gorgo_query_replay_packing(const gorgo_trace* t, const gorgo_model* m, const gorgo_options* options, int32_t P,
                               int32_t* packed);

/* Rows of cells that a replay of this trace keeps in the segment formulation (0 for a trace that is not
 * chain-consistent).  A segment only needs a row from the first to the last request that references it, which the
 * trace fixes for every candidate alike, so the loader lets segments share rows: a segment takes a row slot at its
 * first reference and hands it on after its last.  The number is the most segments in use at one time (plus none of
 * the two rows the kernel adds for its own use); it replaces the number of segments in the workspace size. */
int gorgo_query_row_slots(const gorgo_trace* t, int64_t* slots);

/* Formulation that an evaluation of this trace would use under these options (1 or 2, see gorgo_options), the number
 * of segments of the trace and the total number of (request, segment) references; the last two are 0 for a
 * trace that is not chain-consistent.  Each out pointer may be NULL. */
int gorgo_query_replay_path(const gorgo_trace* t, const gorgo_options* options, int32_t* path, int64_t* n_segments,
                            int64_t* segment_refs);

#ifdef __cplusplus
}
#endif
#endif /* GORGO_H */

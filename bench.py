#!/usr/bin/env python3
"""Benchmark of the batched routing-fitness evaluation on one MI355X.

A "step" is one generation of the tuner on the Large workload (R=32 replicas, N=1,000,000 requests,
16,000-block LRU caches, P=1,024 candidate weight vectors): sample and propose the candidates, replay the
whole trace under all of them (score, route, cache/queue update per request), reduce every replay to its
p95 TTFT, update the parent weights and step size.  The trace is resident in HBM before the timed region.
With --config 4 a step is the saturation sweep instead: one launch of 8 time scales x 128 candidates = 1,024
replays of the 200,000-request trace, reduced to their p95s (there is no tuner step in that workload).

Prints ONE JSON line: candidate-request routings per second (whole job), the replay kernel's HBM roofline
(algorithmic bytes / HIP-event kernel time against 8 TB/s) and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes_per_routing(R, n_mean, hit_mean, outputs_bytes):
    """Bytes one routing has to move in the hashed-block-set formulation with 16-byte table slots
    (8-byte key + 8-byte recency stamp), private to one replay:
      first-block probe on every replica           16 * R
      prefix match on the replica holding it       16 * (hit + 1)
      update on the chosen replica                 16 * n probe reads + 8 * hit stamp writes
                                                   + 16 * (n - hit) inserts
      eviction walk (every logged touch re-read once before its slot is given up)   16 * n
      in-flight record push + pop                  16 + 16
      per-request outputs                          outputs_bytes
    The trace itself (28 B + 5 B per block per request) is shared by all replays and is not counted."""
    n, h = n_mean, hit_mean
    return 16 * R + 16 * (h + 1) + (16 * n + 8 * h + 16 * (n - h)) + 16 * n + 32 + outputs_bytes


def algorithmic_bytes_per_routing_segments(R, segs_mean, outputs_bytes):
    """Bytes one routing has to move in the segment-row formulation (one 4-byte "last request" cell per
    (segment, replica), rows of R cells addressed by segment id), private to one replay:
      rows of the request's segments, read by every replica's lane   4 * R * s
      update of the chosen replica's cells                            4 * s
      log record of the request: written (8), linked from its predecessor on the replica (4), its owned
      suffix moved when a later request takes its segments over (2), read once by the eviction cursor (8)
      per-request outputs                                             outputs_bytes
    Queue state (service slots, the two oldest in-flight requests of a slot, load signal) lives in LDS and
    registers; deeper in-flight records (16 B each way) only exist when a slot is more than two deep and
    are not counted.  The trace itself (28 B + 8 B per segment per request) is shared by all replays and is
    not counted."""
    s = segs_mean
    return 4 * R * s + 4 * s + 22 + outputs_bytes


def kernel_source_digest():
    """Digest of the device sources; HBM counters recorded for another digest are not reported."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2602_11688_amd", "csrc")
    for name in ("device_common.h", "replay_segments.h", "replay_segments_packed.h", "kernels.hip"):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def recorded_counters(kernel, workload_key):
    """Hardware counters of one launch of `kernel` recorded under profiles/ by rocprofv3 runs of this script:
    HBM bytes (FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading for a plain 1 GiB copy) and,
    when present, the instruction counters.  None when the device sources have changed since, or the workload
    differs."""
    path = os.path.join(ROOT, "profiles", "hbm_counters.json")
    try:
        with open(path) as f:
            rec = json.load(f)
    except OSError:
        return None
    if rec.get("source_digest") != kernel_source_digest() or rec.get("kernel") != kernel or \
            rec.get("workload") != workload_key:
        return None
    return rec


def cpu_single_thread(wl, params, n_req):
    """The oracle on one thread: one replay of the first n_req requests (routings/s of one core that has the
    machine to itself, which a run on every core at once does not show)."""
    from oracle import binding as ob
    tr = wl.trace.head(n_req)
    t0 = time.perf_counter()
    ob.replay(tr, R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token, rtt_ms=wl.rtt_ms, w=params[0], scale=1.0)
    dt = time.perf_counter() - t0
    return tr.N / dt, dt, tr.N


def cpu_baseline(wl, params, n_req, threads, online=None, engine=None, proxy=None, scales=None):
    """The oracle as it stands, one replay per thread, on the first n_req requests of the workload (with its online
    tuner when `online` = (z[P, steps, 3], lo, hi, sigma0) is given; under the engine model of a replica when
    `engine` = its parameters is given)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import binding as ob
    tr = wl.trace.head(n_req)
    ob.lib()
    if proxy is not None:
        def one_proxy(p):
            return ob.replay_proxy(tr, R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks,
                                   prefill_ms_per_token=wl.prefill_ms_per_token,
                                   decode_ms_per_token=wl.decode_ms_per_token, rtt_true=proxy.rtt_true_ms,
                                   probe_ms=proxy.probe_interval_ms, alpha=proxy.ewma_alpha,
                                   index_blocks=proxy.index_blocks, w=params[p], scale=1.0).p95_ttft_ms
        t0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one_proxy, range(threads)))
        dt = time.perf_counter() - t0
        return threads * tr.N / dt, dt, tr.N
    if engine is not None:
        def one_engine(p):
            return ob.replay_engine(tr, R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks,
                                    prefill_ms_per_token=wl.prefill_ms_per_token, engine=engine, rtt_ms=wl.rtt_ms,
                                    w=params[p], scale=1.0).p95_ttft_ms
        t0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one_engine, range(threads)))
        dt = time.perf_counter() - t0
        return threads * tr.N / dt, dt, tr.N
    if online is not None:
        z, lo, hi, sigma0 = online
        steps = ob.online_steps(tr.N, 128, 32)

        def one_online(p):
            return ob.replay_online(tr, R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks,
                                    prefill_ms_per_token=wl.prefill_ms_per_token,
                                    decode_ms_per_token=wl.decode_ms_per_token, rtt_ms=wl.rtt_ms, theta0=params[p],
                                    z=z[p, :steps], lo=lo, hi=hi, sigma0=sigma0).p95_ttft_ms
        t0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one_online, range(threads)))
        dt = time.perf_counter() - t0
        return threads * tr.N / dt, dt, tr.N

    def one(p):
        return ob.replay(tr, R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks,
                         prefill_ms_per_token=wl.prefill_ms_per_token, decode_ms_per_token=wl.decode_ms_per_token,
                         rtt_ms=wl.rtt_ms, w=params[p], scale=1.0 if scales is None else float(scales[p])).p95_ttft_ms
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(one, range(threads)))
    dt = time.perf_counter() - t0
    return threads * tr.N / dt, dt, tr.N


def section_table(sec, N, P):
    """The timed instantiation's per-wavefront section budget as text: shader-clock cycles per request of each
    of the three wavefronts of a replay (mean over replays), between the marks the kernel sets, and the cache side's
    event counts.  sec = the [P, 3, 12] array of gorgo_eval_population_sections."""
    m = (sec.astype(np.float64) / max(N, 1)).mean(axis=0)
    lines = []
    cache = {0: "waiting at barrier A (queue terms)", 1: "prefix match (waits for the rows)", 2: "log records, next rows, uncached tokens",
             3: "score, minimum, announcement", 5: "ownership", 4: "waiting at barrier B", 6: "cell, log and link stores",
             7: "eviction, patching the next rows, loop"}
    queue = {10: "lane broadcasts, retiring what is due", 0: "publishing the queue terms", 1: "waiting at barrier A",
             2: "retiring ahead for the next request", 3: "(reading the clock once)", 4: "waiting at barrier B", 8: "reading the choice",
             9: "service: slot, completion time", 5: "outputs, tuner, loop", 6: "batch turnover"}
    front = {0: "descriptor of request r+2", 1: "waiting at barrier A", 3: "references of request r+3 (loads)", 2: "waiting at barrier B"}
    lines.append(f"shader-clock cycles per request (s_memtime), mean over {P} replays")
    k = 1.0
    lines.append("cache wavefront (lane = replica):")
    for i, name in cache.items():
        lines.append(f"  {name:44s} {m[0, i] * k:8.1f}")
    lines.append(f"  {'total':44s} {m[0, :8].sum() * k:8.1f}")
    lines.append(f"  events per request: on-the-spot record fetches {m[0, 8]:.3f}, cursor advances {m[0, 9]:.3f}, "
                 f"dead records dropped {m[0, 10]:.3f}, ownership walks {m[0, 11]:.3f}")
    lines.append("queue wavefront (lane = service slot):")
    for i, name in queue.items():
        lines.append(f"  {name:44s} {m[1, i] * k:8.1f}")
    lines.append(f"  {'total':44s} {sum(m[1, i] for i in queue) * k:8.1f}")
    lines.append("front-end wavefront (lane = segment reference):")
    for i, name in front.items():
        lines.append(f"  {name:44s} {m[2, i] * k:8.1f}")
    lines.append(f"  {'total':44s} {sum(m[2, i] for i in front) * k:8.1f}")
    return "\n".join(lines)


def compare_policies(g, torch, tr, model, wl, tuned, N, engine=None):
    """The paper's comparison of routing policies in synthetic form: one replay of the trace per policy, same replica
    model (the engine model when `engine` is given), time scale 1.  TTFT / E2E in ms; block_hit = cached blocks /
    requested blocks."""
    nb = torch.from_numpy(np.diff(wl.trace.blk_off).astype(np.float64)).to("cuda:0")

    def stats(res, p):
        t = res.ttft_ms[p]
        return {"ttft_p50": t.median().item(), "ttft_p95": res.p95_ttft_ms[p].item(), "ttft_mean": t.mean().item(),
                "e2e_p95": res.p95_e2e_ms[p].item(),
                "block_hit": (res.hit_blocks[p].to(torch.float64).sum() / nb.sum()).item()}
    table = {}
    weights = {"cost model, initial weights (0.5, 1, 0.1)": [0.5, 1.0, 0.1], "cost model, tuner's best weights": tuned,
               "prefix-cache = weights (0, 1, 0)": [0.0, 1.0, 0.0], "least-load (proxy tokens) = weights (0, 0, 1)": [0.0, 0.0, 1.0],
               "nearest replica = weights (1, 0, 0)": [1.0, 0.0, 0.0]}
    par = np.array(list(weights.values()), np.float64)
    res = g.eval_population(tr, model, wl.rtt_ms, par, 1.0) if engine is None else \
        g.eval_engine(tr, model, engine, wl.rtt_ms, 1.0, params=par)
    torch.cuda.synchronize()
    for i, k in enumerate(weights):
        table[k] = stats(res, i)
    del res
    for pol in ("least-request", "session-affinity", "random"):
        seeds = np.array([7], np.uint64)
        res = g.eval_policy(tr, model, wl.rtt_ms, pol, [1.0], seeds=seeds) if engine is None else \
            g.eval_engine(tr, model, engine, wl.rtt_ms, [1.0], policy=pol, seeds=seeds)
        torch.cuda.synchronize()
        table[pol] = stats(res, 0)
        del res
    for k, v in table.items():
        print(f"[bench] {k:46s} ttft p50 {v['ttft_p50']:12.1f} p95 {v['ttft_p95']:12.1f} mean {v['ttft_mean']:12.1f} "
              f"e2e p95 {v['e2e_p95']:12.1f} block hit {v['block_hit']:.3f}", file=sys.stderr, flush=True)
    return table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=5, help="workload index (5 = Large, the one the metric is quoted on)")
    ap.add_argument("--requests", type=int, default=None, help="truncate the trace (experiments only)")
    ap.add_argument("--population", type=int, default=None, help="override P (experiments only)")
    ap.add_argument("--cpu-sample-requests", type=int, default=600000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy before the timed region (reference for HBM counters)")
    ap.add_argument("--path", type=int, default=0, help="0 auto, 1 hashed block tables, 2 segment rows (experiments only)")
    ap.add_argument("--sections", action="store_true",
                    help="after the timed region, launch the kernel's timed instantiation once (it reads the clock at marks "
                         "in each of its three wavefronts) and print the per-section cycle budget to stderr")
    ap.add_argument("--policies", action="store_true",
                    help="also replay the trace once under each routing policy of the paper's comparison (cost model with "
                         "the tuner's weights, its special cases, least-request, session affinity, random) and report "
                         "their latencies under \"policies\" (untimed)")
    ap.add_argument("--online", action="store_true",
                    help="instead of one ES generation per step: one pass of P online tuners (window 128, hop 32) "
                         "over the trace per step -- the tuner as the paper runs it, not the headline metric")
    ap.add_argument("--engine", action="store_true",
                    help="replicas follow the engine model (continuous batching with a KV-token budget, decode slow-down, "
                         "uneven rates: synth.tracegen.engine_recipe) instead of the linear one; a step is still one ES "
                         "generation -- not the headline metric")
    ap.add_argument("--proxy", action="store_true",
                    help="the proxy knows the replicas imperfectly (true round trip times wander per 30 s probe epoch and are "
                         "scored through their moving average; its own cache index holds twice what a replica's cache holds: synth.tracegen.rtt_walk); "
                         "a step is still one ES generation -- not the headline metric")
    args = ap.parse_args()
    if args.engine + args.online + args.proxy > 1:
        sys.exit("bench.py: --engine, --online and --proxy are separate runs")
    sweep = args.config == 4          # the saturation sweep: a population evaluation over (scale, candidate) pairs, no tuner
    if sweep and (args.engine or args.online or args.proxy):
        sys.exit("bench.py: the saturation sweep (--config 4) is timed with the linear replica model and fixed weights")
    if args.gpus != 1:
        sys.exit("bench.py: this library evaluates on ONE GPU (replays are independent and would shard by candidate; "
                 "no multi-GPU path is built) -- run with --gpus 1")

    import torch
    import paper_2602_11688_amd as g
    from synth import tracegen as tg

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    g.set_replay_path(args.path)
    t_setup = time.perf_counter()
    wl = tg.config(args.config, args.requests)
    es_cfg = wl.es if wl.es else dict(tg.ES_DEFAULTS, P=wl.P, seed=tg.MASTER_SEED + args.config)
    P = args.population or es_cfg["P"]
    tr = g.Trace.from_arrays(wl.trace.ts_ms, wl.trace.in_len, wl.trace.out_len, wl.trace.blk_off, wl.trace.hash_ids)
    N = tr.N
    model = g.Model(wl.R, wl.batch, wl.cache_blocks, wl.prefill_ms_per_token, wl.decode_ms_per_token)
    state = g.es_init(es_cfg["seed"])
    ws_bytes = g.workspace_bytes(tr, model, P) if args.online or args.engine or args.proxy or sweep else g.es_workspace_bytes(tr, model, P)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda:0")
    print(f"[bench] workload {wl.name}: R={wl.R} N={N} P={P} C={wl.cache_blocks} mean blocks/request "
          f"{np.diff(wl.trace.blk_off).mean():.1f}; workspace {ws.numel() / 2**30:.1f} GiB; setup "
          f"{time.perf_counter() - t_setup:.1f}s", file=sys.stderr, flush=True)

    if args.online:
        steps_on = g.online_steps(N, 128, 32)
        z_on = torch.from_numpy(g.es_sample(es_cfg["seed"], 0, P * steps_on).reshape(P, steps_on, 3)).to("cuda:0")
        theta0 = np.tile(np.array(state.theta[:]), (P, 1))

    if args.engine:
        recipe = tg.engine_recipe(wl)
        engine = g.Engine(recipe["prefill_ms_per_token"], recipe["decode_ms_per_token"], recipe["kv_tokens"],
                          recipe["slowdown"])

    if args.proxy:
        epochs = int(float(wl.trace.ts_ms[-1]) // 30000) + 1 if N else 1
        proxy = g.Proxy(tg.rtt_walk(wl, epochs), 30000, 0.3, 2 * wl.cache_blocks)

    sweep_par = np.ascontiguousarray(wl.params[:P]) if sweep else None
    sweep_scale = np.ascontiguousarray(wl.scale[:P]) if sweep else None

    def generation():
        if sweep:
            res = g.eval_population(tr, model, wl.rtt_ms, sweep_par, sweep_scale, per_request=False, workspace=ws)
            fit = res.p95_ttft_ms.cpu().numpy()
            return sweep_par, fit, g.last_eval_kernel_ms()
        if args.proxy:
            par = g.es_propose(state, g.es_sample(state.seed, state.generation, P))
            res = g.eval_proxy(tr, model, proxy, par, 1.0, per_request=False, workspace=ws)
            fit = res.p95_ttft_ms.cpu().numpy()
            g.es_update(state, par, fit)
            return par, fit, g.last_eval_kernel_ms()
        if args.engine:
            # the generation loop of gorgo_es_step spelled out, with the engine model's evaluation in the middle
            par = g.es_propose(state, g.es_sample(state.seed, state.generation, P))
            res = g.eval_engine(tr, model, engine, wl.rtt_ms, 1.0, params=par, per_request=False, workspace=ws)
            fit = res.p95_ttft_ms.cpu().numpy()
            g.es_update(state, par, fit)
            return par, fit, g.last_eval_kernel_ms()
        if args.online:
            res = g.eval_online(tr, model, wl.rtt_ms, theta0, z_on, 1.0, lo=state.lo[:], hi=state.hi[:], sigma0=state.sigma,
                                per_request=False, trajectory=False, workspace=ws)
            fit = res.p95_ttft_ms.cpu().numpy()
            return res.theta_final.cpu().numpy(), fit, g.last_eval_kernel_ms()
        par, fit, _ = g.es_step(tr, model, wl.rtt_ms, 1.0, P, state, workspace=ws)
        return par, fit, g.last_eval_kernel_ms()

    if args.calibrate_copy:
        src = torch.zeros((1 << 28,), dtype=torch.float32, device="cuda:0")       # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    warm_wall = []
    for i in range(args.warmup):
        t0 = time.perf_counter()
        generation()
        torch.cuda.synchronize()
        warm_wall.append(time.perf_counter() - t0)
        print(f"[bench] warmup generation {i}: {time.perf_counter() - t0:.2f}s", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    kernel_ms, fill_ms, select_ms = [], [], []
    t0 = time.perf_counter()
    for i in range(args.steps):
        par, fit, km = generation()
        kernel_ms.append(km["replay_ms"])
        fill_ms.append(km["fill_ms"])
        select_ms.append(km["select_ms"])
        print(f"[bench] generation {i}: replay kernel {km['replay_ms']:.1f} ms, best p95 TTFT {fit.min():.1f} ms, "
              f"theta=({state.theta[0]:.3f},{state.theta[2]:.3f}) sigma={state.sigma:.3f}", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1000.0 * wall / args.steps
    value = P * N * args.steps / wall

    # measured mean hit length on a sample of the last generation's candidates (outside the timed region)
    sample = min(P, 16)
    res = g.eval_population(tr, model, wl.rtt_ms, par[:sample], sweep_scale[:sample] if sweep else 1.0, p95=False)
    torch.cuda.synchronize()
    hit_mean = float(res.hit_blocks.to(torch.float64).mean().item())
    del res
    n_mean = float(np.diff(wl.trace.blk_off).mean())
    rp = tr.replay_path()
    segs_mean = rp["segment_refs"] / max(N, 1)
    if rp["path"] == 2:
        bpr = algorithmic_bytes_per_routing_segments(wl.R, segs_mean, outputs_bytes=8)   # ttft f64
        plain = args.online or args.engine or args.proxy
        kernel = "replay_segments_kernel" if plain or not g.replay_packing(tr, model, P) else "replay_segments_packed_kernel"
    else:
        bpr = algorithmic_bytes_per_routing(wl.R, n_mean, hit_mean, outputs_bytes=9)
        kernel = "replay_blocks_kernel"
    k_ms = float(np.mean(kernel_ms))
    counters = None if args.online or args.engine or args.proxy else recorded_counters(kernel, f"config-{args.config} N={N} P={P}")
    traffic = counters["fetch_bytes_per_launch"] + counters["write_bytes_per_launch"] if counters else None
    achieved = bpr * P * N / (k_ms * 1e-3) / 1e9
    # The replay is one dependent chain per candidate, so what limits it is how long one wavefront takes per request,
    # not a throughput ceiling: the recorded counters are reported per routing -- instructions by class, the share of
    # its cycles that the SIMD's vector ALU is busy, and the share of their cycles that the wavefronts spend waiting
    # (for memory, LDS, barriers or issue).  No fraction of an issue "peak" is given: a CU issues vector, scalar,
    # LDS, memory and branch instructions of different wavefronts side by side, so there is no single such limit.
    chain = None
    if counters and "sq_insts_per_routing" in counters:
        per = counters["sq_insts_per_routing"]
        chain = {"instructions_per_routing": per, "total_per_routing": sum(per.values()),
                 "us_per_request_step": k_ms * 1e3 / max(N, 1) * (1 if P <= 1024 else 1024 / P),
                 "valu_busy_frac": counters.get("valu_busy_frac"), "wave_wait_frac": counters.get("wave_wait_frac")}
    per_scale = None
    if sweep:
        # untimed breakdown: one launch per time scale (its 128 candidates)
        per_scale = {}
        for sc in sorted(set(float(x) for x in sweep_scale)):
            idx = np.nonzero(sweep_scale == sc)[0]
            g.eval_population(tr, model, wl.rtt_ms, sweep_par[idx], sweep_scale[idx], per_request=False, workspace=ws)
            torch.cuda.synchronize()
            per_scale[f"{sc:g}"] = g.last_eval_kernel_ms()["replay_ms"] * 1e3 / max(N, 1)
        print("[bench] us per request step by time scale: " + ", ".join(f"{k}: {v:.3f}" for k, v in per_scale.items()),
              file=sys.stderr, flush=True)

    if args.sections and rp["path"] == 2 and not (args.online or args.engine or args.proxy):
        del ws                                     # (the section array needs a workspace of its own size)
        torch.cuda.empty_cache()
        res = g.eval_population(tr, model, wl.rtt_ms, par, sweep_scale if sweep else 1.0, per_request=False, sections=True)
        torch.cuda.synchronize()
        t_ms = g.last_eval_kernel_ms()["replay_ms"]
        print(f"[bench] timed instantiation: replay kernel {t_ms:.1f} ms = {t_ms * 1e3 / max(N, 1):.3f} us per request step "
              f"(plain kernel: {k_ms * 1e3 / max(N, 1):.3f})", file=sys.stderr)
        print(section_table(res.sections.cpu().numpy(), N, P), file=sys.stderr, flush=True)
        del res

    mode = "P online tuners (window 128, hop 32) over the trace per step" if args.online else \
        "one launch of 8 time scales x 128 candidates per step (eval + p95 TTFT / E2E)" if sweep else \
        "one ES generation per step (eval + p95 TTFT fitness + mean update)"
    if args.engine:
        mode += ", replicas under the engine model (uneven rates, KV-token budget, decode slow-down)"
    if args.proxy:
        mode += ", imperfect proxy knowledge (RTT random walk per 30 s epoch scored through an EWMA with alpha 0.3, proxy cache index of twice the replicas' capacity)"
    out = {
        "metric": "candidate-request routings/sec at P=1024" + (" (online tuner)" if args.online else "") +
                  (" (engine model of a replica)" if args.engine else "") +
                  (" (imperfect proxy knowledge)" if args.proxy else ""),
        "value": value, "unit": "routings/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"config-{args.config} {wl.name}: R={wl.R} N={N} P={P} cache={wl.cache_blocks} blocks LRU, "
                               f"{mode}",
                   "es_generation_wall_s": None if sweep else wall / args.steps, "warmup_generation_wall_s": warm_wall,
                   "us_per_request_step_by_time_scale": per_scale},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "kernel": kernel, "mean_segments": segs_mean,
                     "kernel_ms": k_ms, "bytes_per_routing": bpr, "mean_blocks": n_mean, "mean_hit_blocks": hit_mean,
                     "fill_ms": float(np.mean(fill_ms)), "select_ms": float(np.mean(select_ms)),
                     "chain": chain},
    }
    if args.policies:
        out["policies"] = compare_policies(g, torch, tr, model, wl, [float(x) for x in state.best_theta[:]], N,
                                           engine if args.engine else None)
    if not args.no_cpu_baseline:
        cores = min(len(os.sched_getaffinity(0)), 16)
        on = (z_on[:cores].cpu().numpy(), list(state.lo[:]), list(state.hi[:]), state.sigma) if args.online else None
        sel = np.arange(cores) * max(1, P // cores) if sweep else np.arange(cores)      # (the sweep: replays of every time scale)
        v, dt, n_s = cpu_baseline(wl, theta0 if args.online else par[sel % len(par)], min(args.cpu_sample_requests, N), cores, on,
                                  recipe if args.engine else None, proxy if args.proxy else None,
                                  sweep_scale[sel] if sweep else None)
        plain = not (args.online or args.engine or args.proxy)
        v1, dt1, n1 = cpu_single_thread(wl, par, min(150000, N)) if plain else (None, None, None)
        cpu_model = "unknown"
        try:
            with open("/proc/cpuinfo") as f:
                cpu_model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), cpu_model)
        except OSError:
            pass
        out["cpu_baseline"] = {"value": v, "unit": "routings/s", "cores": cores, "kind": "oracle",
                               "sample": f"{cores} replays (one per thread) x first {n_s} requests of the same trace, "
                                         f"{dt:.1f}s wall",
                               "per_core": v / cores, "cpu_model": cpu_model, "host_cpus": os.cpu_count(),
                               "gpu_over_oracle": value / v,
                               "single_thread": None if v1 is None else
                               {"value": v1, "unit": "routings/s", "sample": f"1 replay x first {n1} requests, {dt1:.1f}s wall"}}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

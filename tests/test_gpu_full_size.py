"""GPU parity at the full size of the Large workload (R=32, N=1,000,000, P=1,024), in the launch
configuration the benchmark times: one launch over all 1,024 candidates of the tuner's first generation.

The oracle replays 34 of the candidates (the parent, the last one and 32 seeded picks) in full, one per host
thread; every request of those replays is compared (routes and hit counts bit-exact, latencies to 1e-9
relative), and so are their p95s, both from the launch that writes per-request outputs and from the
p95-only launch of the benchmark.  The p95 of every one of the 1,024 replays is checked against the nearest-rank
percentile of that replay's own latencies."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import paper_2602_11688_amd as g
from synth import tracegen as tg
from oracle import binding as ob
from tests.gpu_helpers import RTOL, load, oracle_eval

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def test_large_workload_sampled_replays_match_oracle():
    import torch
    wl = tg.config(5)
    es_cfg = wl.es if wl.es else dict(tg.ES_DEFAULTS, P=wl.P, seed=tg.MASTER_SEED + 5)
    P = es_cfg["P"]
    assert (wl.R, wl.trace.N, P) == (32, 1_000_000, 1024)
    model = g.Model(wl.R, wl.batch, wl.cache_blocks, wl.prefill_ms_per_token, wl.decode_ms_per_token)
    h = load(wl.trace)
    assert h.replay_path()["path"] == 2            # the formulation the benchmark runs
    state = g.es_init(es_cfg["seed"])
    params = g.es_propose(state, g.es_sample(es_cfg["seed"], 0, P))

    rng = np.random.default_rng(20260211)
    picks = sorted({0, P - 1} | set(rng.choice(np.arange(1, P - 1), 32, replace=False).tolist()))
    assert len(picks) == 34
    with ThreadPoolExecutor(16) as ex:             # ctypes releases the GIL: one oracle replay per thread
        futs = {p: ex.submit(oracle_eval, wl.trace, model, wl.rtt_ms, params[p], 1.0) for p in picks}

        # the p95-only launch keeps its latencies in the workspace, so its workspace also serves the other
        lean = g.eval_population(h, model, wl.rtt_ms, params, 1.0, per_request=False)
        torch.cuda.synchronize()
        full = g.eval_population(h, model, wl.rtt_ms, params, 1.0, workspace=lean.workspace)
        torch.cuda.synchronize()
        assert torch.equal(full.p95_ttft_ms, lean.p95_ttft_ms) and torch.equal(full.p95_e2e_ms, lean.p95_e2e_ms)
        p95_ttft = full.p95_ttft_ms.cpu().numpy()
        p95_e2e = full.p95_e2e_ms.cpu().numpy()
        assert np.isfinite(p95_ttft).all() and (p95_ttft > 0).all() and (p95_e2e >= p95_ttft).all()
        all_replays_p95_is_the_nearest_rank_of_their_latencies(torch, full)

        for p in picks:
            ref = futs[p].result()
            route = full.route[p].cpu().numpy()
            bad = np.nonzero(route != ref.route)[0]
            assert bad.size == 0, f"replay {p}: first route mismatch at request {bad[0]} ({bad.size} in all)"
            assert np.array_equal(full.hit_blocks[p].cpu().numpy(), ref.hit_blocks), f"replay {p}: hit counts"
            np.testing.assert_allclose(full.ttft_ms[p].cpu().numpy(), ref.ttft_ms, rtol=RTOL, atol=0)
            np.testing.assert_allclose(full.e2e_ms[p].cpu().numpy(), ref.e2e_ms, rtol=RTOL, atol=0)
            assert abs(p95_ttft[p] - ref.p95_ttft_ms) <= RTOL * ref.p95_ttft_ms
            assert abs(p95_e2e[p] - ref.p95_e2e_ms) <= RTOL * ref.p95_e2e_ms
            print(f"replay {p}: {ref.route.size} requests equal, p95 TTFT {ref.p95_ttft_ms:.3f} ms", flush=True)


def all_replays_p95_is_the_nearest_rank_of_their_latencies(torch, res):
    """The p95 of EVERY replay of a launch (not only of those the oracle replays in full) is the nearest-rank
    percentile -- the k-th smallest, k = ceil(0.95 N), the oracle's definition -- of that replay's own per-request
    latencies, bit for bit: the reduction is checked on all P, the latencies it reduces on the sampled replays."""
    P, N = res.ttft_ms.shape
    k = (95 * N + 99) // 100
    for lat, p95 in ((res.ttft_ms, res.p95_ttft_ms), (res.e2e_ms, res.p95_e2e_ms)):
        for a in range(0, P, 64):
            kth = torch.kthvalue(lat[a:a + 64], k, dim=1).values
            assert torch.equal(kth, p95[a:a + 64]), f"replays {a}..{a + 63}"


def test_large_workload_under_the_engine_model_matches_oracle():
    """The same launch shape with replicas under the engine model (uneven rates, KV-token budget, decode slow-down):
    18 replays against the oracle in full."""
    import torch
    wl = tg.config(5)
    es_cfg = wl.es if wl.es else dict(tg.ES_DEFAULTS, P=wl.P, seed=tg.MASTER_SEED + 5)
    P = es_cfg["P"]
    model = g.Model(wl.R, wl.batch, wl.cache_blocks, wl.prefill_ms_per_token, wl.decode_ms_per_token)
    recipe = tg.engine_recipe(wl)
    engine = g.Engine(recipe["prefill_ms_per_token"], recipe["decode_ms_per_token"], recipe["kv_tokens"], recipe["slowdown"])
    h = load(wl.trace)
    state = g.es_init(es_cfg["seed"])
    params = g.es_propose(state, g.es_sample(es_cfg["seed"], 0, P))
    rng = np.random.default_rng(20260212)
    picks = sorted({0, P - 1} | set(rng.choice(np.arange(1, P - 1), 16, replace=False).tolist()))

    def oracle(p):
        return ob.replay_engine(wl.trace, R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks,
                                prefill_ms_per_token=wl.prefill_ms_per_token, engine=recipe, rtt_ms=wl.rtt_ms,
                                w=params[p], scale=1.0)
    with ThreadPoolExecutor(16) as ex:
        futs = {p: ex.submit(oracle, p) for p in picks}
        full = g.eval_engine(h, model, engine, wl.rtt_ms, 1.0, params=params)
        torch.cuda.synchronize()
        p95_ttft = full.p95_ttft_ms.cpu().numpy()
        p95_e2e = full.p95_e2e_ms.cpu().numpy()
        assert np.isfinite(p95_ttft).all() and (p95_ttft > 0).all() and (p95_e2e >= p95_ttft).all()
        all_replays_p95_is_the_nearest_rank_of_their_latencies(torch, full)
        for p in picks:
            ref = futs[p].result()
            route = full.route[p].cpu().numpy()
            bad = np.nonzero(route != ref.route)[0]
            assert bad.size == 0, f"replay {p}: first route mismatch at request {bad[0]} ({bad.size} in all)"
            assert np.array_equal(full.hit_blocks[p].cpu().numpy(), ref.hit_blocks), f"replay {p}: hit counts"
            np.testing.assert_allclose(full.ttft_ms[p].cpu().numpy(), ref.ttft_ms, rtol=RTOL, atol=0)
            np.testing.assert_allclose(full.e2e_ms[p].cpu().numpy(), ref.e2e_ms, rtol=RTOL, atol=0)
            assert abs(p95_ttft[p] - ref.p95_ttft_ms) <= RTOL * ref.p95_ttft_ms
            assert abs(p95_e2e[p] - ref.p95_e2e_ms) <= RTOL * ref.p95_e2e_ms
            print(f"replay {p}: {ref.route.size} requests equal, p95 TTFT {ref.p95_ttft_ms:.3f} ms, p95 E2E "
                  f"{ref.p95_e2e_ms:.3f} ms", flush=True)


def test_large_workload_with_imperfect_proxy_knowledge_matches_oracle():
    """The same launch shape with round trip times that wander per 30 s probe epoch (scored through their moving
    average) and a proxy cache index of twice the replicas' capacity: 18 replays against the oracle in full."""
    import torch
    wl = tg.config(5)
    es_cfg = wl.es if wl.es else dict(tg.ES_DEFAULTS, P=wl.P, seed=tg.MASTER_SEED + 5)
    P = es_cfg["P"]
    model = g.Model(wl.R, wl.batch, wl.cache_blocks, wl.prefill_ms_per_token, wl.decode_ms_per_token)
    epochs = int(float(wl.trace.ts_ms[-1]) // 30000) + 1
    px = g.Proxy(tg.rtt_walk(wl, epochs), 30000, 0.3, 2 * wl.cache_blocks)
    h = load(wl.trace)
    state = g.es_init(es_cfg["seed"])
    params = g.es_propose(state, g.es_sample(es_cfg["seed"], 0, P))
    rng = np.random.default_rng(20260213)
    picks = sorted({0, P - 1} | set(rng.choice(np.arange(1, P - 1), 16, replace=False).tolist()))

    def oracle(p):
        return ob.replay_proxy(wl.trace, R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks,
                               prefill_ms_per_token=wl.prefill_ms_per_token, decode_ms_per_token=wl.decode_ms_per_token,
                               rtt_true=px.rtt_true_ms, probe_ms=30000, alpha=0.3, index_blocks=px.index_blocks, w=params[p], scale=1.0)
    with ThreadPoolExecutor(16) as ex:
        futs = {p: ex.submit(oracle, p) for p in picks}
        full = g.eval_proxy(h, model, px, params, 1.0)
        torch.cuda.synchronize()
        p95_ttft = full.p95_ttft_ms.cpu().numpy()
        p95_e2e = full.p95_e2e_ms.cpu().numpy()
        assert np.isfinite(p95_ttft).all() and (p95_ttft > 0).all() and (p95_e2e >= p95_ttft).all()
        all_replays_p95_is_the_nearest_rank_of_their_latencies(torch, full)
        for p in picks:
            ref = futs[p].result()
            route = full.route[p].cpu().numpy()
            bad = np.nonzero(route != ref.route)[0]
            assert bad.size == 0, f"replay {p}: first route mismatch at request {bad[0]} ({bad.size} in all)"
            assert np.array_equal(full.hit_blocks[p].cpu().numpy(), ref.hit_blocks), f"replay {p}: hit counts"
            assert np.array_equal(full.believed_hit_blocks[p].cpu().numpy(), ref.believed_hit), f"replay {p}: believed hits"
            np.testing.assert_allclose(full.ttft_ms[p].cpu().numpy(), ref.ttft_ms, rtol=RTOL, atol=0)
            np.testing.assert_allclose(full.e2e_ms[p].cpu().numpy(), ref.e2e_ms, rtol=RTOL, atol=0)
            assert abs(p95_ttft[p] - ref.p95_ttft_ms) <= RTOL * ref.p95_ttft_ms
            assert abs(p95_e2e[p] - ref.p95_e2e_ms) <= RTOL * ref.p95_e2e_ms
            over = float((ref.believed_hit > ref.hit_blocks).mean())
            print(f"replay {p}: {ref.route.size} requests equal, p95 TTFT {ref.p95_ttft_ms:.3f} ms, index overestimates on "
                  f"{100 * over:.1f}% of requests", flush=True)
        assert np.array_equal(full.rtt_est_ms.cpu().numpy(), futs[picks[0]].result().rtt_est)


def _against_oracle(wl, params, scale, picks, label):
    """One launch over all replays with per-request outputs; the picked replays against the oracle in full, one
    oracle replay per host thread."""
    import torch
    model = g.Model(wl.R, wl.batch, wl.cache_blocks, wl.prefill_ms_per_token, wl.decode_ms_per_token)
    h = load(wl.trace)
    with ThreadPoolExecutor(16) as ex:
        futs = {p: ex.submit(oracle_eval, wl.trace, model, wl.rtt_ms, params[p], float(scale[p])) for p in picks}
        full = g.eval_population(h, model, wl.rtt_ms, params, scale)
        torch.cuda.synchronize()
        p95_ttft = full.p95_ttft_ms.cpu().numpy()
        p95_e2e = full.p95_e2e_ms.cpu().numpy()
        assert np.isfinite(p95_ttft).all() and (p95_ttft > 0).all() and (p95_e2e >= p95_ttft).all()
        all_replays_p95_is_the_nearest_rank_of_their_latencies(torch, full)
        for p in picks:
            ref = futs[p].result()
            bad = np.nonzero(full.route[p].cpu().numpy() != ref.route)[0]
            assert bad.size == 0, f"{label} replay {p}: first route mismatch at request {bad[0]} ({bad.size} in all)"
            assert np.array_equal(full.hit_blocks[p].cpu().numpy(), ref.hit_blocks), f"{label} replay {p}: hit counts"
            np.testing.assert_allclose(full.ttft_ms[p].cpu().numpy(), ref.ttft_ms, rtol=RTOL, atol=0)
            np.testing.assert_allclose(full.e2e_ms[p].cpu().numpy(), ref.e2e_ms, rtol=RTOL, atol=0)
            assert abs(p95_ttft[p] - ref.p95_ttft_ms) <= RTOL * ref.p95_ttft_ms
            assert abs(p95_e2e[p] - ref.p95_e2e_ms) <= RTOL * ref.p95_e2e_ms
    print(f"{label}: {len(picks)} replays x {wl.trace.N} requests equal", flush=True)


@pytest.mark.parametrize("cfg", [2, 3])
def test_smaller_workloads_at_full_size_every_replay(cfg):
    """Configs 2 (R=8, N=50,000, P=64) and 3 (R=16, N=200,000, P=256) whole: every replay against the oracle."""
    wl = tg.config(cfg)
    _against_oracle(wl, wl.params, wl.scale, list(range(wl.params.shape[0])), f"config {cfg}")


def test_saturation_sweep_at_full_size_sampled_replays():
    """Config 4 (R=16, N=200,000, 1,024 (time scale, candidate) pairs in one launch): replay 0, the last one and 32
    seeded picks against the oracle in full."""
    wl = tg.config(4)
    P = wl.params.shape[0]
    assert P == 1024 and len(set(np.asarray(wl.scale).tolist())) > 1
    rng = np.random.default_rng(20260214)
    picks = sorted({0, P - 1} | set(rng.choice(np.arange(1, P - 1), 32, replace=False).tolist()))
    _against_oracle(wl, wl.params, wl.scale, picks, "config 4")

"""GPU parity of the engine model of a replica (continuous batching with a concurrency limit and a KV-token budget,
decode slow-down under occupancy, per-replica rates; Sec. 2.2, Sec. 5 "Exploiting Continuous Batching", Sec. 7)
against the CPU oracle, through the C ABI: routes and hit counts bit-exact, latencies to 1e-9 relative."""
import numpy as np
import pytest

import paper_2602_11688_amd as g
from oracle import binding as ob
from synth import tracegen as tg
from tests.gpu_helpers import RTOL, assert_replay_equal, load
from tests.helpers import load_golden

pytestmark = pytest.mark.gpu


def _numpy(res):
    import torch
    torch.cuda.synchronize()
    return dict(route=res.route.cpu().numpy(), hit=res.hit_blocks.cpu().numpy(), ttft=res.ttft_ms.cpu().numpy(),
                e2e=res.e2e_ms.cpu().numpy(), p95_ttft=res.p95_ttft_ms.cpu().numpy(), p95_e2e=res.p95_e2e_ms.cpu().numpy())


def _oracle(tr, model, eng, rtt, **kw):
    return ob.replay_engine(tr, R=model.R, batch=model.batch, cache_blocks=model.cache_blocks,
                            prefill_ms_per_token=model.prefill_ms_per_token, block_tokens=model.block_tokens, rtt_ms=rtt,
                            engine=dict(prefill_ms_per_token=eng.prefill_ms_per_token,
                                        decode_ms_per_token=eng.decode_ms_per_token, kv_tokens=eng.kv_tokens,
                                        slowdown=eng.decode_slowdown), **kw)


def check_engine(tr, model, eng, rtt, params, scale, label="engine", handle=None):
    """Fixed weights: every replay against the oracle."""
    params = np.asarray(params, np.float64)
    P = params.shape[0]
    scale = np.broadcast_to(np.asarray(scale, np.float64), (P,))
    got = _numpy(g.eval_engine(handle if handle is not None else load(tr), model, eng, rtt, scale, params=params))
    for p in range(P):
        assert_replay_equal(got, p, _oracle(tr, model, eng, rtt, w=params[p], scale=float(scale[p])), label)
    return got


def check_engine_policy(tr, model, eng, rtt, policy, scales, seeds=None):
    got = _numpy(g.eval_engine(load(tr), model, eng, rtt, scales, policy=policy, seeds=seeds))
    for p, sc in enumerate(scales):
        ref = _oracle(tr, model, eng, rtt, policy=policy, seed=0 if seeds is None else int(seeds[p]), scale=float(sc))
        assert_replay_equal(got, p, ref, policy)
    return got


def check_engine_online(tr, model, eng, rtt, theta0, z, scale, window, hop, lo, hi, sigma0):
    theta0 = np.asarray(theta0, np.float64)
    P = theta0.shape[0]
    scale = np.broadcast_to(np.asarray(scale, np.float64), (P,))
    res = g.eval_engine(load(tr), model, eng, rtt, scale, params=theta0,
                        online=dict(z=z, lo=lo, hi=hi, sigma0=sigma0, window=window, hop=hop))
    got = _numpy(res)
    for p in range(P):
        ref = _oracle(tr, model, eng, rtt, w=theta0[p], scale=float(scale[p]),
                      online=dict(z=z[p], lo=lo, hi=hi, sigma0=sigma0, window=window, hop=hop))
        assert_replay_equal(got, p, ref, "engine online")
        assert np.array_equal(res.theta_step[p].cpu().numpy(), ref.theta_step)
        np.testing.assert_allclose(res.fitness_step[p].cpu().numpy(), ref.fitness_step, rtol=RTOL, atol=0)
        assert np.array_equal(res.theta_final[p].cpu().numpy(), ref.theta_final)
        assert float(res.sigma_final[p]) == ref.sigma_final and int(res.accepted[p]) == ref.accepted
    return res


def _model(wl, **over):
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token)
    kw.update(over)
    return g.Model(**kw)


def _uneven(wl, seed, kv_factor, slowdown):
    rng = np.random.default_rng(seed)
    most = int((wl.trace.in_len.astype(np.int64) + wl.trace.out_len).max())
    return g.Engine(wl.prefill_ms_per_token * rng.uniform(0.5, 2.0, wl.R), wl.decode_ms_per_token * rng.uniform(0.5, 2.0, wl.R),
                    None if kv_factor is None else [int(kv_factor * most)] * wl.R, slowdown)


@pytest.mark.parametrize("name", ["engine_hand_A.json", "engine_hand_B.json"])
def test_hand_worked_traces(name):
    gold, tr = load_golden(name)
    m, e = gold["model"], gold["model"]["engine"]
    model = g.Model(m["R"], m["batch"], m["cache_blocks"], m["prefill_ms_per_token"], 0.0, block_tokens=m["block_tokens"])
    eng = g.Engine(e["prefill_ms_per_token"], e["decode_ms_per_token"], e["kv_tokens"], e["slowdown"])
    h = g.Trace.from_arrays(tr.ts_ms, tr.in_len, tr.out_len, tr.blk_off, tr.hash_ids, block_tokens=m["block_tokens"])
    got = _numpy(g.eval_engine(h, model, eng, gold["rtt_ms"], [gold["scale"]], params=[gold["w"]]))
    x = gold["expected"]
    assert got["route"][0].tolist() == x["route"] and got["hit"][0].tolist() == x["hit_blocks"]
    assert got["ttft"][0].tolist() == x["ttft_ms"] and got["e2e"][0].tolist() == x["e2e_ms"]
    assert got["p95_ttft"][0] == x["p95_ttft_ms"] and got["p95_e2e"][0] == x["p95_e2e_ms"]


def test_equals_the_linear_model_without_slowdown_and_budget():
    import torch
    wl = tg.config(1)
    model = _model(wl)
    h = load(wl.trace)
    lin = g.eval_population(h, model, wl.rtt_ms, wl.params[:8], wl.scale[:8])
    eng = g.Engine([wl.prefill_ms_per_token] * wl.R, [wl.decode_ms_per_token] * wl.R, None, 0.0)
    res = g.eval_engine(h, model, eng, wl.rtt_ms, wl.scale[:8], params=wl.params[:8])
    torch.cuda.synchronize()
    for name in ("route", "hit_blocks", "ttft_ms", "e2e_ms", "p95_ttft_ms", "p95_e2e_ms"):
        assert torch.equal(getattr(lin, name), getattr(res, name)), name


@pytest.mark.parametrize("kv_factor,slowdown", [(None, 0.0), (None, 0.25), (3.0, 0.0), (2.0, 0.1), (1.0, 1.0)])
def test_saturated_and_idle_replicas(kv_factor, slowdown):
    wl = tg.config(1)
    eng = _uneven(wl, 1, kv_factor, slowdown)
    got = check_engine(wl.trace, _model(wl), eng, wl.rtt_ms, wl.params[:6], [1.0, 1.0, 2.0, 4.0, 8.0, 0.5])
    assert len(set(got["route"][0].tolist())) > 1


def test_bounded_caches_and_many_replicas():
    wl = tg.config(2, 8000)
    check_engine(wl.trace, _model(wl), _uneven(wl, 2, 2.5, 0.2), wl.rtt_ms, wl.params[:4], wl.scale[:4])
    wl = tg.config(3, 6000)
    check_engine(wl.trace, _model(wl), _uneven(wl, 3, 4.0, 0.05), wl.rtt_ms, wl.params[:4], wl.scale[:4])


@pytest.mark.parametrize("B", [1, 2, 7, 8, 9, 16, 33, 64])
def test_slot_counts(B):
    R = 1024 // B if B > 16 else 8
    R = min(R, 12)
    tr = tg.random_forest(40 + B, 1500, max_blocks=12, gap_ms=6)
    most = int((tr.in_len.astype(np.int64) + tr.out_len).max())
    rng = np.random.default_rng(B)
    eng = g.Engine(rng.uniform(0.01, 0.1, R), rng.uniform(5.0, 40.0, R), [int(most * min(B, 3))] * R, 0.3)
    par = rng.uniform(0.0, 2.0, (3, 3))
    check_engine(tr, g.Model(R, B, 30, 0.05, 20.0), eng, np.linspace(5.0, 150.0, R), par, [1.0, 0.3, 3.0], f"B={B}")


def test_zero_rates_zero_outputs_and_simultaneous_arrivals():
    tr = tg.random_small(5, 400, 3, n_ids=40, max_blocks=4, gap_ms=2)
    tr = tg.Trace((tr.ts_ms // 4) * 4, tr.in_len, np.where(np.arange(tr.N) % 3 == 0, 0, tr.out_len).astype(np.int32),
                  tr.blk_off, tr.hash_ids)
    eng = g.Engine([0.0, 0.05, 0.0], [0.0, 0.0, 10.0], [0, 5000, 3000], 2.0)
    check_engine(tr, g.Model(3, 4, 0, 0.05, 20.0), eng, [0.0, 10.0, 0.0], [[1, 1, 1], [0, 0, 0], [0.3, 0, 2]], [1.0, 0.0, 2.0])


@pytest.mark.parametrize("policy", ["least-request", "session-affinity", "random"])
def test_baseline_policies_under_the_engine_model(policy):
    wl = tg.config(1)
    seeds = np.array([11, 12, 13], np.uint64) if policy == "random" else None
    check_engine_policy(wl.trace, _model(wl), _uneven(wl, 4, 2.0, 0.15), wl.rtt_ms, policy, [1.0, 3.0, 0.5], seeds)


def test_online_tuner_under_the_engine_model():
    wl = tg.config(1)
    tr = wl.trace.head(1200)
    rng = np.random.default_rng(5)
    P, window, hop = 6, 128, 32
    steps = g.online_steps(tr.N, window, hop)
    theta0 = np.tile([1.0, 0.5, 0.1], (P, 1))
    res = check_engine_online(tr, _model(wl), _uneven(wl, 6, 3.0, 0.2), wl.rtt_ms, theta0,
                              rng.standard_normal((P, steps, 3)), 16.0, window, hop, [0.05] * 3, [2.0] * 3, 0.5)
    assert int(res.accepted.sum()) > 0


@pytest.mark.parametrize("seed", range(24))
def test_random_cases(seed):
    rng = np.random.default_rng(7000 + seed)
    R = int(rng.choice([1, 2, 3, 5, 8, 16, 32, 64]))
    B = int(rng.choice([1, 2, 3, 8, 16]))
    N = int(rng.integers(60, 700))
    tr = tg.random_forest(100 + seed, N, roots=int(rng.integers(1, 5)), max_blocks=int(rng.integers(4, 40)),
                          grow=int(rng.integers(1, 9)), gap_ms=int(rng.integers(1, 60)), keep=float(rng.choice([0.0, 0.5, 0.85])))
    nmax = int(np.diff(tr.blk_off).max())
    most = int((tr.in_len.astype(np.int64) + tr.out_len).max())
    model = g.Model(R, B, int(rng.choice([0, nmax, 3 * nmax + 1])), float(rng.choice([0.0, 0.01, 0.05])), 0.0)
    kv = None if seed % 4 == 0 else [int(rng.choice([0, 1, most, 2 * most, 4 * most])) for _ in range(R)]
    eng = g.Engine(rng.choice([0.0, 0.02, 0.05, 0.2], R), rng.choice([0.0, 1.0, 10.0, 30.0], R), kv,
                   float(rng.choice([0.0, 0.1, 1.0, 5.0])))
    rtt = np.round(rng.uniform(0.0, 300.0, R), 1)
    par = rng.uniform(0.0, 2.0, (3, 3))
    scale = rng.choice([0.25, 1.0, 3.0], 3)
    check_engine(tr, model, eng, rtt, par, scale, f"fuzz {seed}")
    for policy in ("least-request", "random"):
        check_engine_policy(tr, model, eng, rtt, policy, list(scale[:2]), np.array([seed, seed + 1], np.uint64))
    window, hop = int(rng.integers(1, 150)), int(rng.integers(1, 60))
    steps = g.online_steps(tr.N, window, hop)
    check_engine_online(tr, model, eng, rtt, np.clip(par, 0.05, 2.0), 2.0 * rng.standard_normal((3, steps, 3)), scale,
                        window, hop, [0.05] * 3, [2.0] * 3, 0.5)


def test_concentrating_load_trades_e2e_for_ttft():
    """The effect the engine model is there for (Sec. 5 "Exploiting Continuous Batching"): with room in the batch, a
    router that ignores load and sends everything to the nearest replica gets the lower p95 TTFT and the higher
    p95 E2E than one that spreads by load."""
    wl = tg.config(1)
    model = _model(wl, batch=64, cache_blocks=0)
    eng = g.Engine([wl.prefill_ms_per_token] * wl.R, [wl.decode_ms_per_token] * wl.R, None, 0.05)
    got = check_engine(wl.trace, model, eng, wl.rtt_ms, [[1.0, 0.0, 0.0], [0.0, 0.0, 1.0]], 8.0)
    assert len(set(got["route"][0].tolist())) == 1
    assert got["p95_ttft"][0] < got["p95_ttft"][1] and got["p95_e2e"][0] > got["p95_e2e"][1]

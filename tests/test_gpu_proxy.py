"""GPU parity of imperfect proxy knowledge (round trip times per probe epoch scored through their moving average,
Sec. 2.2 and the RTT figure of Sec. 4; a proxy cache index that does not see replica-side eviction, Sec. 7) against
the CPU oracle, through the C ABI: routes, hit counts and believed hit counts bit-exact, latencies to 1e-9 relative."""
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
                e2e=res.e2e_ms.cpu().numpy(), p95_ttft=res.p95_ttft_ms.cpu().numpy(), p95_e2e=res.p95_e2e_ms.cpu().numpy(),
                believed=res.believed_hit_blocks.cpu().numpy(), rtt_est=res.rtt_est_ms.cpu().numpy())


def _oracle(tr, model, px, w, scale, engine=None, online=None):
    e = None if engine is None else dict(prefill_ms_per_token=engine.prefill_ms_per_token,
                                         decode_ms_per_token=engine.decode_ms_per_token, kv_tokens=engine.kv_tokens,
                                         slowdown=engine.decode_slowdown)
    return ob.replay_proxy(tr, R=model.R, batch=model.batch, cache_blocks=model.cache_blocks,
                           prefill_ms_per_token=model.prefill_ms_per_token, decode_ms_per_token=model.decode_ms_per_token,
                           block_tokens=model.block_tokens, rtt_true=px.rtt_true_ms, probe_ms=px.probe_interval_ms,
                           alpha=px.ewma_alpha, index_blocks=px.index_blocks, engine=e, w=w, scale=scale, online=online)


def check_proxy(tr, model, px, params, scale, engine=None, label="proxy", handle=None):
    params = np.asarray(params, np.float64)
    P = params.shape[0]
    scale = np.broadcast_to(np.asarray(scale, np.float64), (P,))
    got = _numpy(g.eval_proxy(handle if handle is not None else load(tr), model, px, params, scale, engine=engine))
    for p in range(P):
        ref = _oracle(tr, model, px, params[p], float(scale[p]), engine)
        assert_replay_equal(got, p, ref, label)
        assert np.array_equal(got["believed"][p], ref.believed_hit), f"{label} believed hits replay {p}"
        assert np.array_equal(got["rtt_est"], ref.rtt_est), f"{label} smoothed round trip times"
    return got


def _model(wl, **over):
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token)
    kw.update(over)
    return g.Model(**kw)


def _wander(rtt, epochs, seed, amount=0.5):
    """True round trip times that wander around the workload's: a seeded multiplicative random walk per replica."""
    rng = np.random.default_rng(seed)
    steps = np.exp(amount * rng.standard_normal((epochs, len(rtt))) * 0.5)
    return np.round(np.asarray(rtt)[None, :] * np.cumprod(steps, axis=0) / steps[0], 3)


def test_hand_worked_trace():
    gold, tr = load_golden("proxy_hand.json")
    m, x, e = gold["model"], gold["proxy"], gold["expected"]
    model = g.Model(m["R"], m["batch"], m["cache_blocks"], m["prefill_ms_per_token"], m["decode_ms_per_token"],
                    block_tokens=m["block_tokens"])
    px = g.Proxy(x["rtt_true"], x["probe_ms"], x["alpha"], x["index_blocks"])
    h = g.Trace.from_arrays(tr.ts_ms, tr.in_len, tr.out_len, tr.blk_off, tr.hash_ids, block_tokens=m["block_tokens"])
    got = _numpy(g.eval_proxy(h, model, px, [gold["w"]], [gold["scale"]]))
    assert got["route"][0].tolist() == e["route"] and got["hit"][0].tolist() == e["hit_blocks"]
    assert got["believed"][0].tolist() == e["believed_hit"] and got["rtt_est"].tolist() == e["rtt_est"]
    assert got["ttft"][0].tolist() == e["ttft_ms"] and got["e2e"][0].tolist() == e["e2e_ms"]
    assert got["p95_ttft"][0] == e["p95_ttft_ms"] and got["p95_e2e"][0] == e["p95_e2e_ms"]


@pytest.mark.parametrize("index", [-1, "cache"])
def test_equals_the_plain_replay_with_perfect_knowledge(index):
    """Constant round trip times and either no index of its own or one exactly as large as the replicas' caches."""
    import torch
    wl = tg.config(2, 8000)
    model = _model(wl)
    index = wl.cache_blocks if index == "cache" else index
    h = load(wl.trace)
    plain = g.eval_population(h, model, wl.rtt_ms, wl.params[:6], wl.scale[:6])
    res = g.eval_proxy(h, model, g.Proxy(np.tile(wl.rtt_ms, (4, 1)), 5000, 0.3, index), wl.params[:6], wl.scale[:6])
    torch.cuda.synchronize()
    for name in ("route", "hit_blocks", "ttft_ms", "e2e_ms", "p95_ttft_ms", "p95_e2e_ms"):
        assert torch.equal(getattr(plain, name), getattr(res, name)), name
    assert torch.equal(res.believed_hit_blocks, res.hit_blocks)


@pytest.mark.parametrize("index", ["none", "unbounded", "double", "tight"])
@pytest.mark.parametrize("cfg,head", [(1, None), (2, 8000), (3, 6000)])
def test_workloads(cfg, head, index):
    wl = tg.config(cfg, head)
    C = wl.cache_blocks
    if C == 0 and index in ("double", "tight"):
        pytest.skip("replicas that never evict leave no room for an index that forgets later")
    stale = index != "none"
    index = {"none": -1, "unbounded": 0, "double": 2 * C, "tight": C + 1}[index]
    horizon = float(wl.trace.ts_ms[-1]) * float(max(wl.scale[:4]))
    probe = max(1, int(horizon / 12))
    px = g.Proxy(_wander(wl.rtt_ms, 10, cfg), probe, 0.3, index)     # the last epochs repeat the tenth
    got = check_proxy(wl.trace, _model(wl), px, wl.params[:4], wl.scale[:4], label=f"config {cfg} index={index}")
    if stale and wl.cache_blocks > 0:
        assert (got["believed"] > got["hit"]).any()


def test_epoch_boundaries_and_time_scales():
    tr = tg.random_forest(3, 900, max_blocks=10, gap_ms=7)
    model = g.Model(3, 2, 14, 0.05, 5.0)
    true = _wander([10.0, 60.0, 25.0], 40, 9, amount=1.0)
    for probe in (1, 50, 333):
        check_proxy(tr, model, g.Proxy(true, probe, 0.5, [0, 20, 14][probe % 3]), [[1.0, 1.0, 0.2]] * 4, [1.0, 0.37, 2.5, 0.0], label=f"probe {probe}")


def test_with_the_engine_model_and_the_online_tuner():
    wl = tg.config(1)
    tr = wl.trace.head(1500)
    model = _model(wl, cache_blocks=600)
    recipe = tg.engine_recipe(wl)
    engine = g.Engine(recipe["prefill_ms_per_token"], recipe["decode_ms_per_token"], recipe["kv_tokens"], 0.2)
    px = g.Proxy(_wander(wl.rtt_ms, 8, 4), 20000, 0.4, 900)
    check_proxy(tr, model, px, wl.params[:3], [1.0, 4.0, 16.0], engine=engine, label="engine")
    rng = np.random.default_rng(8)
    P, window, hop = 4, 128, 32
    steps = g.online_steps(tr.N, window, hop)
    z = rng.standard_normal((P, steps, 3))
    theta0 = np.tile([1.0, 0.5, 0.1], (P, 1))
    on = dict(lo=[0.05] * 3, hi=[2.0] * 3, sigma0=0.5, window=window, hop=hop)
    for eng in (None, engine):
        res = g.eval_proxy(load(tr), model, px, theta0, 16.0, engine=eng, online=dict(on, z=z))
        got = _numpy(res)
        for p in range(P):
            ref = _oracle(tr, model, px, theta0[p], 16.0, eng, online=dict(on, z=z[p]))
            assert_replay_equal(got, p, ref, "proxy online")
            assert np.array_equal(got["believed"][p], ref.believed_hit)
            assert np.array_equal(res.theta_step[p].cpu().numpy(), ref.theta_step)
            np.testing.assert_allclose(res.fitness_step[p].cpu().numpy(), ref.fitness_step, rtol=RTOL, atol=0)
            assert int(res.accepted[p]) == ref.accepted and float(res.sigma_final[p]) == ref.sigma_final


@pytest.mark.parametrize("seed", range(24))
def test_random_cases(seed):
    rng = np.random.default_rng(9000 + seed)
    R = int(rng.choice([1, 2, 3, 5, 8, 16, 32, 64]))
    B = int(rng.choice([1, 2, 3, 8, 16]))
    N = int(rng.integers(60, 700))
    tr = tg.random_forest(200 + seed, N, roots=int(rng.integers(1, 5)), max_blocks=int(rng.integers(4, 60)),
                          grow=int(rng.integers(1, 9)), gap_ms=int(rng.integers(1, 60)), keep=float(rng.choice([0.0, 0.5, 0.85])))
    nmax = int(np.diff(tr.blk_off).max())
    model = g.Model(R, B, int(rng.choice([0, nmax, nmax + 1, 2 * nmax + 3, 10 * nmax])), float(rng.choice([0.0, 0.01, 0.05])),
                    float(rng.choice([0.0, 1.0, 20.0])))
    E = int(rng.integers(1, 30))
    C = model.cache_blocks
    index = -1 if seed % 3 == 0 else (0 if seed % 3 == 1 or C == 0 else int(rng.choice([C, C + 1, C + nmax, 3 * C])))
    px = g.Proxy(np.round(rng.uniform(0.0, 300.0, (E, R)), 1), int(rng.choice([1, 100, 1000, 30000])),
                 float(rng.choice([0.05, 0.5, 1.0])), index)
    par = rng.uniform(0.0, 2.0, (3, 3))
    if seed % 5 == 0:
        par[0] = [0.0, 1.0, 0.0]
    scale = rng.choice([0.25, 1.0, 3.0], 3)
    engine = None
    if seed % 2:
        most = int((tr.in_len.astype(np.int64) + tr.out_len).max())
        engine = g.Engine(rng.choice([0.0, 0.02, 0.2], R), rng.choice([0.0, 1.0, 30.0], R),
                          [int(rng.choice([0, most, 4 * most])) for _ in range(R)], float(rng.choice([0.0, 0.1, 1.0])))
    check_proxy(tr, model, px, par, scale, engine=engine, label=f"fuzz {seed}")


def test_long_paths_and_an_index_of_its_own():
    """Requests with more segments than are preloaded (the deep-match path), tight caches, an index of its own."""
    tr = tg.random_forest(77, 1200, roots=2, max_blocks=120, grow=3, gap_ms=5, keep=0.8)
    nmax = int(np.diff(tr.blk_off).max())
    segs = load(tr).replay_path()["segment_refs"] / tr.N
    assert segs > 6
    for C in (nmax, 2 * nmax + 1, 6 * nmax):
        for index in (0, C + nmax // 2, 3 * C):
            got = check_proxy(tr, g.Model(4, 2, C, 0.05, 3.0), g.Proxy([[5.0, 40.0, 90.0, 20.0]], 30000, 0.5, index),
                              [[0.5, 1.0, 0.1], [0.0, 1.0, 0.0], [1.0, 1.0, 1.0]], [1.0, 1.0, 3.0], label=f"deep C={C} index={index}")
            assert (got["believed"] >= got["hit"]).all() and (got["believed"] > got["hit"]).any()


@pytest.mark.parametrize("B", [1, 3])
def test_completion_events_that_overtake_each_other(B):
    """Round trip times that fall by seconds from one probe epoch to the next: completion events of later requests
    reach the proxy before those of many earlier ones on the same service slot, at the head, inside and at the end
    of the slot's in-flight list.  Routing on the load signal alone makes every misplaced event show in the routes."""
    tr = tg.random_forest(31, 2500, roots=3, max_blocks=8, grow=3, gap_ms=6)
    R = 2
    cycle = np.array([[8000.0, 6000.0], [0.0, 3000.0], [4000.0, 100.0], [6000.0, 7000.0], [1000.0, 0.0], [5000.0, 2500.0]])
    px = g.Proxy(np.tile(cycle, (8, 1)), 150, 0.5, -1)
    got = check_proxy(tr, g.Model(R, B, 0, 0.001, 0.01), px, [[0.0, 0.0, 1.0], [0.1, 1.0, 1.0], [0.0, 0.0, 1.0]], [1.0, 1.0, 0.3],
                      label=f"overtaking B={B}")
    assert len(set(got["route"][0].tolist())) == R


def test_largest_launch_shape():
    """64 replicas x 16 slots, a 1,024-request tuner window, engine model and imperfect proxy knowledge together: the
    variant with the most per-replay state in LDS and registers still launches and matches the oracle."""
    R, B = 64, 16
    tr = tg.random_forest(55, 2600, roots=4, max_blocks=30, grow=5, gap_ms=4, keep=0.5)
    nmax = int(np.diff(tr.blk_off).max())
    most = int((tr.in_len.astype(np.int64) + tr.out_len).max())
    rng = np.random.default_rng(55)
    model = g.Model(R, B, 3 * nmax, 0.05, 0.0)
    engine = g.Engine(rng.uniform(0.02, 0.1, R), rng.uniform(1.0, 20.0, R), [6 * most] * R, 0.1)
    px = g.Proxy(np.round(rng.uniform(1.0, 200.0, (12, R)), 1), 900, 0.3, 5 * nmax)
    P, window, hop = 3, 1024, 64
    steps = g.online_steps(tr.N, window, hop)
    z = rng.standard_normal((P, steps, 3))
    theta0 = np.tile([1.0, 0.5, 0.1], (P, 1))
    on = dict(lo=[0.05] * 3, hi=[2.0] * 3, sigma0=0.5, window=window, hop=hop)
    res = g.eval_proxy(load(tr), model, px, theta0, [1.0, 2.0, 0.5], engine=engine, online=dict(on, z=z))
    got = _numpy(res)
    for p, sc in enumerate([1.0, 2.0, 0.5]):
        ref = _oracle(tr, model, px, theta0[p], sc, engine, online=dict(on, z=z[p]))
        assert_replay_equal(got, p, ref, "largest shape")
        assert np.array_equal(got["believed"][p], ref.believed_hit)
        assert np.array_equal(res.theta_step[p].cpu().numpy(), ref.theta_step)

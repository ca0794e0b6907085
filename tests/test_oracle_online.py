"""Pins of the oracle's online tuner (Sec. 2.3 "GORGO Proxy Design", Sec. 4 "Tuning and evaluation windows")
against things other than itself: the step count the paper prints, a hand-worked run, the sorted-array order
statistic, an independent forced-route/forced-schedule model, the separately pinned generation step of the
tuner at P = 2, and the C library's exp."""
import json
import math
import os

import numpy as np
import pytest

from oracle import binding as ob
from oracle import es_oracle as eo
from synth import tracegen as tg
from synth.tracegen import Trace
from tests.helpers import GOLDEN, ForcedRouteModel

LO, HI = [0.05, 1.0, 0.05], [2.0, 1.0, 0.5]


def _kw(wl, **over):
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token, rtt_ms=wl.rtt_ms, block_tokens=wl.block_tokens)
    kw.update(over)
    return kw


def _same(a, b):
    assert np.array_equal(a.route, b.route) and np.array_equal(a.hit_blocks, b.hit_blocks)
    assert np.array_equal(a.ttft_ms, b.ttft_ms) and np.array_equal(a.e2e_ms, b.e2e_ms)


def test_tuner_exp_against_the_c_library():
    assert ob.tuner_exp(0.0) == 1.0
    rng = np.random.default_rng(3)
    xs = np.concatenate([np.linspace(-231.0, 231.0, 2001), rng.uniform(-5, 5, 2000), [math.log(0.05), math.log(2.0)]])
    for x in xs:
        ref = math.exp(float(x))
        assert abs(ob.tuner_exp(float(x)) - ref) <= 4 * math.ulp(ref), x
    # monotone where the tuner uses it (clipping in log space and in linear space must agree)
    ys = np.sort(rng.uniform(math.log(0.05), math.log(2.0), 4000))
    vals = [ob.tuner_exp(float(y)) for y in ys]
    assert all(b >= a for a, b in zip(vals, vals[1:]))


def test_step_count_of_the_paper():
    # Sec. 4 / Fig. "Convergence of the evolutionary strategy": 672 samples are the 18th evolutionary step of a
    # 128-request window with hop 32 (128 + 17 * 32 = 672)
    assert ob.online_steps(672, 128, 32) == 18
    assert ob.online_steps(671, 128, 32) == 17
    assert ob.online_steps(127, 128, 32) == 0 and ob.online_steps(128, 128, 32) == 1


def test_hand_worked_tuner_run():
    with open(os.path.join(GOLDEN, "online_tuner_hand.json")) as f:
        g = json.load(f)
    L = np.array(g["input_length"], np.int32)
    n = L.astype(np.int64)                      # one block per token, all fresh
    tr = Trace(np.arange(len(L), dtype=np.int64) * 1000, L, np.ones(len(L), np.int32),
               np.concatenate([[0], np.cumsum(n)]).astype(np.int64), np.arange(1, int(n.sum()) + 1, dtype=np.int64))
    m = g["model"]
    res = ob.replay_online(tr, R=m["R"], batch=m["batch"], cache_blocks=m["cache_blocks"], block_tokens=m["block_tokens"],
                           prefill_ms_per_token=m["prefill_ms_per_token"], decode_ms_per_token=m["decode_ms_per_token"],
                           rtt_ms=g["rtt_ms"], theta0=g["theta0"], z=g["z"], lo=g["lo"], hi=g["hi"], sigma0=g["sigma0"],
                           window=g["window"], hop=g["hop"])
    e = g["expected"]
    assert res.ttft_ms.tolist() == e["ttft_ms"]
    assert res.fitness_step.tolist() == e["fitness_step"]
    np.testing.assert_allclose(res.theta_step, e["theta_step"], rtol=4e-16, atol=0)
    np.testing.assert_allclose(res.theta_final, e["theta_final"], rtol=4e-16, atol=0)
    assert (res.steps, res.accepted) == (e["steps"], e["accepted"])
    assert abs(math.log(res.sigma_final / g["sigma0"]) - e["sigma_final_log_over_sigma0"]) < 1e-15


def test_constant_schedule_is_the_static_replay():
    wl = tg.config(1, 600)
    w = [0.7, 1.0, 0.3]
    steps = ob.online_steps(wl.trace.N, 128, 32)
    a = ob.replay(wl.trace, w=w, **_kw(wl))
    b = ob.replay_schedule(wl.trace, w=w, schedule=np.tile(w, (steps, 1)), window=128, hop=32, **_kw(wl))
    _same(a, b)


def test_schedule_takes_effect_on_the_request_after_the_step():
    # weights switch between RTT-only and queue-only routing; an independent model that is told the routes and
    # the weight every request was scored with must find every route the minimum of its scores, and must not
    # when the schedule is applied one request early or late
    wl = tg.config(1, 90)
    tr, W, H = wl.trace, 16, 8
    steps = ob.online_steps(tr.N, W, H)
    sched = np.array([[0.0, 0.0, 1.0] if h % 2 == 0 else [1.0, 0.0, 0.0] for h in range(steps)])
    w0 = [1.0, 0.0, 0.0]
    res = ob.replay_schedule(tr, w=w0, schedule=sched, window=W, hop=H, **_kw(wl))

    def per_request(shift):
        out = []
        for r in range(tr.N):
            done = (r + shift - W) // H + 1 if r + shift >= W else 0      # steps taken before request r is scored
            out.append(list(w0) if done <= 0 else list(sched[min(done, steps) - 1]))
        return out

    def consistent(shift):
        fm = ForcedRouteModel(tr, wl.R, wl.batch, wl.cache_blocks, wl.block_tokens, wl.prefill_ms_per_token,
                              wl.decode_ms_per_token, wl.rtt_ms, per_request(shift), 1.0)
        return fm.run(res.route.tolist())["consistent"]

    assert consistent(0)
    assert not consistent(1) and not consistent(-1)
    assert len(set(res.route.tolist())) > 1


@pytest.mark.parametrize("seed", [0, 1])
def test_online_run_is_the_replay_of_its_own_schedule_and_fitness_is_the_window_order_statistic(seed):
    wl = tg.config(1, 1500)
    W, H = 128, 32
    steps = ob.online_steps(wl.trace.N, W, H)
    z = np.random.default_rng(seed).standard_normal((steps, 3))
    on = ob.replay_online(wl.trace, theta0=[0.5, 1.0, 0.1], z=z, lo=LO, hi=HI, sigma0=0.5, window=W, hop=H, **_kw(wl))
    assert on.steps == steps
    sc = ob.replay_schedule(wl.trace, w=[0.5, 1.0, 0.1], schedule=on.theta_step, window=W, hop=H, **_kw(wl))
    _same(on, sc)
    k = math.ceil(0.95 * W)
    for h in range(steps):
        end = W + h * H
        assert on.fitness_step[h] == np.sort(on.ttft_ms[end - W:end])[k - 1]
    assert len({tuple(t) for t in on.theta_step.tolist()}) > 3          # the weights do move


def test_tuner_steps_follow_the_generation_rule_at_population_two():
    # the separately pinned generation step (candidate 0 = parent, candidate 1 = offspring) must give the same
    # accept decisions, step sizes and proposals, up to the rounding of exp/log
    wl = tg.config(1, 1200)
    W, H = 128, 32
    steps = ob.online_steps(wl.trace.N, W, H)
    z = np.random.default_rng(5).standard_normal((steps, 3))
    theta0, sigma0 = np.array([0.5, 1.0, 0.1]), 0.5
    # (time scale 4: the replicas are not saturated, so the window p95 goes up and down and offspring do win)
    on = ob.replay_online(wl.trace, theta0=theta0, z=z, lo=LO, hi=HI, sigma0=sigma0, window=W, hop=H, scale=4.0,
                          **_kw(wl))
    parent, f_par, sigma, accepted = theta0.copy(), None, sigma0, 0
    current = theta0.copy()
    for h in range(steps):
        f = on.fitness_step[h]
        if f_par is None:
            f_par = f
        else:
            new_parent, sigma, _, _ = eo.update(parent, sigma, LO, HI, np.stack([parent, current]), [f_par, f])
            if f < f_par:
                assert np.array_equal(new_parent, current)
                f_par, accepted = f, accepted + 1
            parent = new_parent
        current = eo.offspring(parent, sigma, LO, HI, np.stack([np.zeros(3), z[h]]))[1]
        np.testing.assert_allclose(on.theta_step[h], current, rtol=1e-13, atol=0)
        current = on.theta_step[h].copy()                   # follow the oracle's bits from here on
    assert accepted == on.accepted and 0 < accepted < steps - 1
    assert abs(on.sigma_final / sigma - 1) < 1e-13
    np.testing.assert_allclose(on.theta_final, parent, rtol=1e-13, atol=0)


def test_zero_step_size_keeps_unit_weights_and_matches_the_static_replay():
    # ln 1 = 0 and exp 0 = 1 exactly, so with sigma = 0 the tuner proposes (1, 1, 1) for ever
    wl = tg.config(1, 500)
    steps = ob.online_steps(wl.trace.N, 128, 32)
    on = ob.replay_online(wl.trace, theta0=[1.0, 1.0, 1.0], z=np.ones((steps, 3)), lo=[0.5] * 3, hi=[2.0] * 3,
                          sigma0=0.0, window=128, hop=32, **_kw(wl))
    _same(on, ob.replay(wl.trace, w=[1.0, 1.0, 1.0], **_kw(wl)))
    assert np.array_equal(on.theta_step, np.ones((steps, 3))) and on.accepted == 0

"""CPU pins of the oracle's imperfect proxy knowledge (Sec. 2.2: T_network is a moving average of pings; Sec. 4,
RTT figure: probed at fixed intervals; Sec. 7: the proxy's cache index does not see replica-side eviction): a
hand-worked trace, closed forms of the moving average, probe epochs recovered from latencies, reductions to the
plain replay, an independent forced-route model, and the one-sidedness of the index's error."""
import numpy as np
import pytest

from oracle import binding as ob
from synth import tracegen as tg
from synth.tracegen import Trace
from tests.helpers import ForcedRouteModel, load_golden


def test_hand_worked_trace():
    g, tr = load_golden("proxy_hand.json")
    m, px, e = g["model"], g["proxy"], g["expected"]
    out = ob.replay_proxy(tr, R=m["R"], batch=m["batch"], cache_blocks=m["cache_blocks"], block_tokens=m["block_tokens"],
                          prefill_ms_per_token=m["prefill_ms_per_token"], decode_ms_per_token=m["decode_ms_per_token"],
                          rtt_true=px["rtt_true"], probe_ms=px["probe_ms"], alpha=px["alpha"],
                          index_blocks=px["index_blocks"], w=g["w"], scale=g["scale"])
    assert out.route.tolist() == e["route"] and out.hit_blocks.tolist() == e["hit_blocks"]
    assert out.believed_hit.tolist() == e["believed_hit"] and out.rtt_est.tolist() == e["rtt_est"]
    assert out.ttft_ms.tolist() == e["ttft_ms"] and out.e2e_ms.tolist() == e["e2e_ms"]
    assert out.p95_ttft_ms == e["p95_ttft_ms"] and out.p95_e2e_ms == e["p95_e2e_ms"]


def _empty(R):
    return Trace(np.zeros(0, np.int64), np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(1, np.int64),
                 np.zeros(0, np.int64))


def _estimates(rtt_true, alpha):
    rtt_true = np.asarray(rtt_true, np.float64)
    return ob.replay_proxy(_empty(rtt_true.shape[1]), R=rtt_true.shape[1], batch=1, cache_blocks=0,
                           prefill_ms_per_token=0.05, rtt_true=rtt_true, alpha=alpha, w=[1, 1, 1]).rtt_est


def test_moving_average_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.uniform(1.0, 300.0, (40, 5))
    assert np.array_equal(_estimates(x, 1.0), x)                              # alpha 1: the latest probe
    const = np.tile(rng.uniform(1.0, 300.0, 5), (40, 1))
    np.testing.assert_allclose(_estimates(const, 0.3), const, rtol=1e-15)     # constant series: itself
    # step from x0 to x1 after the first probe: est_e = x1 + (x0 - x1) (1 - alpha)^e
    x0, x1, alpha = 200.0, 40.0, 0.2
    step = np.full((30, 1), x1)
    step[0] = x0
    e = np.arange(30)
    np.testing.assert_allclose(_estimates(step, alpha)[:, 0], x1 + (x0 - x1) * (1 - alpha) ** e, rtol=1e-13)
    # the explicit weighted sum: est_e = (1-a)^e x_0 + sum_{j>=1} a (1-a)^(e-j) x_j
    alpha = 0.35
    got = _estimates(x, alpha)
    for e in (1, 7, 39):
        wts = np.array([(1 - alpha) ** e] + [alpha * (1 - alpha) ** (e - j) for j in range(1, e + 1)])
        np.testing.assert_allclose(got[e], (wts[:, None] * x[:e + 1]).sum(0), rtol=1e-13)
    # dyadic alpha: exact
    assert _estimates([[8.0], [16.0], [0.0], [4.0]], 0.5)[:, 0].tolist() == [8.0, 12.0, 6.0, 5.0]


@pytest.mark.parametrize("scale", [1.0, 0.5, 1.7, 3.0])
def test_probe_epochs_recovered_from_latencies(scale):
    """One replica, no service time: ttft = the true RTT of the request's epoch; two replicas and weights (1, 0, 0):
    the route is the argmin of that epoch's estimates.  Requests sit on and next to the epoch boundaries."""
    probe, E = 1000, 7
    base = np.array([0, 1, 999, 1000, 1001, 1999, 2000, 2500, 3000, 3000, 4999, 5000, 5999, 6000, 6001, 9000, 50000])
    ts = np.unique(np.concatenate([base, np.ceil(base / scale).astype(np.int64), np.floor(base / scale).astype(np.int64)]))
    N = ts.size
    tr = Trace(ts.astype(np.int64), np.full(N, 10, np.int32), np.zeros(N, np.int32), np.arange(N + 1, dtype=np.int64),
               np.arange(1, N + 1, dtype=np.int64))
    t = ts.astype(np.float64) * scale
    epoch = np.array([max(e for e in range(E) if e * probe <= x) for x in t])
    true1 = np.arange(1, E + 1, dtype=np.float64).reshape(E, 1) * 16.0
    out = ob.replay_proxy(tr, R=1, batch=64, cache_blocks=0, prefill_ms_per_token=0.0, decode_ms_per_token=0.0,
                          rtt_true=true1, probe_ms=probe, alpha=0.5, w=[1, 1, 1], scale=scale)
    np.testing.assert_allclose(out.ttft_ms, true1[epoch, 0], rtol=1e-12)
    assert len(set(epoch.tolist())) == E
    # estimates alternate in favour of replica 0 / replica 1 from epoch to epoch (alpha 1: estimate = truth)
    true2 = np.array([[10.0, 20.0] if e % 2 == 0 else [20.0, 10.0] for e in range(E)])
    out = ob.replay_proxy(tr, R=2, batch=64, cache_blocks=0, prefill_ms_per_token=0.0, decode_ms_per_token=0.0,
                          rtt_true=true2, probe_ms=probe, alpha=1.0, w=[1, 0, 0], scale=scale)
    assert out.route.tolist() == (epoch % 2).tolist()
    # and with smoothing the score side lags the truth: weight only on RTT, series that flips once
    flip = np.array([[10.0, 20.0]] + [[40.0, 20.0]] * (E - 1))
    out = ob.replay_proxy(tr, R=2, batch=64, cache_blocks=0, prefill_ms_per_token=0.0, decode_ms_per_token=0.0,
                          rtt_true=flip, probe_ms=probe, alpha=0.25, w=[1, 0, 0], scale=scale)
    est0 = out.rtt_est[:, 0]                      # 10, 17.5, 23.125, ...: above 20 from epoch 2 on
    assert out.route.tolist() == (est0[epoch] > 20.0).astype(int).tolist() and est0[1] < 20.0 < est0[2]


def test_reductions_to_the_plain_replay():
    wl = tg.config(2, 5000)
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token)
    a = ob.replay(wl.trace, rtt_ms=wl.rtt_ms, w=wl.params[0], scale=wl.scale[0], **kw)
    # constant RTTs, truthful index
    b = ob.replay_proxy(wl.trace, rtt_true=np.tile(wl.rtt_ms, (9, 1)), alpha=0.5, w=wl.params[0], scale=wl.scale[0], **kw)
    assert np.array_equal(a.route, b.route) and np.array_equal(a.hit_blocks, b.hit_blocks)
    assert np.array_equal(b.believed_hit, b.hit_blocks)
    assert np.array_equal(a.ttft_ms, b.ttft_ms) and np.array_equal(a.e2e_ms, b.e2e_ms)
    # replicas that never evict: an index that never forgets is right
    kw0 = dict(kw, cache_blocks=0)
    a = ob.replay(wl.trace, rtt_ms=wl.rtt_ms, w=wl.params[0], scale=wl.scale[0], **kw0)
    c = ob.replay_proxy(wl.trace, rtt_true=wl.rtt_ms[None, :], index_blocks=0, w=wl.params[0], scale=wl.scale[0], **kw0)
    assert np.array_equal(a.route, c.route) and np.array_equal(c.believed_hit, c.hit_blocks)
    assert np.array_equal(a.ttft_ms, c.ttft_ms) and np.array_equal(a.e2e_ms, c.e2e_ms)
    # an index with the replicas' own capacity evicts exactly what they evict
    a = ob.replay(wl.trace, rtt_ms=wl.rtt_ms, w=wl.params[0], scale=wl.scale[0], **kw)
    d = ob.replay_proxy(wl.trace, rtt_true=wl.rtt_ms[None, :], index_blocks=wl.cache_blocks, w=wl.params[0],
                        scale=wl.scale[0], **kw)
    assert np.array_equal(a.route, d.route) and np.array_equal(d.believed_hit, d.hit_blocks)
    assert np.array_equal(a.ttft_ms, d.ttft_ms) and np.array_equal(a.e2e_ms, d.e2e_ms)


@pytest.mark.parametrize("seed", range(6))
def test_forced_route_model_agrees(seed):
    """The oracle's routes, dictated to an independent pure-Python model with the same imperfect knowledge, are that
    model's own argmin choices, and its latencies, hits and believed hits are the oracle's."""
    rng = np.random.default_rng(seed)
    R, B, C = int(rng.integers(2, 5)), int(rng.integers(1, 4)), int(rng.choice([6, 9, 20]))
    tr = tg.random_small(20 + seed, 150, R, n_ids=25, max_blocks=5, gap_ms=int(rng.integers(5, 60)))
    E = 6
    true = np.round(rng.uniform(2.0, 200.0, (E, R)), 1)
    px = dict(rtt_true=true.tolist(), probe_ms=700, alpha=float(rng.choice([0.125, 0.3, 1.0])),
              index_blocks=[0, -1, 2 * C, C + 3, 0, 3 * C][seed])
    w = [1.0, 1.0, 0.5]
    out = ob.replay_proxy(tr, R=R, batch=B, cache_blocks=C, prefill_ms_per_token=0.05, decode_ms_per_token=3.0,
                          rtt_true=true, probe_ms=700, alpha=px["alpha"], index_blocks=px["index_blocks"], w=w, scale=1.5,
                          debug=True)
    fm = ForcedRouteModel(tr, R, B, C, 512, 0.05, 3.0, true[0], w, 1.5, proxy=px).run(out.route.tolist())
    assert fm["consistent"]
    assert fm["hit"] == out.hit_blocks.tolist() and fm["believed"] == out.believed_hit.tolist()
    np.testing.assert_allclose(fm["score"], out.score, rtol=1e-12)
    np.testing.assert_allclose(fm["ttft"], out.ttft_ms, rtol=1e-12)
    np.testing.assert_allclose(fm["e2e"], out.e2e_ms, rtol=1e-12)
    if px["index_blocks"] >= 0:
        assert (out.believed_hit >= out.hit_blocks).all() and (out.believed_hit > out.hit_blocks).any()


def test_a_stale_index_only_overestimates_and_misleads():
    wl = tg.config(2, 6000)
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token, rtt_true=wl.rtt_ms[None, :], w=[0.5, 1.0, 0.1], scale=4.0)
    good = ob.replay_proxy(wl.trace, **kw)
    stale = ob.replay_proxy(wl.trace, index_blocks=0, **kw)
    assert (stale.believed_hit >= stale.hit_blocks).all() and (stale.believed_hit > stale.hit_blocks).mean() > 0.1
    assert np.array_equal(good.believed_hit, good.hit_blocks)
    # the misled proxy routes differently and finds fewer blocks really cached
    assert (stale.route != good.route).any() and stale.hit_blocks.sum() < good.hit_blocks.sum()
    # an index that forgets, but later than the replicas: still one-sided, and wrong less often
    lag = ob.replay_proxy(wl.trace, index_blocks=2 * wl.cache_blocks, **kw)
    assert (lag.believed_hit >= lag.hit_blocks).all()
    assert 0 < (lag.believed_hit > lag.hit_blocks).sum() < (stale.believed_hit > stale.hit_blocks).sum()

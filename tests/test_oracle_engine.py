"""CPU pins of the oracle's engine model of a replica (continuous batching with a maximum number of concurrent
requests and a KV-token budget, decode slow-down under occupancy, per-replica rates; Sec. 2.2, Sec. 5 "Exploiting
Continuous Batching", Sec. 7): two hand-worked traces, a time-stepped simulation of the admission rule on
integer-valued inputs, closed forms (serial server, simultaneous arrivals), the reduction to the linear model,
independence of the replicas under a route-only policy, and the model's invariants rebuilt from its outputs."""
import numpy as np
import pytest

from oracle import binding as ob
from synth import tracegen as tg
from synth.tracegen import Trace
from tests.helpers import load_golden


def _engine_kwargs(g):
    m = g["model"]
    return dict(R=m["R"], batch=m["batch"], cache_blocks=m["cache_blocks"], block_tokens=m["block_tokens"],
                prefill_ms_per_token=m["prefill_ms_per_token"], engine=m["engine"], rtt_ms=g["rtt_ms"], w=g["w"],
                scale=g["scale"])


@pytest.mark.parametrize("name", ["engine_hand_A.json", "engine_hand_B.json"])
def test_hand_worked_traces(name):
    g, tr = load_golden(name)
    out = ob.replay_engine(tr, **_engine_kwargs(g))
    e = g["expected"]
    assert out.route.tolist() == e["route"] and out.hit_blocks.tolist() == e["hit_blocks"]
    assert out.ttft_ms.tolist() == e["ttft_ms"] and out.e2e_ms.tolist() == e["e2e_ms"]
    assert out.p95_ttft_ms == e["p95_ttft_ms"] and out.p95_e2e_ms == e["p95_e2e_ms"]


def _tick_simulation(tr, route, uncached, R, B, rtt, a_pf, a_dec, kv_budget, slowdown, scale):
    """Replicas stepped one millisecond at a time (all inputs integers, so every event falls on a tick): at each
    tick requests whose last token is out leave, then the head of the arrival-ordered queue is admitted while a
    slot is free and its tokens fit (or nothing is running)."""
    N = tr.N
    ttft, e2e = np.zeros(N), np.zeros(N)
    for i in range(R):
        mine = [r for r in range(N) if route[r] == i]
        half = rtt[i] // 2
        queue = [(int(tr.ts_ms[r]) * scale + half, r) for r in mine]      # arrival order = request order
        running = []                                                       # (end, tokens)
        tick = 0
        while queue:
            running = [x for x in running if x[0] > tick]
            while queue and queue[0][0] <= tick:
                arr, r = queue[0]
                tok = int(tr.in_len[r]) + int(tr.out_len[r])
                held = sum(x[1] for x in running)
                if len(running) >= B or (running and kv_budget[i] and held + tok > kv_budget[i]):
                    break
                queue.pop(0)
                first = tick + a_pf[i] * int(uncached[r])
                end = first + a_dec[i] * int(tr.out_len[r]) * (1 + slowdown * len(running))
                t = int(tr.ts_ms[r]) * scale
                ttft[r] = first + half - t
                e2e[r] = end + half - t
                running.append((end, tok))
                running = [x for x in running if x[0] > tick]               # a request without work is gone at once
            tick += 1
    return ttft, e2e


@pytest.mark.parametrize("seed", range(24))
def test_time_stepped_simulation_of_admission(seed):
    rng = np.random.default_rng(500 + seed)
    R = int(rng.integers(1, 4))
    B = int(rng.integers(1, 5))
    bt = 4
    tr = tg.random_small(seed, 60, R, n_ids=30, max_blocks=4, gap_ms=int(rng.integers(1, 12)), block_tokens=bt)
    # small outputs so that runs overlap without the horizon exploding; zero-output requests included
    tr = Trace(tr.ts_ms, tr.in_len, rng.integers(0, 6, tr.N).astype(np.int32), tr.blk_off, tr.hash_ids)
    rtt = (2 * rng.integers(0, 6, R)).astype(float)
    a_pf = rng.integers(0, 3, R).astype(float)
    a_dec = rng.integers(1, 4, R).astype(float)
    most = int((tr.in_len + tr.out_len).max())
    kv = [int(rng.choice([0, most // 2 + 1, most, 2 * most, 5 * most])) for _ in range(R)]
    slowdown = float(rng.integers(0, 3))
    scale = int(rng.integers(1, 3))
    policy = ["cost-model", "least-request", "random"][seed % 3]
    out = ob.replay_engine(tr, R=R, batch=B, cache_blocks=0, prefill_ms_per_token=1.0, block_tokens=bt, rtt_ms=rtt,
                           engine=dict(prefill_ms_per_token=a_pf, decode_ms_per_token=a_dec, kv_tokens=kv,
                                       slowdown=slowdown), w=[0.5, 1.0, 1.0], policy=policy, seed=seed, scale=scale)
    uncached = tr.in_len - np.minimum(tr.in_len, bt * out.hit_blocks.astype(np.int64))
    ttft, e2e = _tick_simulation(tr, out.route, uncached, R, B, rtt.astype(int), a_pf.astype(int), a_dec.astype(int),
                                 kv, int(slowdown), scale)
    assert np.array_equal(out.ttft_ms, ttft) and np.array_equal(out.e2e_ms, e2e)


def test_reduces_to_the_linear_model():
    """No slow-down, no budget, equal rates: bit for bit the B-slot model (pinned by its own tests)."""
    for cfg, head in ((1, None), (2, 3000)):
        wl = tg.config(cfg)
        tr = wl.trace if head is None else wl.trace.head(head)
        kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
                  rtt_ms=wl.rtt_ms, w=wl.params[1], scale=wl.scale[1])
        a = ob.replay(tr, decode_ms_per_token=wl.decode_ms_per_token, **kw)
        for kv in (None, [0] * wl.R, [10 ** 12] * wl.R):
            b = ob.replay_engine(tr, engine=dict(prefill_ms_per_token=[wl.prefill_ms_per_token] * wl.R,
                                                 decode_ms_per_token=[wl.decode_ms_per_token] * wl.R, kv_tokens=kv,
                                                 slowdown=0.0), **kw)
            assert np.array_equal(a.route, b.route) and np.array_equal(a.hit_blocks, b.hit_blocks)
            assert np.array_equal(a.ttft_ms, b.ttft_ms) and np.array_equal(a.e2e_ms, b.e2e_ms)


def test_budget_of_one_token_is_a_serial_server():
    """Nothing fits beside anything: one request at a time in arrival order (Lindley's recurrence), never slowed."""
    tr = tg.random_small(7, 200, 1, n_ids=40, max_blocks=6, gap_ms=300)
    a_pf, a_dec, rtt = 0.07, 13.0, 30.0
    out = ob.replay_engine(tr, R=1, batch=8, cache_blocks=0, prefill_ms_per_token=a_pf, rtt_ms=[rtt],
                           engine=dict(prefill_ms_per_token=[a_pf], decode_ms_per_token=[a_dec], kv_tokens=[1],
                                       slowdown=3.0))
    uncached = tr.in_len - np.minimum(tr.in_len, 512 * out.hit_blocks.astype(np.int64))
    end = 0.0
    for r in range(tr.N):
        t = float(tr.ts_ms[r])
        start = max(t + 0.5 * rtt, end)
        first = start + a_pf * float(uncached[r])
        end = first + a_dec * float(tr.out_len[r]) * 1.0
        assert out.ttft_ms[r] == (first + 0.5 * rtt) - t and out.e2e_ms[r] == (end + 0.5 * rtt) - t


def test_simultaneous_arrivals_slow_each_other_down():
    """Closed form: N requests at t = 0 on one replica with room for all: the j-th is admitted at once beside j
    others, so e2e_j = a_pf L_j + a_dec O_j (1 + slowdown j)."""
    N = 12
    L = np.arange(1, N + 1, dtype=np.int32) * 100
    O = np.arange(N, 0, -1, dtype=np.int32) * 3
    tr = Trace(np.zeros(N, np.int64), L, O, np.arange(N + 1, dtype=np.int64), np.arange(1, N + 1, dtype=np.int64))
    out = ob.replay_engine(tr, R=1, batch=N, cache_blocks=0, prefill_ms_per_token=0.5, rtt_ms=[0.0],
                           engine=dict(prefill_ms_per_token=[0.5], decode_ms_per_token=[2.0], kv_tokens=None,
                                       slowdown=0.25))
    j = np.arange(N)
    assert np.array_equal(out.ttft_ms, 0.5 * L)
    assert np.array_equal(out.e2e_ms, 0.5 * L + 2.0 * O * (1 + 0.25 * j))
    # with one slot fewer the last request waits for the first end, and is then slowed by those still running
    out2 = ob.replay_engine(tr, R=1, batch=N - 1, cache_blocks=0, prefill_ms_per_token=0.5, rtt_ms=[0.0],
                            engine=dict(prefill_ms_per_token=[0.5], decode_ms_per_token=[2.0], kv_tokens=None,
                                        slowdown=0.25))
    ends = out.e2e_ms[:N - 1]
    s = ends.min()
    running = int((ends > s).sum())
    assert out2.ttft_ms[N - 1] == s + 0.5 * L[N - 1]
    assert out2.e2e_ms[N - 1] == (s + 0.5 * L[N - 1]) + (2.0 * O[N - 1]) * (1 + 0.25 * running)


def test_replicas_are_independent_under_a_route_only_policy():
    """Random routing ignores the state: every replica then serves its own sub-trace exactly as a one-replica
    system with that replica's rates, budget and RTT would (a wrong per-replica index shows here)."""
    R = 4
    tr = tg.random_small(11, 400, R, n_ids=60, max_blocks=5, gap_ms=25)
    rtt = np.array([10.0, 40.0, 90.0, 200.0])
    eng = dict(prefill_ms_per_token=[0.03, 0.05, 0.08, 0.02], decode_ms_per_token=[15.0, 25.0, 10.0, 30.0],
               kv_tokens=[0, 9000, 4000, 20000], slowdown=0.3)
    out = ob.replay_engine(tr, R=R, batch=3, cache_blocks=12, prefill_ms_per_token=0.05, rtt_ms=rtt, engine=eng,
                           policy="random", seed=99)
    assert len(set(out.route.tolist())) == R
    for i in range(R):
        idx = np.nonzero(out.route == i)[0]
        nblk = np.diff(tr.blk_off)[idx]
        sub = Trace(tr.ts_ms[idx], tr.in_len[idx], tr.out_len[idx], np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64),
                    np.concatenate([tr.ids_of(int(r)) for r in idx]).astype(np.int64))
        one = ob.replay_engine(sub, R=1, batch=3, cache_blocks=12, prefill_ms_per_token=0.05, rtt_ms=[rtt[i]],
                               engine=dict(prefill_ms_per_token=[eng["prefill_ms_per_token"][i]],
                                           decode_ms_per_token=[eng["decode_ms_per_token"][i]],
                                           kv_tokens=[eng["kv_tokens"][i]], slowdown=0.3))
        assert np.array_equal(one.hit_blocks, out.hit_blocks[idx])
        assert np.array_equal(one.ttft_ms, out.ttft_ms[idx]) and np.array_equal(one.e2e_ms, out.e2e_ms[idx])


def test_invariants_rebuilt_from_the_outputs():
    """On a loaded mid-size run: never more than B requests running on a replica, their KV tokens within the
    budget unless one runs alone, admissions in arrival order, every request admitted as early as those allow."""
    wl = tg.config(1)
    tr, R, B = wl.trace, wl.R, wl.batch
    rng = np.random.default_rng(3)
    a_pf = wl.prefill_ms_per_token * rng.uniform(0.5, 2.0, R)
    a_dec = wl.decode_ms_per_token * rng.uniform(0.5, 2.0, R)
    kv = np.full(R, 3 * int((tr.in_len + tr.out_len).max()), np.int64)
    slowdown = 0.1
    out = ob.replay_engine(tr, R=R, batch=B, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
                           rtt_ms=wl.rtt_ms, engine=dict(prefill_ms_per_token=a_pf, decode_ms_per_token=a_dec,
                                                         kv_tokens=kv, slowdown=slowdown), w=wl.params[0], scale=4.0)
    t = tr.ts_ms * 4.0
    uncached = tr.in_len - np.minimum(tr.in_len, 512 * out.hit_blocks.astype(np.int64))
    waited = 0
    for i in range(R):
        idx = np.nonzero(out.route == i)[0]
        half = 0.5 * wl.rtt_ms[i]
        start = t[idx] + out.ttft_ms[idx] - half - a_pf[i] * uncached[idx]
        end = t[idx] + out.e2e_ms[idx] - half
        tok = (tr.in_len[idx] + tr.out_len[idx]).astype(np.int64)
        eps = 1e-6
        assert (np.diff(start) >= -eps).all()                                   # arrival order
        assert (start >= t[idx] + half - eps).all()
        for j in range(len(idx)):
            run = (end[:j] > start[j] + eps)                                    # earlier ones still running
            n = int(run.sum())
            assert n < B
            assert n == 0 or tok[:j][run].sum() + tok[j] <= kv[i]
            # the decode time carries the slow-down of exactly those
            dec = end[j] - start[j] - a_pf[i] * uncached[idx[j]]
            assert abs(dec - a_dec[i] * tr.out_len[idx[j]] * (1 + slowdown * n)) <= 1e-6 * max(1.0, dec)
            # admitted as early as allowed: just before its admission it could not have been
            lower = max(t[idx[j]] + half, start[j - 1] if j else 0.0)
            if start[j] > lower + eps:
                waited += 1
                before = end[:j] > start[j] - eps                               # running just before
                nb = int(before.sum())
                assert nb >= B or (nb > 0 and tok[:j][before].sum() + tok[j] > kv[i])
    assert waited > 50                                                          # the run does exercise waiting

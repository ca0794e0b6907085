"""CPU-only pins of the replay oracle against things other than itself: hand-worked traces, brute force
with an independent forced-route model, weight special cases, post-hoc recomputation of the load signal,
textbook queueing recurrences, a list-based LRU, sorted-array percentiles."""
import itertools

import numpy as np
import pytest

from oracle import binding as ob
from synth import tracegen as tg
from tests.helpers import ForcedRouteModel, load_golden, model_kwargs


# ---------------------------------------------------------------- hand-worked traces (tests/golden)

@pytest.mark.parametrize("name", ["hand_trace_A.json", "hand_trace_B.json", "hand_trace_D.json"])
def test_hand_traces_scores_routes_latencies(name):
    g, tr = load_golden(name)
    r = ob.replay(tr, debug=True, **model_kwargs(g))
    e = g["expected"]
    assert r.score.tolist() == e["score"]
    assert r.q.tolist() == e["q_before"]
    assert r.route.tolist() == e["route"]
    assert r.hit_blocks.tolist() == e["hit_blocks"]
    assert r.ttft_ms.tolist() == e["ttft_ms"]
    assert r.e2e_ms.tolist() == e["e2e_ms"]
    assert r.p95_ttft_ms == e["p95_ttft_ms"] and r.p95_e2e_ms == e["p95_e2e_ms"]


def test_hand_trace_lru():
    g, tr = load_golden("hand_trace_C.json")
    r = ob.replay(tr, debug=True, **model_kwargs(g))
    e = g["expected"]
    assert r.route.tolist() == e["route"]
    assert r.hit_blocks.tolist() == e["hit_blocks"]
    assert r.size.tolist() == e["cache_size_after"]
    assert r.ttft_ms.tolist() == e["ttft_ms"]
    assert r.e2e_ms.tolist() == e["e2e_ms"]


# ---------------------------------------------------------------- brute force over every route sequence

@pytest.mark.parametrize("seed,C,B,consistent", [(0, 0, 1, True), (1, 5, 1, True), (2, 6, 2, False),
                                                 (3, 0, 2, False), (4, 7, 1, True)])
def test_bruteforce_all_route_sequences(seed, C, B, consistent):
    """R=2, N=10: among all 2^10 dictated route sequences exactly one is self-consistent with 'each
    choice is the lowest-index minimum of Eq. 3 given the state its predecessors induce'; the oracle must
    produce that one, with the same hits and latencies."""
    R, N = 2, 10
    tr = tg.random_small(seed, N, R, n_ids=10, max_blocks=5, consistent=consistent, gap_ms=60)
    rng = np.random.default_rng(seed)
    w = rng.uniform(0.0, 2.0, 3)
    rtt = [10.0, 35.0]
    a_pf, a_dec = 0.05, 20.0
    fm = ForcedRouteModel(tr, R, B, C, 512, a_pf, a_dec, rtt, w, 1.0)
    good = []
    for routes in itertools.product(range(R), repeat=N):
        out = fm.run(routes)
        if out["consistent"]:
            good.append((routes, out))
    assert len(good) == 1
    routes, out = good[0]
    r = ob.replay(tr, R=R, batch=B, cache_blocks=C, prefill_ms_per_token=a_pf, decode_ms_per_token=a_dec,
                  rtt_ms=rtt, w=w, scale=1.0, debug=True)
    assert r.route.tolist() == list(routes)
    assert r.hit_blocks.tolist() == out["hit"]
    np.testing.assert_allclose(r.ttft_ms, out["ttft"], rtol=1e-12)
    np.testing.assert_allclose(r.e2e_ms, out["e2e"], rtol=1e-12)
    np.testing.assert_allclose(r.score, out["score"], rtol=1e-12)
    assert r.q.tolist() == out["q"]


# ---------------------------------------------------------------- weight special cases (Eq. 3)

def _cfg1(w, n=600, **over):
    wl = tg.config(1, n)
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token, rtt_ms=wl.rtt_ms, w=w, scale=1.0)
    kw.update(over)
    return wl, ob.replay(wl.trace, debug=True, **kw)


def test_all_zero_weights_route_to_replica_zero():
    _, r = _cfg1([0.0, 0.0, 0.0])
    assert (r.route == 0).all()


def test_rtt_only_routes_to_nearest_replica():
    # the "reward hacking" regime: no queue weight, RTT dominant -> 100 % of traffic to the nearest replica
    # (Sec. 5 "Exploiting Continuous Batching", Appendix load ablation)
    _, r = _cfg1([1.0, 0.0, 0.0], rtt_ms=[40.0, 10.0, 10.0, 300.0])
    assert (r.route == 1).all()          # lowest index among the two nearest


def test_prefix_only_is_prefix_cache_policy():
    """w=(0,1,0): route = lowest-index replica with the most cached prefix tokens, recomputed post hoc from
    the routes alone (unbounded cache: replica i holds every block of every earlier request sent to it)."""
    wl, r = _cfg1([0.0, 1.0, 0.0])
    tr = wl.trace
    held = [set() for _ in range(wl.R)]
    for q in range(tr.N):
        ids = tr.ids_of(q).tolist()
        L = int(tr.in_len[q])
        hit = []
        for i in range(wl.R):
            m = 0
            while m < len(ids) and ids[m] in held[i]:
                m += 1
            hit.append(min(L, 512 * m))
        best = max(range(wl.R), key=lambda i: (hit[i], -i))
        assert r.route[q] == best
        assert r.hit_blocks[q] * 512 >= hit[best] and min(L, int(r.hit_blocks[q]) * 512) == hit[best]
        held[best].update(ids)
    assert r.hit_blocks.max() > 0


def _posthoc_q(tr, route, e2e, R, scale):
    t = tr.ts_ms.astype(np.float64) * scale
    done = t + e2e
    q = np.zeros((tr.N, R), np.int64)
    near_tie = False
    for r in range(tr.N):
        for j in range(r):
            if done[j] > t[r]:
                q[r, route[j]] += int(tr.in_len[j])
            if abs(done[j] - t[r]) < 1e-6:
                near_tie = True
    return q, near_tie


def test_load_signal_is_tokens_without_completion_event():
    """Eq. 2: the queue input of replica i at request r is the input tokens of earlier requests routed to i
    whose completion event has not yet reached the proxy -- recomputed O(N^2) from (route, t + e2e)."""
    wl, r = _cfg1([0.7, 1.0, 0.3], n=500)
    q, near = _posthoc_q(wl.trace, r.route, r.e2e_ms, wl.R, 1.0)
    assert not near
    assert (q == r.q).all()
    assert r.q.max() > 0


def test_queue_only_routes_to_least_loaded():
    wl, r = _cfg1([0.0, 0.0, 1.0], n=500)
    q, near = _posthoc_q(wl.trace, r.route, r.e2e_ms, wl.R, 1.0)
    assert not near
    assert (r.route == q.argmin(axis=1)).all()      # numpy argmin returns the lowest index on ties
    assert len(set(r.route.tolist())) == wl.R


@pytest.mark.parametrize("k", [-3, 1, 5])
def test_only_weight_ratios_matter(k):
    """Sec. 2.3: only the ratio of weights matters -- scaling all three by a power of two (exact in fp64)
    leaves every route, hit count and latency bit-identical."""
    w = np.array([0.37, 1.0, 0.21])
    _, a = _cfg1(w)
    _, b = _cfg1(w * 2.0 ** k)
    assert (a.route == b.route).all() and (a.hit_blocks == b.hit_blocks).all()
    assert (a.ttft_ms == b.ttft_ms).all() and (a.e2e_ms == b.e2e_ms).all()
    assert (a.score * 2.0 ** k == b.score).all()


def test_weights_change_routes():
    # guards against a replay that ignores its weights
    _, a = _cfg1([1.0, 1.0, 0.05])
    _, b = _cfg1([0.05, 1.0, 1.5])
    assert (a.route != b.route).any()


# ---------------------------------------------------------------- service model: textbook recurrences

def _unique_trace(N, seed, gap=30):
    rng = np.random.default_rng(seed)
    ts = np.cumsum(rng.integers(0, gap, N)).astype(np.int64)
    nblk = rng.integers(1, 4, N)
    off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64)
    ids = np.arange(1, off[-1] + 1, dtype=np.int64)          # every block new: no cache hits
    return tg.Trace(ts, (nblk * 512).astype(np.int32), rng.integers(1, 5, N).astype(np.int32), off, ids)


def test_single_server_is_lindley_recursion():
    """R=1, B=1: waiting times follow W_{r+1} = max(0, W_r + S_r - A_r) (single-server FIFO queue);
    TTFT = RTT + wait + prefill (Eq. 1).  Constants exact in binary, so equality is exact."""
    tr = _unique_trace(300, 7)
    a_pf, a_dec, rtt = 0.0625, 16.0, 8.0
    r = ob.replay(tr, R=1, batch=1, cache_blocks=0, prefill_ms_per_token=a_pf, decode_ms_per_token=a_dec,
                  rtt_ms=[rtt], w=[1, 1, 1])
    W = 0.0
    for k in range(tr.N):
        pf = a_pf * tr.in_len[k]
        S = pf + a_dec * tr.out_len[k]
        assert r.ttft_ms[k] == rtt + W + pf
        assert r.e2e_ms[k] == rtt + W + S
        assert r.hit_blocks[k] == 0
        if k + 1 < tr.N:
            W = max(0.0, W + S - float(tr.ts_ms[k + 1] - tr.ts_ms[k]))
    assert (r.ttft_ms > rtt + a_pf * tr.in_len).any()     # some request did wait


@pytest.mark.parametrize("B", [2, 3, 8])
def test_multi_server_is_kiefer_wolfowitz(B):
    """R=1, B>1: FIFO B-server queue.  Workload vector kept sorted; the arriving customer waits for the
    smallest component, its service time is added there, the inter-arrival gap is subtracted everywhere."""
    tr = _unique_trace(400, 11, gap=14)
    a_pf, a_dec, rtt = 0.0625, 16.0, 8.0
    r = ob.replay(tr, R=1, batch=B, cache_blocks=0, prefill_ms_per_token=a_pf, decode_ms_per_token=a_dec,
                  rtt_ms=[rtt], w=[1, 1, 1])
    V = [0.0] * B
    for k in range(tr.N):
        pf = a_pf * tr.in_len[k]
        S = pf + a_dec * tr.out_len[k]
        V.sort()
        assert r.ttft_ms[k] == rtt + V[0] + pf
        V[0] += S
        if k + 1 < tr.N:
            A = float(tr.ts_ms[k + 1] - tr.ts_ms[k])
            V = [max(0.0, v - A) for v in V]
    assert (r.ttft_ms > rtt + a_pf * tr.in_len).any()


def test_large_time_scale_gives_closed_form():
    """Stretching the gaps (Table 3: larger time_scale = lighter load) removes all waiting and all
    outstanding load: TTFT = RTT of the chosen replica + a_pf * uncached tokens, E2E adds the decode."""
    wl = tg.config(1, 400)
    w = [1.0, 1.0, 0.5]
    tr = wl.trace.head(400)
    tr.ts_ms = np.arange(400, dtype=np.int64) * 25               # distinct timestamps, 25 ms apart
    r = ob.replay(tr, R=wl.R, batch=wl.batch, cache_blocks=0, prefill_ms_per_token=0.0625,
                  decode_ms_per_token=16.0, rtt_ms=wl.rtt_ms, w=w, scale=4096.0, debug=True)
    assert (r.q == 0).all()
    u = tr.in_len - np.minimum(tr.in_len, 512 * r.hit_blocks.astype(np.int64))
    # every constant is exact in binary (RTTs are integers, a_pf = 1/16), so the closed form is exact
    assert (r.ttft_ms == wl.rtt_ms[r.route] + 0.0625 * u).all()
    assert (r.e2e_ms - r.ttft_ms == 16.0 * tr.out_len).all()
    assert r.hit_blocks.max() > 0


def test_saturation_trend_with_time_scale():
    # sanity trend only: lighter load cannot have a worse tail than 16x heavier load on this workload
    wl = tg.config(1)
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=0, prefill_ms_per_token=0.05, decode_ms_per_token=20.0,
              rtt_ms=wl.rtt_ms, w=[0.5, 1.0, 0.1])
    heavy = ob.replay(wl.trace, scale=0.25, **kw)
    light = ob.replay(wl.trace, scale=4.0, **kw)
    assert light.p95_ttft_ms < heavy.p95_ttft_ms


# ---------------------------------------------------------------- cache

class ListLRU:
    """Textbook recency list: touch moves to the hot end; evict from the cold end."""

    def __init__(self, C):
        self.C, self.order = C, []

    def request(self, ids):
        m = 0
        while m < len(ids) and ids[m] in self.order:
            m += 1
        mine = set(ids)
        new = [x for x in mine if x not in self.order]
        excess = len(self.order) + len(new) - self.C
        k = 0
        while excess > 0:
            if self.order[k] in mine:
                k += 1
                continue
            self.order.pop(k)
            excess -= 1
        seen = []
        for x in ids:
            if x not in seen:
                seen.append(x)
        for x in reversed(seen):                 # deepest first, root last = hottest
            if x in self.order:
                self.order.remove(x)
            self.order.append(x)
        return m


@pytest.mark.parametrize("consistent", [True, False])
@pytest.mark.parametrize("C", [5, 9, 40])
def test_lru_against_recency_list(C, consistent):
    tr = tg.random_small(21 + C, 400, 1, n_ids=30, max_blocks=5, consistent=consistent)
    r = ob.replay(tr, R=1, batch=4, cache_blocks=C, prefill_ms_per_token=0.05, decode_ms_per_token=20.0,
                  rtt_ms=[10.0], w=[1, 1, 1], debug=True)
    lru = ListLRU(C)
    for k in range(tr.N):
        assert r.hit_blocks[k] == lru.request(tr.ids_of(k).tolist())
        assert r.size[k] == len(lru.order) <= C
    assert 0 < r.hit_blocks.sum()
    assert (r.hit_blocks < np.diff(tr.blk_off)).any()          # some evictions mattered


def test_hit_tokens_never_exceed_input_tokens():
    """A partial last block: cached tokens are capped at the input length, so the prefill term of Eq. 1 is
    never negative and a full hit costs exactly zero prefill."""
    ts = np.array([0, 100000], np.int64)
    tr = tg.Trace(ts, np.array([700, 700], np.int32), np.array([1, 1], np.int32), np.array([0, 2, 4]),
                  np.array([3, 4, 3, 4]))
    r = ob.replay(tr, R=1, batch=1, cache_blocks=0, prefill_ms_per_token=0.0625, decode_ms_per_token=1.0,
                  rtt_ms=[8.0], w=[1, 1, 1])
    assert r.hit_blocks.tolist() == [0, 2]
    assert r.ttft_ms.tolist() == [8.0 + 0.0625 * 700, 8.0]


def test_capacity_error_when_request_exceeds_cache():
    tr = tg.Trace(np.array([0]), np.array([2048], np.int32), np.array([1], np.int32), np.array([0, 4]),
                  np.array([1, 2, 3, 4]))
    with pytest.raises(RuntimeError):
        ob.replay(tr, R=1, batch=1, cache_blocks=3, prefill_ms_per_token=0.05, decode_ms_per_token=1.0,
                  rtt_ms=[1.0], w=[1, 1, 1])


def test_bounded_cache_on_growing_conversations():
    """Chain-consistent trace + root-newest stamps: the cache stays prefix-closed, so the number of a
    request's blocks present equals its longest prefix match, and the size never exceeds C."""
    wl = tg.config(2, 1500)
    r = ob.replay(wl.trace, R=2, batch=8, cache_blocks=600, prefill_ms_per_token=0.05, decode_ms_per_token=20.0,
                  rtt_ms=[10.0, 20.0], w=[1.0, 1.0, 0.0], debug=True)
    assert r.size.max() == 600
    assert (r.hit_blocks <= np.diff(wl.trace.blk_off)).all()
    assert r.hit_blocks.max() > 50


# ---------------------------------------------------------------- percentile

def test_p95_is_nearest_rank_order_statistic():
    rng = np.random.default_rng(5)
    for n in [1, 2, 19, 20, 21, 100, 128, 1000, 4097]:
        x = rng.lognormal(3, 1, n)
        k = -(-95 * n // 100)                       # ceil(0.95 n)
        assert ob.p95(x) == np.sort(x)[k - 1]
        assert ob.p95(rng.permutation(x)) == ob.p95(x)
    # the tuner's 128-request window (Sec. 4): the 122nd smallest
    x = np.arange(1, 129, dtype=np.float64)[::-1].copy()
    assert ob.p95(x) == 122.0

"""Pins of the oracle's baseline policies (Sec. 4 "Baseline policies") and of the two generators they use."""
import numpy as np
import pytest

from oracle import binding as ob
from synth import tracegen as tg
from tests.helpers import ForcedRouteModel


def _kw(wl, **over):
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token, rtt_ms=wl.rtt_ms, block_tokens=wl.block_tokens)
    kw.update(over)
    return kw


def test_generators_against_their_published_answers():
    # Philox-4x32-10: the known-answer vectors distributed with the generator (zeros; digits of pi)
    assert [hex(x) for x in ob.philox4x32_10([0, 0, 0, 0], [0, 0])] == ['0x6627e8d5', '0xe169c58d', '0xbc57ac4c', '0x9b00dbd8']
    assert [hex(x) for x in ob.philox4x32_10([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0])] == \
        ['0xd16cfe09', '0x94fdcceb', '0x5001e420', '0x24126ea1']
    # SplitMix64: first outputs of the reference generator seeded with 1234567
    x, out = 1234567, []
    for _ in range(5):
        out.append(ob.splitmix64_next(x))
        x = (x + 0x9E3779B97F4A7C15) & (2**64 - 1)
    assert out == [6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431,
                   16408922859458223821]


@pytest.mark.parametrize("scale", [1.0, 3.0])
def test_least_request_is_fewest_in_flight_of_an_independent_model(scale):
    wl = tg.config(1, 700)
    res = ob.replay_policy(wl.trace, policy="least-request", scale=scale, **_kw(wl))
    fm = ForcedRouteModel(wl.trace, wl.R, wl.batch, wl.cache_blocks, wl.block_tokens, wl.prefill_ms_per_token,
                          wl.decode_ms_per_token, wl.rtt_ms, [0.0, 0.0, 0.0], scale)
    out = fm.run(res.route.tolist())
    for r in range(wl.trace.N):
        cnt = out["cnt"][r]
        assert res.route[r] == min(range(wl.R), key=lambda i: (cnt[i], i)), r
    np.testing.assert_array_equal(res.ttft_ms, out["ttft"])
    assert len(set(res.route.tolist())) == wl.R


def test_session_affinity_depends_on_the_first_block_only():
    wl = tg.config(2, 5000)
    tr = wl.trace
    a = ob.replay_policy(tr, policy="session-affinity", **_kw(wl))
    b = ob.replay_policy(tr, policy="session-affinity", scale=7.0, **_kw(wl, cache_blocks=300, batch=2))
    assert np.array_equal(a.route, b.route)                       # no state, no load, no cache involved
    first = tr.hash_ids[tr.blk_off[:-1]]
    by_first = {}
    for r in range(tr.N):
        assert by_first.setdefault(int(first[r]), int(a.route[r])) == a.route[r]      # a conversation stays put
        assert a.route[r] == ((ob.splitmix64_next(int(first[r])) >> 32) * wl.R) >> 32
    share = np.bincount([v for v in by_first.values()], minlength=wl.R) / len(by_first)
    assert share.min() > 0.5 / wl.R and share.max() < 2.0 / wl.R  # conversations spread over the replicas


def test_random_policy_is_the_counter_based_draw_and_uniform():
    wl = tg.config(2, 8000)
    a = ob.replay_policy(wl.trace, policy="random", seed=42, **_kw(wl))
    assert np.array_equal(a.route, ob.replay_policy(wl.trace, policy="random", seed=42, scale=2.0, **_kw(wl)).route)
    assert not np.array_equal(a.route, ob.replay_policy(wl.trace, policy="random", seed=43, **_kw(wl)).route)
    for r in (0, 1, 77, 7999):
        assert a.route[r] == (int(ob.philox4x32_10([r, 0, 0, 0], [42, 0])[0]) * wl.R) >> 32
    share = np.bincount(a.route, minlength=wl.R) / wl.trace.N
    assert abs(share - 1 / wl.R).max() < 4 * np.sqrt((1 / wl.R) * (1 - 1 / wl.R) / wl.trace.N)


def test_policy_latencies_follow_from_the_routes():
    # whatever picks the routes, cache and service behave as in the cost-model replay: an independent model told the
    # same routes gives the same hits and latencies
    wl = tg.config(1, 400)
    for pol, seed in (("session-affinity", 0), ("random", 5)):
        res = ob.replay_policy(wl.trace, policy=pol, seed=seed, **_kw(wl))
        fm = ForcedRouteModel(wl.trace, wl.R, wl.batch, wl.cache_blocks, wl.block_tokens, wl.prefill_ms_per_token,
                              wl.decode_ms_per_token, wl.rtt_ms, [0.0, 0.0, 0.0], 1.0)
        out = fm.run(res.route.tolist())
        assert res.hit_blocks.tolist() == out["hit"]
        np.testing.assert_array_equal(res.ttft_ms, out["ttft"])
        np.testing.assert_array_equal(res.e2e_ms, out["e2e"])

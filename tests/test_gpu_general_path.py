"""GPU parity of the online tuner, the baseline policies, the engine model of a replica and imperfect proxy knowledge
on hashed block tables -- the formulation of the cache state that assumes nothing about the trace -- against the CPU
oracle, through the C ABI: on traces that are not chain-consistent (the same id under several predecessors, at
several positions, twice in one request), where it is the only formulation, and on chain-consistent ones, where it
has to give what the segment rows give."""
import numpy as np
import pytest

import paper_2602_11688_amd as g
from synth import tracegen as tg
from tests.gpu_helpers import check_population, formulation, load
from tests.test_gpu_engine import check_engine, check_engine_online, check_engine_policy
from tests.test_gpu_online import _check as check_online
from tests.test_gpu_policies import _check as check_policy
from tests.test_gpu_proxy import _wander, check_proxy

pytestmark = pytest.mark.gpu

LO, HI = [0.05, 0.05, 0.05], [2.0, 2.0, 0.5]
PAR = [[0.5, 1.0, 0.1], [0.276, 0.5, 0.3], [2.0, 0.05, 0.05]]


def _tangled(seed, N=1500, R=6, **kw):
    """A trace that is not chain-consistent, with enough distinct ids and long enough requests that bounded caches
    evict all the time and tables are compacted."""
    kw.setdefault("n_ids", 300)
    kw.setdefault("max_blocks", 24)
    kw.setdefault("gap_ms", 6)
    tr = tg.random_small(seed, N, R, consistent=False, **kw)
    assert not load(tr).info()["chain_consistent"]
    return tr


def _engine(R, seed, kv=60000, slowdown=0.05):
    rng = np.random.default_rng(seed)
    return g.Engine(0.05 * 2.0 ** rng.uniform(-1, 1, R), 20.0 * 2.0 ** rng.uniform(-1, 1, R), np.full(R, kv, np.int64),
                    slowdown)


@pytest.mark.parametrize("cache", [0, 60, 400])
def test_online_tuner_on_a_trace_that_is_not_chain_consistent(cache):
    tr = _tangled(1)
    rtt = np.linspace(5.0, 80.0, 6)
    steps = g.online_steps(tr.N, 128, 32)
    z = np.random.default_rng(3).standard_normal((3, steps, 3))
    check_online(tr, g.Model(6, 4, cache, 0.05, 20.0), rtt, PAR, z, [1.0, 0.5, 2.0], 128, 32, lo=LO, hi=HI, sigma0=0.5)


@pytest.mark.parametrize("policy", ["least-request", "session-affinity", "random"])
def test_policies_on_a_trace_that_is_not_chain_consistent(policy):
    tr = _tangled(2)
    seeds = np.array([7, 2**40 + 1], np.uint64) if policy == "random" else None
    got = check_policy(tr, g.Model(6, 4, 80, 0.05, 20.0), np.linspace(5.0, 80.0, 6), policy, [1.0, 0.25], seeds)
    assert len(set(got["route"][0].tolist())) == 6


def test_engine_model_on_a_trace_that_is_not_chain_consistent():
    tr = _tangled(3)
    rtt = np.linspace(5.0, 80.0, 6)
    model = g.Model(6, 4, 80, 0.05, 20.0)
    eng = _engine(6, 1)
    check_engine(tr, model, eng, rtt, PAR, [1.0, 0.5, 2.0])
    check_engine_policy(tr, model, eng, rtt, "least-request", [1.0])
    check_engine_policy(tr, model, eng, rtt, "random", [1.0, 3.0], np.array([5, 6], np.uint64))
    steps = g.online_steps(tr.N, 64, 16)
    z = np.random.default_rng(4).standard_normal((2, steps, 3))
    check_engine_online(tr, model, eng, rtt, PAR[:2], z, 1.0, 64, 16, LO, HI, 0.5)


@pytest.mark.parametrize("index", [-1, "cache", "twice", "larger", 0])
def test_proxy_knowledge_on_a_trace_that_is_not_chain_consistent(index):
    tr = _tangled(4)
    cache = 80
    model = g.Model(6, 4, cache, 0.05, 20.0)
    blocks = {"cache": cache, "twice": 2 * cache, "larger": 5 * cache}.get(index, index)
    px = g.Proxy(_wander(np.linspace(5.0, 80.0, 6), 9, seed=5), 1000, 0.3, blocks)
    # (the tables also hold what only the index still holds: all the trace's ids when it never forgets)
    with formulation(1, table_factor_percent=800):
        got = check_proxy(tr, model, px, PAR, [1.0, 0.5, 2.0])
    if index in ("twice", "larger", 0):
        assert (got["believed"] > got["hit"]).any()          # the index remembers what the replica evicted


def test_proxy_knowledge_with_the_engine_model_and_the_tuner_on_block_tables():
    tr = _tangled(5, N=1200)
    model = g.Model(6, 4, 100, 0.05, 20.0)
    px = g.Proxy(_wander(np.linspace(5.0, 80.0, 6), 5, seed=6), 1500, 0.5, 250)
    with formulation(1, table_factor_percent=400):
        check_proxy(tr, model, px, PAR[:2], 1.0, engine=_engine(6, 2))


def test_an_index_the_tables_cannot_hold_is_refused():
    tr = _tangled(6, N=300)
    px = g.Proxy(_wander(np.linspace(5.0, 80.0, 6), 3, seed=1), 1000, 0.3, 0)      # never forgets: every id of the trace
    with pytest.raises(g.GorgoError, match="table_factor_percent"):
        g.eval_proxy(load(tr), g.Model(6, 4, 30, 0.05, 20.0), px, PAR[:1], [1.0])


def test_replica_and_slot_limits_on_block_tables():
    tr = _tangled(7, N=1200, R=64, n_ids=500, max_blocks=8, gap_ms=3)
    rtt = np.linspace(5.0, 200.0, 64)
    model = g.Model(64, 16, 40, 0.05, 20.0)
    for policy in ("least-request", "session-affinity", "random"):
        check_policy(tr, model, rtt, policy, [1.0], np.array([3], np.uint64))
    check_engine(tr, model, _engine(64, 3), rtt, PAR[:1], 1.0)
    check_policy(tr, g.Model(1, 64, 12, 0.05, 20.0), [9.0], "least-request", [1.0])


def test_long_requests_many_compactions():
    # requests of up to 200 blocks over more ids than a table has slots: every lane-strided loop of the match, the update and the eviction
    # walk runs more than once per request, and tables fill up and are compacted again and again
    tr = _tangled(8, N=600, R=3, n_ids=5000, max_blocks=200, gap_ms=30)
    rtt = [10.0, 20.0, 30.0]
    model = g.Model(3, 2, 260, 0.05, 20.0)
    check_population(tr, model, rtt, PAR, [1.0, 0.5, 2.0])
    steps = g.online_steps(tr.N, 32, 8)
    check_online(tr, model, rtt, PAR[:2], np.random.default_rng(9).standard_normal((2, steps, 3)), 1.0, 32, 8, lo=LO,
                 hi=HI, sigma0=1.0)
    px = g.Proxy(_wander(np.asarray(rtt), 4, seed=2), 2000, 0.4, 520)
    with formulation(1, table_factor_percent=300):
        check_proxy(tr, model, px, PAR[:2], 1.0)


@pytest.mark.parametrize("config,n", [(1, 2000), (2, 4000)])
def test_block_tables_give_what_segment_rows_give(config, n):
    """Chain-consistent workloads, forced onto block tables: every variant against the oracle (the segment rows'
    tests compare the same calls with the same oracle results)."""
    wl = tg.config(config, n)
    tr, rtt = wl.trace, wl.rtt_ms
    model = g.Model(wl.R, wl.batch, wl.cache_blocks, wl.prefill_ms_per_token, wl.decode_ms_per_token)
    steps = g.online_steps(tr.N, 128, 32)
    z = np.random.default_rng(config).standard_normal((2, steps, 3))
    recipe = tg.engine_recipe(wl, 1)
    eng = g.Engine(recipe["prefill_ms_per_token"], recipe["decode_ms_per_token"], recipe["kv_tokens"], recipe["slowdown"])
    blocks = 2 * wl.cache_blocks if wl.cache_blocks else 0
    px = g.Proxy(tg.rtt_walk(wl, 6, 1), max(1, int(tr.ts_ms[-1]) // 6), 0.3, blocks)
    with formulation(1, table_factor_percent=400):
        assert load(tr).replay_path()["path"] == 1
        check_online(tr, model, rtt, PAR[:2], z, [1.0, 2.0], 128, 32, lo=LO, hi=HI, sigma0=0.5)
        for policy in ("least-request", "session-affinity", "random"):
            check_policy(tr, model, rtt, policy, [1.0], np.array([11], np.uint64))
        check_engine(tr, model, eng, rtt, PAR[:2], [1.0, 0.5])
        check_proxy(tr, model, px, PAR[:2], [1.0, 0.5])
        check_proxy(tr, model, px, PAR[:1], 1.0, engine=eng)


def test_empty_trace_and_single_request_on_block_tables():
    one = tg.random_small(1, 1, 2, consistent=False)
    none = one.head(0)
    model = g.Model(2, 2, 0, 0.05, 20.0)
    with formulation(1):
        for tr in (none, one):
            check_policy(tr, model, [10.0, 20.0], "least-request", [1.0])
            check_online(tr, model, [10.0, 20.0], PAR[:1], np.zeros((1, g.online_steps(tr.N, 4, 2), 3)), 1.0, 4, 2,
                         lo=LO, hi=HI, sigma0=0.5)

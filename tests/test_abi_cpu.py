"""CPU-only tests of the C-ABI library: it loads, exports every declared symbol, and its host-side logic
(trace loading, validation, tuner arithmetic, random draws) behaves as declared.  No compute call here."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

import paper_2602_11688_amd as g
from paper_2602_11688_amd import binding as gb
from oracle import es_oracle as eo
from synth import tracegen as tg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "gorgo.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(gorgo_[a-z0-9_]+)\s*\(", hdr))
    assert {"gorgo_load_trace", "gorgo_eval_population", "gorgo_es_step"} <= names and len(names) >= 15
    L = g.lib()
    for n in sorted(names):
        assert hasattr(L, n), f"{n} declared in gorgo.h but not exported"


def _trace(tr):
    return g.Trace.from_arrays(tr.ts_ms, tr.in_len, tr.out_len, tr.blk_off, tr.hash_ids)


def test_trace_info_and_chain_consistency():
    w = tg.config(1)
    t = _trace(w.trace)
    i = t.info()
    assert i["N"] == 2000 and i["total_blocks"] == w.trace.blk_off[-1] and i["unique_ids"] == w.notes["unique_ids"]
    assert i["max_blocks"] == w.notes["max_blocks"] and i["chain_consistent"]
    bad = tg.random_small(3, 50, 2, consistent=False)
    assert not _trace(bad).info()["chain_consistent"]
    assert _trace(tg.random_small(3, 50, 2, consistent=True)).info()["chain_consistent"]
    for seed in range(4):                                 # branching forests: consistent by construction
        f = tg.random_forest(seed, 300, max_blocks=5 + 10 * seed)
        i = _trace(f).info()
        assert i["chain_consistent"] and i["max_blocks"] <= 5 + 10 * seed and np.diff(f.blk_off).min() >= 1


def test_jsonl_loader_matches_arrays(tmp_path):
    w = tg.config(1, 300)
    p = tmp_path / "t.jsonl"
    w.trace.write_jsonl(str(p))
    with open(p, "a") as f:          # unknown members and blank lines are ignored
        f.write('\n{"extra": {"a": [1, "x"]}, "timestamp": 999999, "hash_ids": [], "input_length": 0, '
                '"output_length": 1, "note": "end"}\n')
    t = g.Trace.from_jsonl(str(p))
    i = t.info()
    assert i["N"] == 301 and i["total_blocks"] == w.trace.blk_off[-1]
    assert i == dict(_trace(w.trace).info(), N=301)


@pytest.mark.parametrize("text,code", [
    ('{"timestamp": 1, "input_length": 2, "output_length": 1}\n', -3),                       # hash_ids missing
    ('{"timestamp": 1, "input_length": 2, "output_length": 1, "hash_ids": [1, }\n', -3),
    ('{"timestamp": "x", "input_length": 2, "output_length": 1, "hash_ids": []}\n', -3),
    ('not json\n', -3),
    ('{"timestamp": 5, "input_length": 2, "output_length": 1, "hash_ids": [1]}\n'
     '{"timestamp": 4, "input_length": 2, "output_length": 1, "hash_ids": [1]}\n', -4),       # unsorted
])
def test_jsonl_loader_errors(tmp_path, text, code):
    p = tmp_path / "bad.jsonl"
    p.write_text(text)
    with pytest.raises(g.GorgoError) as e:
        g.Trace.from_jsonl(str(p))
    assert e.value.code == code and len(str(e.value)) > 15


def test_loader_io_and_argument_errors(tmp_path):
    with pytest.raises(g.GorgoError) as e:
        g.Trace.from_jsonl(str(tmp_path / "missing.jsonl"))
    assert e.value.code == -2
    with pytest.raises(g.GorgoError) as e:
        g.Trace.from_arrays([0, 1], [1, 1], [1, 1], [0, 1, 0], [1])          # blk_off decreases
    assert e.value.code == -1
    with pytest.raises(g.GorgoError) as e:
        g.Trace.from_arrays([0], [-1], [1], [0, 1], [1])
    assert e.value.code == -1
    t = g.Trace.from_arrays([], [], [], [0], [])
    assert t.info()["N"] == 0


def test_model_validation_without_gpu():
    t = _trace(tg.config(1, 100).trace)
    ok = g.Model(4, 8, 0, 0.05, 20.0)
    assert g.workspace_bytes(t, ok, 16) > 0
    for bad, code in [(g.Model(0, 8, 0, 0.05, 20.0), -1), (g.Model(65, 8, 0, 0.05, 20.0), -1),
                      (g.Model(64, 64, 0, 0.05, 20.0), -1), (g.Model(4, 8, 0, float("nan"), 20.0), -6),
                      (g.Model(4, 8, 3, 0.05, 20.0), -5), (g.Model(4, 8, 0, 0.05, 20.0, block_tokens=256), -1)]:
        with pytest.raises(g.GorgoError) as e:
            g.workspace_bytes(t, bad, 16)
        assert e.value.code == code
    with pytest.raises(g.GorgoError):
        g.workspace_bytes(t, ok, 0)
    # tokens of a cached prefix (block_tokens * blocks, blocks < 2^16) are counted in 32 bits: block sizes beyond
    # 32767 tokens are refused, the largest allowed one is accepted
    tr = tg.config(1, 100).trace
    big = g.Trace.from_arrays(tr.ts_ms, tr.in_len, tr.out_len, tr.blk_off, tr.hash_ids, block_tokens=32767)
    assert g.workspace_bytes(big, g.Model(4, 8, 0, 0.05, 20.0, block_tokens=32767), 16) > 0
    too_big = g.Trace.from_arrays(tr.ts_ms, tr.in_len, tr.out_len, tr.blk_off, tr.hash_ids, block_tokens=32768)
    with pytest.raises(g.GorgoError) as e:
        g.workspace_bytes(too_big, g.Model(4, 8, 0, 0.05, 20.0, block_tokens=32768), 16)
    assert e.value.code == -1 and "32767" in str(e.value)


def test_eval_rejects_bad_arguments_before_touching_a_device():
    t = _trace(tg.config(1, 50).trace)
    m = g.Model(4, 8, 0, 0.05, 20.0).c()
    L = g.lib()
    rtt = np.array([10.0, 40.0, 120.0, 300.0])
    par = np.ones((2, 3))
    sc = np.ones(2)
    o = gb._Outputs()

    def call(rtt=rtt, par=par, sc=sc, ws=C.c_void_p(256), nbytes=1 << 40):
        return L.gorgo_eval_population(t._h, C.byref(m), None, gb._ptr(rtt), gb._ptr(par), gb._ptr(sc), 2, C.byref(o), ws,
                                       nbytes, None)
    assert call(rtt=np.array([10.0, np.inf, 1, 1])) == -6
    assert call(par=np.array([[1, 1, np.nan], [1, 1, 1]])) == -6
    assert call(par=np.array([[1, 1, 1e200], [1, 1, 1]])) == -6
    assert call(sc=np.array([1.0, -1.0])) == -6
    assert call(ws=None) == -7
    assert call(ws=C.c_void_p(264)) == -7
    assert call(nbytes=1024) == -7
    assert b"workspace" in L.gorgo_last_error()


def test_options_are_per_call_and_validated():
    """The library keeps no settings: options travel with each call (NULL = defaults) and are checked there."""
    L = g.lib()
    for name in ("gorgo_set_replay_path", "gorgo_set_replay_packing", "gorgo_set_handover_poll_limit",
                 "gorgo_set_table_factor_percent"):
        assert not hasattr(L, name)
    d = g.Options()
    L.gorgo_options_default(C.byref(d))
    assert (d.replay_path, d.replay_packing, d.handover_poll_limit, d.table_factor_percent) == (0, 2, 1 << 24, 200)
    wl = tg.config(1)
    t = g.Trace.from_arrays(wl.trace.ts_ms, wl.trace.in_len, wl.trace.out_len, wl.trace.blk_off, wl.trace.hash_ids)
    m = g.Model(wl.R, wl.batch, wl.cache_blocks, wl.prefill_ms_per_token, wl.decode_ms_per_token).c()
    path, n = C.c_int32(), C.c_size_t()

    def query(**kw):
        o = g.Options(0, 2, 1 << 24, 200)
        for k, v in kw.items():
            setattr(o, k, v)
        return L.gorgo_query_replay_path(t._h, C.byref(o), C.byref(path), None, None)
    assert query() == 0 and path.value == 2
    assert query(replay_path=1) == 0 and path.value == 1
    for bad in (dict(replay_path=3), dict(replay_path=-1), dict(replay_packing=3), dict(replay_packing=-1),
                dict(handover_poll_limit=-1), dict(table_factor_percent=109), dict(table_factor_percent=1601)):
        assert query(**bad) == -1 and b"options." in L.gorgo_last_error()
        o = g.Options(0, 2, 1 << 24, 200)
        for k, v in bad.items():
            setattr(o, k, v)
        assert L.gorgo_workspace_bytes(t._h, C.byref(m), C.byref(o), 4, None, C.byref(n)) == -1
    # two calls with different options do not influence each other: the workspace follows the call's own options
    sizes = {}
    for rp in (1, 2, 1):
        o = g.Options(rp, 2, 1 << 24, 200)
        assert L.gorgo_workspace_bytes(t._h, C.byref(m), C.byref(o), 4, None, C.byref(n)) == 0
        sizes.setdefault(rp, set()).add(n.value)
    assert len(sizes[1]) == 1 and sizes[1] != sizes[2]
    assert L.gorgo_workspace_bytes(t._h, C.byref(m), None, 4, None, C.byref(n)) == 0 and {n.value} == sizes[2]
    # the binding's own defaults object is what its set_* helpers change
    g.set_replay_path(1)
    try:
        assert g.default_options().replay_path == 1 and t.replay_path()["path"] == 1
        with pytest.raises(g.GorgoError):
            g.set_replay_path(3)
    finally:
        g.set_replay_path(0)
    assert t.replay_path()["path"] == 2


def test_online_and_policy_entry_points_reject_bad_arguments_before_touching_a_device():
    t = _trace(tg.config(1, 300).trace)
    m = g.Model(4, 8, 0, 0.05, 20.0).c()
    L = g.lib()
    rtt = np.array([10.0, 40.0, 120.0, 300.0])
    th = np.tile([0.5, 1.0, 0.1], (2, 1))
    sc = np.ones(2)
    o = gb._Outputs()
    assert L.gorgo_online_steps(672, 128, 32) == 18 and L.gorgo_online_steps(127, 128, 32) == 0
    assert L.gorgo_online_steps(10, 0, 1) < 0 and L.gorgo_online_steps(10, 4, 0) < 0

    def online(window=128, hop=32, lo=(0.05, 1.0, 0.05), hi=(2.0, 1.0, 0.5), sigma0=0.5, z=C.c_void_p(256), th=th):
        on = gb._Online(window, hop, (C.c_double * 3)(*lo), (C.c_double * 3)(*hi), sigma0, z, None, None, None, None, None)
        return L.gorgo_eval_online(t._h, C.byref(m), None, gb._ptr(rtt), gb._ptr(th), gb._ptr(sc), 2, C.byref(on), C.byref(o),
                                   None, 1 << 40, None)
    assert online(window=0) == -1 and online(window=2048) == -1 and online(hop=0) == -1
    assert online(z=None) == -1
    assert online(lo=(0.0, 1.0, 0.05)) == -6 and online(lo=(3.0, 1.0, 0.05)) == -6
    assert online(sigma0=float("nan")) == -6
    assert online(th=np.tile([5.0, 1.0, 0.1], (2, 1))) == -1          # theta0 outside [lo, hi]
    assert online() == -7                                             # everything valid up to the workspace
    assert L.gorgo_eval_online(t._h, C.byref(m), None, gb._ptr(rtt), gb._ptr(th), gb._ptr(sc), 2, None, C.byref(o), None, 0,
                               None) == -1

    def policy(pol, seeds=None):
        return L.gorgo_eval_policy(t._h, C.byref(m), None, gb._ptr(rtt), pol, seeds, gb._ptr(sc), 2, C.byref(o), None,
                                   1 << 40, None)
    assert policy(0) == -1 and policy(4) == -1 and policy(3) == -1    # random without seeds
    assert policy(1) == -7 and policy(3, gb._ptr(np.array([1, 2], np.uint64))) == -7
    bad = _trace(tg.random_small(3, 50, 2, consistent=False))
    mb = g.Model(2, 2, 0, 0.05, 20.0).c()
    assert L.gorgo_eval_policy(bad._h, C.byref(mb), None, gb._ptr(rtt[:2]), 1, None, gb._ptr(sc), 2, C.byref(o), None, 1 << 40,
                               None) == -7                            # any trace will do: valid up to the workspace


def test_engine_entry_point_rejects_bad_arguments_before_touching_a_device():
    t = _trace(tg.config(1, 300).trace)
    m = g.Model(4, 8, 0, 0.05, 20.0).c()
    L = g.lib()
    rtt = np.array([10.0, 40.0, 120.0, 300.0])
    par = np.ones((2, 3))
    sc = np.ones(2)
    o = gb._Outputs()
    ok_pf, ok_dec = np.full(4, 0.05), np.full(4, 20.0)

    def engine(pf=ok_pf, dec=ok_dec, kv=None, slow=0.1, policy=0, par=par, seeds=None, online=None, null=False, tr=t, mm=m):
        e = gb._Engine(gb._ptr(pf), gb._ptr(dec), gb._ptr(kv), slow)
        return L.gorgo_eval_engine(tr._h, C.byref(mm), None, None if null else C.byref(e), gb._ptr(rtt), policy, gb._ptr(par),
                                   seeds, online, gb._ptr(sc), 2, C.byref(o), None, 1 << 40, None)
    assert engine(null=True) == -1 and engine(pf=None) == -1 and engine(dec=None) == -1
    assert engine(pf=np.array([0.05, np.nan, 0.05, 0.05])) == -6 and engine(dec=np.array([20.0, -1.0, 20.0, 20.0])) == -6
    assert engine(slow=-0.5) == -6 and engine(slow=float("inf")) == -6
    assert engine(kv=np.array([0, -1, 0, 0], np.int64)) == -1 and engine(kv=np.array([0, 1 << 60, 0, 0], np.int64)) == -1
    assert engine(policy=-1) == -1 and engine(policy=4) == -1 and engine(policy=3) == -1       # random without seeds
    assert engine(par=None) == -1                                                                # the cost model needs weights
    on = gb._Online(128, 32, (C.c_double * 3)(0.05, 0.05, 0.05), (C.c_double * 3)(2.0, 2.0, 2.0), 0.5, C.c_void_p(256),
                    None, None, None, None, None)
    assert engine(policy=1, online=C.byref(on)) == -1                                            # the tuner tunes the cost model
    # everything valid up to the workspace
    assert engine() == -7 and engine(kv=np.array([0, 5000, 1, 1 << 52], np.int64)) == -7
    assert engine(policy=1, par=None) == -7 and engine(policy=3, par=None, seeds=gb._ptr(np.array([1, 2], np.uint64))) == -7
    assert engine(online=C.byref(on)) == -7
    bad = _trace(tg.random_small(3, 50, 2, consistent=False))
    mb = g.Model(2, 2, 0, 0.05, 20.0).c()
    assert engine(tr=bad, mm=mb) == -7                                                           # any trace will do


def test_proxy_entry_point_rejects_bad_arguments_before_touching_a_device():
    t = _trace(tg.config(1, 300).trace)
    m = g.Model(4, 8, 0, 0.05, 20.0).c()
    L = g.lib()
    par = np.ones((2, 3))
    sc = np.ones(2)
    o = gb._Outputs()
    ok = np.tile([10.0, 40.0, 120.0, 300.0], (3, 1))

    def proxy(rt=ok, epochs=3, probe=30000, alpha=0.5, index=0, tables=C.c_void_p(256), null=False, par=par, tr=t, mm=m):
        x = gb._Proxy(epochs, probe, gb._ptr(rt), alpha, index, tables, None)
        return L.gorgo_eval_proxy(tr._h, C.byref(mm), None, None if null else C.byref(x), None, gb._ptr(par), None, gb._ptr(sc), 2,
                                  C.byref(o), None, 1 << 40, None)
    assert proxy(null=True) == -1 and proxy(rt=None) == -1 and proxy(tables=None) == -1
    assert proxy(epochs=0) == -1 and proxy(epochs=1 << 20) == -1 and proxy(probe=0) == -1 and proxy(index=-2) == -1
    assert proxy(index=500) == -1                                     # the replicas' caches are unbounded here
    assert proxy(alpha=0.0) == -6 and proxy(alpha=1.5) == -6 and proxy(alpha=float("nan")) == -6
    bad_rt = ok.copy()
    bad_rt[2, 1] = -1.0
    assert proxy(rt=bad_rt) == -6
    assert b"rtt_true_ms[2][1]" in L.gorgo_last_error()
    assert proxy(par=None) == -1
    assert proxy() == -7 and proxy(epochs=1, alpha=1.0, index=-1) == -7           # everything valid up to the workspace
    mc = g.Model(4, 8, 200, 0.05, 20.0).c()
    assert proxy(index=199, mm=mc) == -1 and proxy(index=200, mm=mc) == -7 and proxy(index=1000, mm=mc) == -7
    bad = _trace(tg.random_small(3, 50, 2, consistent=False))
    mb = g.Model(2, 2, 0, 0.05, 20.0).c()
    assert proxy(rt=ok[:, :2].copy(), tr=bad, mm=mb) == -7                        # any trace will do
    # on block tables the index lives in the replicas' tables: a bounded cache's tables must be large enough for it
    tangled = _trace(tg.random_small(6, 300, 6, consistent=False, n_ids=300, max_blocks=24))
    assert not tangled.info()["chain_consistent"]
    mt = g.Model(6, 4, 30, 0.05, 20.0).c()
    rt6 = np.tile(np.linspace(5.0, 80.0, 6), (3, 1))
    assert proxy(rt=rt6, tr=tangled, mm=mt, index=-1) == -7 and proxy(rt=rt6, tr=tangled, mm=mt, index=30) == -7
    assert proxy(rt=rt6, tr=tangled, mm=mt, index=0) == -5                        # it never forgets: every id of the trace
    assert b"table_factor_percent" in L.gorgo_last_error()
    big = gb.Options()
    L.gorgo_options_default(C.byref(big))
    big.table_factor_percent = 1200
    x = gb._Proxy(3, 30000, gb._ptr(rt6), 0.5, 0, C.c_void_p(256), None)
    assert L.gorgo_eval_proxy(tangled._h, C.byref(mt), C.byref(big), C.byref(x), None, gb._ptr(par), None, gb._ptr(sc), 2,
                              C.byref(o), None, 1 << 40, None) == -7


# ------------------------------------------------------------------------------------------------ tuner

def test_philox_known_answers():
    """Known-answer vectors of Philox-4x32-10 as published with the generator (Random123 test vectors)."""
    assert [hex(x) for x in g.philox4x32_10([0, 0, 0, 0], [0, 0])] == ['0x6627e8d5', '0xe169c58d', '0xbc57ac4c', '0x9b00dbd8']
    assert [hex(x) for x in g.philox4x32_10([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0])] == \
        ['0xd16cfe09', '0x94fdcceb', '0x5001e420', '0x24126ea1']


def test_normal_draws_are_reproducible_and_standard():
    z = g.es_sample(7, 3, 40000)
    assert (z == g.es_sample(7, 3, 40000)).all()
    assert (z[:100] == g.es_sample(7, 3, 100)).all()                 # counter-based: prefix-stable
    assert (z != g.es_sample(7, 4, 40000)).any() and (z != g.es_sample(8, 3, 40000)).any()
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    assert abs((np.abs(z) < 1.959964).mean() - 0.95) < 0.004
    assert abs(np.corrcoef(z[:, 0], z[:, 1])[0, 1]) < 0.02


def test_propose_matches_oracle_mutation_rule():
    s = g.es_init(11)
    assert list(s.theta) == [0.5, 1.0, 0.1] and s.sigma == 0.5 and list(s.lo) == [0.05, 1.0, 0.05] and list(s.hi) == [2.0, 1.0, 0.5]
    z = g.es_sample(11, 0, 64)
    z[5] = [50, 0, 50]
    z[6] = [-50, 0, -50]
    p = g.es_propose(s, z)
    ref = eo.offspring(list(s.theta), s.sigma, list(s.lo), list(s.hi), z)
    np.testing.assert_allclose(p, ref, rtol=1e-15)
    assert p[0].tolist() == [0.5, 1.0, 0.1] and p[5].tolist() == [2.0, 1.0, 0.5] and p[6].tolist() == [0.05, 1.0, 0.05]


@pytest.mark.parametrize("P", [1, 2, 5, 8, 64, 1024])
def test_update_matches_oracle(P):
    rng = np.random.default_rng(P)
    s = g.es_init(3)
    for gen in range(4):
        z = g.es_sample(3, s.generation, P)
        par = g.es_propose(s, z)
        fit = rng.uniform(100, 200, P).round(0)                      # rounded: ties do occur
        th, sg, bf, bt = eo.update(list(s.theta), s.sigma, list(s.lo), list(s.hi), par, fit, s.best_fitness,
                                   np.array(list(s.best_theta)))
        g.es_update(s, par, fit)
        np.testing.assert_allclose(list(s.theta), th, rtol=1e-14)
        assert abs(s.sigma - sg) <= 1e-15 * sg and s.best_fitness == bf and list(s.best_theta) == list(bt)
        assert s.generation == gen + 1


def test_update_one_plus_one_accepts_only_strict_improvement():
    s = g.es_init(0)
    par = np.array([[0.5, 1.0, 0.1], [0.9, 1.0, 0.3]])
    g.es_update(s, par, [10.0, 10.0])
    assert list(s.theta) == [0.5, 1.0, 0.1] and s.sigma == 0.5 * math.exp(-0.1)
    g.es_update(s, par, [10.0, 9.0])
    assert list(s.theta) == [0.9, 1.0, 0.3] and s.best_fitness == 9.0


def test_es_rejects_bad_state():
    s = g.es_init(0)
    s.theta[0] = -1.0
    with pytest.raises(g.GorgoError):
        g.es_propose(s, np.zeros((2, 3)))
    s = g.es_init(0)
    with pytest.raises(g.GorgoError):
        g.es_update(s, np.ones((2, 3)), [float("nan"), 1.0])


def test_segments_share_row_slots_between_their_first_and_last_reference():
    """The loader's row slots: as many as the most segments in use at one time -- checked against a count made here
    from the block lists alone (a segment = a maximal run of blocks that the same set of requests touches; it is in
    use from the first to the last request that touches it)."""
    for cfg, n in ((1, None), (2, 4000), (5, 20000)):
        wl = tg.config(cfg, n)
        tr = wl.trace
        t = _trace(tr)
        info = t.replay_path()
        assert t.info()["chain_consistent"]
        # first and last request of every block id; blocks with the same (first, last, predecessor chain) form segments,
        # and what matters here is only how many distinct segments are alive at once: count blocks' [first, last]
        # intervals per segment through the segment's last block (ids are unique per position in a consistent trace)
        first, last = {}, {}
        for r in range(tr.N):
            for b in tr.hash_ids[tr.blk_off[r]:tr.blk_off[r + 1]].tolist():
                first.setdefault(b, r)
                last[b] = r
        # a request's path is cut wherever the set of touching requests changes: count, per request, the distinct
        # (first, last) pairs among its blocks = its segments; a segment is identified by its last block
        seg_first, seg_last = {}, {}
        refs = 0
        for r in range(tr.N):
            ids = tr.hash_ids[tr.blk_off[r]:tr.blk_off[r + 1]].tolist()
            for k, b in enumerate(ids):
                nxt = ids[k + 1] if k + 1 < len(ids) else None
                if nxt is None or (first[nxt], last[nxt]) != (first[b], last[b]):
                    refs += 1
                    seg_first.setdefault(b, r)
                    seg_last[b] = r
        events = np.zeros(tr.N + 1, np.int64)
        for b in seg_first:
            events[seg_first[b]] += 1
            events[seg_last[b] + 1] -= 1
        alive_most = int(np.cumsum(events).max())
        # (the loader's segments are at least as fine as the ones counted here, never coarser: a cut also falls where
        # the touching sets agree but a request ends; so its counts can only be larger, and equal on these traces)
        assert info["segment_refs"] >= refs and info["n_segments"] >= len(seg_first)
        slots = t.row_slots()
        assert alive_most <= slots <= info["n_segments"]
        if info["n_segments"] == len(seg_first):
            assert slots == alive_most
        if cfg == 5:
            assert slots < info["n_segments"] // 3         # (most conversations of the workload are over at any time)
    bad = _trace(tg.random_small(3, 200, 4, n_ids=40, max_blocks=8, consistent=False, gap_ms=5))
    assert not bad.info()["chain_consistent"] and bad.row_slots() == 0

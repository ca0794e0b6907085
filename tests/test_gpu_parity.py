"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest

import paper_2602_11688_amd as g
from oracle import binding as ob
from oracle import es_oracle as eo
from synth import tracegen as tg
from tests.gpu_helpers import RTOL, assert_replay_equal, check_population, gpu_eval, load, oracle_eval
from tests.helpers import load_golden

pytestmark = pytest.mark.gpu


def _model(wl, **over):
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token)
    kw.update(over)
    return g.Model(**kw)


@pytest.mark.parametrize("name", ["hand_trace_A.json", "hand_trace_B.json", "hand_trace_C.json", "hand_trace_D.json"])
def test_hand_traces(name):
    gold, tr = load_golden(name)
    m = gold["model"]
    model = g.Model(m["R"], m["batch"], m["cache_blocks"], m["prefill_ms_per_token"], m["decode_ms_per_token"])
    got = gpu_eval(tr, model, gold["rtt_ms"], [gold["w"]], gold["scale"])
    e = gold["expected"]
    assert got["route"][0].tolist() == e["route"]
    assert got["hit"][0].tolist() == e["hit_blocks"]
    assert got["ttft"][0].tolist() == e["ttft_ms"]
    assert got["e2e"][0].tolist() == e["e2e_ms"]
    if "p95_ttft_ms" in e:
        assert got["p95_ttft"][0] == e["p95_ttft_ms"] and got["p95_e2e"][0] == e["p95_e2e_ms"]


def test_config1_all_replays_unbounded_cache():
    wl = tg.config(1)
    got = check_population(wl.trace, _model(wl), wl.rtt_ms, wl.params, wl.scale, label="config1")
    assert len(set(got["route"].ravel().tolist())) == wl.R


def test_config2_lru_prefix():
    # 7,000 requests fill the eight 4,000-block caches several times over
    wl = tg.config(2, 7000)
    got = check_population(wl.trace, _model(wl), wl.rtt_ms, wl.params[:6], wl.scale[:6], label="config2")
    assert got["hit"].max() > 64          # matches span more than one 64-block tile


def test_small_cache_heavy_eviction_and_table_compaction():
    wl = tg.config(2, 2500)
    g.set_table_factor_percent(110)       # smallest tables: compaction happens often
    try:
        model = _model(wl, R=3, cache_blocks=300, batch=4)
        rng = np.random.default_rng(1)
        par = rng.uniform(0, 2, (6, 3))
        par[0] = [0.0, 1.0, 0.0]          # prefix-only: concentrates traffic, evicts the most
        par[1] = [1.0, 1.0, 0.0]
        check_population(wl.trace, model, [10.0, 12.0, 15.0], par, 1.0, label="small-cache")
    finally:
        g.set_table_factor_percent(200)


@pytest.mark.parametrize("seed,C,R,B", [(0, 0, 2, 1), (1, 6, 3, 2), (2, 9, 5, 3), (3, 40, 64, 16), (4, 12, 1, 64)])
def test_inconsistent_traces_with_repeated_ids(seed, C, R, B):
    tr = tg.random_small(seed, 700, R, n_ids=40, max_blocks=6, consistent=False, gap_ms=30)
    rng = np.random.default_rng(seed)
    model = g.Model(R, B, C, 0.05, 20.0)
    check_population(tr, model, rng.uniform(5, 80, R), rng.uniform(0, 2, (5, 3)), 1.0, label=f"random{seed}")


def test_weight_special_cases_and_negative_weights():
    wl = tg.config(1, 800)
    par = np.array([[0, 0, 0], [1, 0, 0], [0, 1, 0], [0, 0, 1], [-1.0, 1.0, 0.5], [1.0, -0.5, 0.25]], np.float64)
    got = check_population(wl.trace, _model(wl), wl.rtt_ms, par, 1.0, label="special")
    assert (got["route"][0] == 0).all() and (got["route"][1] == 0).all()


def test_time_scales_in_one_launch():
    wl = tg.config(4, 3000)
    idx = [0, 127, 128, 400, 640, 1023]
    check_population(wl.trace, _model(wl, cache_blocks=1500), wl.rtt_ms, wl.params[idx], wl.scale[idx], label="sweep")


def test_edge_cases():
    z = np.zeros(0, np.int64)
    # empty trace
    tr = tg.Trace(z, z.astype(np.int32), z.astype(np.int32), np.zeros(1, np.int64), z)
    got = gpu_eval(tr, g.Model(2, 2, 0, 0.05, 20.0), [1.0, 2.0], [[1, 1, 1]], 1.0)
    assert got["route"].shape == (1, 0) and got["p95_ttft"][0] == 0.0
    # requests without blocks, zero-length prompts, identical timestamps, one request
    tr = tg.Trace(np.array([5, 5, 5, 9]), np.array([0, 100, 700, 0], np.int32), np.array([1, 0, 3, 2], np.int32),
                  np.array([0, 0, 0, 2, 2]), np.array([4, 5]))
    check_population(tr, g.Model(2, 1, 0, 0.05, 20.0), [3.0, 3.0], [[1, 1, 1], [0.1, 1, 2]], [1.0, 0.0], label="edge")
    check_population(tr.head(1), g.Model(1, 1, 2, 0.05, 20.0), [3.0], [[1, 1, 1]], 2.5, label="single")


def test_max_blocks_request_and_ragged_tails():
    # one conversation that grows past several 64-lane tiles with ragged lengths, bounded cache
    rng = np.random.default_rng(9)
    lens = [1, 63, 64, 65, 127, 128, 129, 200, 255, 256, 300, 64, 1, 300]
    ids, off = [], [0]
    for n in lens:
        ids += list(range(1, n + 1))
        off.append(len(ids))
    N = len(lens)
    tr = tg.Trace(np.arange(N, dtype=np.int64) * 700, (np.array(lens) * 512 - 7).astype(np.int32),
                  rng.integers(1, 40, N).astype(np.int32), np.array(off, np.int64), np.array(ids, np.int64))
    check_population(tr, g.Model(2, 2, 310, 0.05, 20.0), [10.0, 11.0], [[1, 1, 0.0], [1, 1, 1], [0, 0, 1]], 1.0,
                     label="ragged")


@pytest.mark.parametrize("path", [1, 2])
def test_same_launch_twice_is_identical(path):
    wl = tg.config(2, 3000)
    h = load(wl.trace)
    a = gpu_eval(wl.trace, _model(wl, cache_blocks=1000), wl.rtt_ms, wl.params[:4], 1.0, handle=h, path=path)
    b = gpu_eval(wl.trace, _model(wl, cache_blocks=1000), wl.rtt_ms, wl.params[:4], 1.0, handle=h, path=path)
    for k in a:
        assert a[k].tobytes() == b[k].tobytes()


def test_formulations_agree_bit_for_bit():
    wl = tg.config(3, 4000)
    h = load(wl.trace)
    m = _model(wl, cache_blocks=900)
    a = gpu_eval(wl.trace, m, wl.rtt_ms, wl.params[:8], 1.0, handle=h, path=1)
    b = gpu_eval(wl.trace, m, wl.rtt_ms, wl.params[:8], 1.0, handle=h, path=2)
    for k in a:
        assert a[k].tobytes() == b[k].tobytes(), k


def test_segment_rows_rejected_for_inconsistent_trace():
    tr = tg.random_small(5, 50, 2, consistent=False)
    with pytest.raises(g.GorgoError) as e:
        gpu_eval(tr, g.Model(2, 2, 0, 0.05, 20.0), [1.0, 2.0], [[1, 1, 1]], 1.0, path=2)
    assert e.value.code == -1


def test_shared_prefix_forest():
    """Chain-consistent trace with branching: a common root run shared by every request (a system prompt),
    a few second-level branches, then per-conversation tails that grow turn by turn; bounded caches."""
    rng = np.random.default_rng(17)
    root = list(range(1, 8))
    branches = [list(range(100 + 10 * b, 100 + 10 * b + int(rng.integers(1, 9)))) for b in range(4)]
    convs, lists, nxt = [], [], 1000
    for _ in range(900):
        if not convs or rng.random() < 0.3:
            convs.append(root + branches[int(rng.integers(0, 4))])
        c = int(rng.integers(0, len(convs)))
        if rng.random() < 0.15:
            lists.append(list(convs[c][:int(rng.integers(1, len(convs[c]) + 1))]))   # a request that ends mid-way
            continue
        add = int(rng.integers(0, 5))
        convs[c] = convs[c] + list(range(nxt, nxt + add))
        nxt += add
        lists.append(list(convs[c]))
    nblk = np.array([len(x) for x in lists], np.int64)
    tr = tg.Trace(np.cumsum(rng.integers(0, 50, len(lists))).astype(np.int64), (nblk * 512).astype(np.int32),
                  rng.integers(1, 30, len(lists)).astype(np.int32), np.concatenate([[0], np.cumsum(nblk)]),
                  np.array([x for l in lists for x in l], np.int64))
    assert load(tr).info()["chain_consistent"]
    par = rng.uniform(0, 2, (6, 3))
    par[0] = [0.0, 1.0, 0.0]
    check_population(tr, g.Model(4, 2, 120, 0.05, 20.0), [10.0, 14.0, 30.0, 11.0], par, 1.0, label="forest")
    check_population(tr, g.Model(3, 2, 0, 0.05, 20.0), [10.0, 14.0, 30.0], par[:3], 1.0, label="forest-unbounded")


def test_many_segments_per_request():
    # one conversation growing by one block per turn: turn t is t single-block segments (> one 64-lane tile)
    lens = list(range(1, 150)) + [10, 149, 3]
    ids, off = [], [0]
    for n in lens:
        ids += list(range(1, n + 1))
        off.append(len(ids))
    N = len(lens)
    rng = np.random.default_rng(4)
    tr = tg.Trace(np.arange(N, dtype=np.int64) * 300, (np.array(lens) * 512).astype(np.int32),
                  rng.integers(1, 20, N).astype(np.int32), np.array(off, np.int64), np.array(ids, np.int64))
    check_population(tr, g.Model(2, 2, 160, 0.05, 20.0), [10.0, 11.0], [[1, 1, 0.0], [1, 1, 1], [0, 0, 1]], 1.0,
                     label="many-segments")


def test_requests_with_more_segments_than_a_staged_batch_holds():
    # the same growth continued past 512 segments per request: such a request is processed on its own, its
    # segment references read from global memory
    lens = list(range(1, 540, 3)) + list(range(520, 560)) + [7, 559, 2, 530]
    ids, off = [], [0]
    for n in lens:
        ids += list(range(1, n + 1))
        off.append(len(ids))
    N = len(lens)
    rng = np.random.default_rng(5)
    tr = tg.Trace(np.arange(N, dtype=np.int64) * 300, (np.array(lens) * 512).astype(np.int32),
                  rng.integers(1, 20, N).astype(np.int32), np.array(off, np.int64), np.array(ids, np.int64))
    assert load(tr).replay_path()["segment_refs"] > 40 * N
    check_population(tr, g.Model(3, 2, 600, 0.05, 20.0), [10.0, 11.0, 30.0], [[1, 1, 0.0], [1, 1, 1], [0, 0, 1], [0.5, 1, 0.1]],
                     [1.0, 1.0, 2.0, 0.5], label="beyond-stage", paths=[2])


def test_p95_only_outputs_and_percentile_selection():
    import torch
    wl = tg.config(1)
    h = load(wl.trace)
    res = g.eval_population(h, _model(wl), wl.rtt_ms, wl.params, wl.scale, per_request=False)
    full = g.eval_population(h, _model(wl), wl.rtt_ms, wl.params, wl.scale)
    torch.cuda.synchronize()
    assert res.route is None
    assert res.p95_ttft_ms.cpu().numpy().tobytes() == full.p95_ttft_ms.cpu().numpy().tobytes()
    t = full.ttft_ms.cpu().numpy()
    k = -(-95 * t.shape[1] // 100)
    assert (np.sort(t, axis=1)[:, k - 1] == full.p95_ttft_ms.cpu().numpy()).all()
    assert (np.array([ob.p95(row) for row in full.e2e_ms.cpu().numpy()]) == full.p95_e2e_ms.cpu().numpy()).all()


def test_es_generations_match_oracle():
    wl = tg.config(1, 1200)
    h = load(wl.trace)
    model = _model(wl)
    P = 12
    s = g.es_init(2024)
    theta, sigma, bf, bt = list(s.theta), s.sigma, float("inf"), None
    ws = None
    for gen in range(3):
        z = g.es_sample(2024, gen, P)
        par_ref = eo.offspring(theta, sigma, list(s.lo), list(s.hi), z)
        fit_ref = np.array([oracle_eval(wl.trace, model, wl.rtt_ms, par_ref[p], 1.0).p95_ttft_ms for p in range(P)])
        theta, sigma, bf, bt = eo.update(theta, sigma, list(s.lo), list(s.hi), par_ref, fit_ref, bf, bt)
        par, fit, ws = g.es_step(h, model, wl.rtt_ms, 1.0, P, s, workspace=ws)
        np.testing.assert_allclose(par, par_ref, rtol=1e-15)
        np.testing.assert_allclose(fit, fit_ref, rtol=1e-9)
        np.testing.assert_allclose(list(s.theta), theta, rtol=1e-12)
        assert abs(s.sigma - sigma) <= 1e-12 * sigma and s.generation == gen + 1
        assert abs(s.best_fitness - bf) <= 1e-9 * bf


def test_missing_library_is_an_error(monkeypatch):
    from paper_2602_11688_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libgorgo.so")
    with pytest.raises(RuntimeError):
        binding.lib()


def test_given_up_replays_end_and_poison_their_latencies():
    """Two replays per wavefront pair hand over through polled words, and the polls are bounded: with the limit at 0
    a wavefront whose partner is not ready at its first poll gives its replays up; every wavefront still ends, a
    given-up replay's latencies and p95 are all NaN (never a mixture), and the next evaluation with the default
    limit is exact again.  (Whether a given replay is given up depends on timing; one replay per workgroup meets at
    barriers and cannot be given up.)"""
    import torch
    wl = tg.config(1, 900)
    h = load(wl.trace)
    model = _model(wl)
    g.set_handover_poll_limit(0)
    g.set_replay_packing(1)
    try:
        res = g.eval_population(h, model, wl.rtt_ms, wl.params[:8], 1.0)
        torch.cuda.synchronize()
        p95 = res.p95_ttft_ms.cpu().numpy()
        ttft = res.ttft_ms.cpu().numpy()
        gave_up = np.isnan(p95)
        for p in range(8):
            assert np.isnan(ttft[p]).all() == gave_up[p] and np.isnan(ttft[p]).any() == gave_up[p]
        if gave_up.any():
            with pytest.raises(g.GorgoError):
                g.es_update(g.es_init(3), wl.params[:8], p95)
    finally:
        g.set_handover_poll_limit(1 << 24)
        g.set_replay_packing(2)
    got = gpu_eval(wl.trace, model, wl.rtt_ms, wl.params[:2], 1.0, handle=h, path=2)
    for p in range(2):
        assert_replay_equal(got, p, oracle_eval(wl.trace, model, wl.rtt_ms, wl.params[p], 1.0), "after give-up")


def test_two_replays_per_wavefront_pair_give_the_same_results():
    """Packed and unpacked launches of the segment-row kernel on the same inputs, bit for bit, at a shape where the
    automatic choice packs as well (more replays than fit on the GPU at once, the pairs do), with per-request outputs and
    without."""
    import torch
    wl = tg.config(3, 1500)
    model = g.Model(wl.R, wl.batch, 300, wl.prefill_ms_per_token, wl.decode_ms_per_token)
    h = load(wl.trace)
    rng = np.random.default_rng(12)
    P = 1800
    params = rng.uniform(0.05, 2.0, (P, 3))
    assert g.replay_packing(h, model, P) and not g.replay_packing(h, model, 1000) and not g.replay_packing(h, model, 6000)
    scale = rng.choice([0.5, 1.0, 2.0], P)
    out = {}
    for mode in (0, 1, 2):
        g.set_replay_packing(mode)
        try:
            res = g.eval_population(h, model, wl.rtt_ms, params, scale)
            lean = g.eval_population(h, model, wl.rtt_ms, params, scale, per_request=False)
            torch.cuda.synchronize()
        finally:
            g.set_replay_packing(2)
        assert torch.equal(res.p95_ttft_ms, lean.p95_ttft_ms) and torch.equal(res.p95_e2e_ms, lean.p95_e2e_ms)
        out[mode] = res
    for mode in (1, 2):
        for name in ("route", "hit_blocks", "ttft_ms", "e2e_ms", "p95_ttft_ms", "p95_e2e_ms"):
            assert torch.equal(getattr(out[0], name), getattr(out[mode], name)), (mode, name)
    # and the unpacked launch is the oracle's
    for p in (0, 1, 899, 1798, 1799):
        ref = oracle_eval(wl.trace, model, wl.rtt_ms, params[p], float(scale[p]))
        assert np.array_equal(out[0].route[p].cpu().numpy(), ref.route)
        np.testing.assert_allclose(out[0].ttft_ms[p].cpu().numpy(), ref.ttft_ms, rtol=RTOL, atol=0)


def _churn_trace(seed, conversations, turns_max, branch):
    """Conversations one after the other: each is a few turns that extend the previous turn's blocks, then it is over
    for good -- so the row slots of its segments are handed on to the next conversation at once, a request's path
    often sits in slots that the previous request's path has just given up, and long conversations have paths of more
    segments than the kernels preload.  With `branch`, later requests also end in the middle of what an earlier
    turn added, which cuts that turn's blocks into several segments that all start with the same request."""
    rng = np.random.default_rng(seed)
    ts, in_len, out_len, off, ids = [], [], [], [0], []
    t, next_id = 0, 1
    for c in range(conversations):
        path = []
        turns = int(rng.integers(1, turns_max + 1))
        history = []
        for k in range(turns):
            add = int(rng.integers(1, 5))
            path = path + list(range(next_id, next_id + add))
            next_id += add
            history.append(list(path))
            t += int(rng.integers(0, 30))
            ts.append(t)
            ids += path
            off.append(len(ids))
            in_len.append(len(path) * 512 - int(rng.integers(0, 512)))
            out_len.append(int(rng.integers(1, 200)))
            if branch and k >= 1 and rng.random() < 0.4:
                # a request that stops inside an earlier turn's addition, then goes its own way
                cut = history[int(rng.integers(0, len(history)))]
                stop = int(rng.integers(1, len(cut) + 1))
                own = list(range(next_id, next_id + int(rng.integers(0, 3))))
                next_id += len(own)
                t += int(rng.integers(0, 30))
                ts.append(t)
                ids += cut[:stop] + own
                off.append(len(ids))
                in_len.append((stop + len(own)) * 512)
                out_len.append(int(rng.integers(1, 200)))
    return tg.Trace(np.array(ts, np.int64), np.array(in_len, np.int32), np.array(out_len, np.int32),
                    np.array(off, np.int64), np.array(ids, np.int64))


@pytest.mark.parametrize("seed,R,B,turns_max,branch,cache", [(1, 32, 8, 4, False, 0), (2, 32, 8, 4, True, 40), (3, 8, 2, 14, True, 60),
                                                              (4, 64, 4, 12, True, 50), (5, 33, 3, 3, False, 12), (6, 5, 16, 20, True, 0),
                                                              (7, 16, 8, 2, True, 9)])
def test_row_slots_handed_on_between_segments(seed, R, B, turns_max, branch, cache):
    tr = _churn_trace(seed, 120, turns_max, branch)
    h = load(tr)
    assert h.info()["chain_consistent"]
    # the point of the trace: far fewer rows than segments, so every slot serves many segments in turn
    assert h.row_slots() * 4 < h.replay_path()["n_segments"]
    nmax = int(np.diff(tr.blk_off).max())
    rng = np.random.default_rng(seed)
    model = g.Model(R, B, max(cache, nmax) if cache else 0, 0.05, 20.0)
    rtt = np.round(rng.uniform(1.0, 200.0, R), 1)
    par = rng.uniform(0.0, 2.0, (6, 3))
    par[0] = [0.0, 1.0, 0.0]            # prefix-cache routing: follows the cached prefix wherever it is
    check_population(tr, model, rtt, par, [1.0, 0.3, 4.0, 1.0, 1.0, 2.0], label=f"churn {seed}")


@pytest.mark.parametrize("R,B,burst", [(8, 8, 700), (32, 8, 2200), (5, 3, 300)])
def test_deep_in_flight_lists_in_bursts(R, B, burst):
    """Bursts of arrivals a millisecond apart with a minute of silence between them: during a burst every service
    slot's list of in-flight requests goes many deep and loses its oldest request one at a time (the record that
    moves up comes from memory); the first request after the silence finds every list completed at once."""
    rng = np.random.default_rng(R * 100 + B)
    N = 3 * burst + 50
    gaps = rng.integers(0, 3, size=N).astype(np.int64)
    gaps[burst::burst] = 60000
    sessions = 4 * R
    nblk = rng.integers(1, 6, size=N)
    who = rng.integers(0, sessions, size=N)
    lists = [[1 + int(who[r]) * 8 + k for k in range(int(nblk[r]))] for r in range(N)]
    blk_off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64)
    ids = np.array([x for l in lists for x in l], np.int64)
    tr = tg.Trace(np.cumsum(gaps), (nblk * 512).astype(np.int32), rng.integers(1, 6, size=N).astype(np.int32), blk_off, ids)
    rtt = np.linspace(5.0, 60.0, R)
    params = [[0.5, 1.0, 0.1], [0.0, 0.0, 1.0], [1.0, 0.1, 0.01]]
    check_population(tr, g.Model(R, B, 0, 0.05, 40.0), rtt, params, [1.0, 1.0, 0.5])

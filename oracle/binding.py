"""ctypes wrapper around the oracle library (TEST INFRASTRUCTURE ONLY)."""
import ctypes as C
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.gorgo_oracle_p95.restype = C.c_double
        L.gorgo_oracle_p95.argtypes = [C.c_void_p, C.c_int64]
        L.gorgo_oracle_replay.restype = C.c_int
        L.gorgo_oracle_replay.argtypes = [C.c_int64] + [C.c_void_p] * 5 + [C.c_int32, C.c_int32, C.c_int32,
                                                                          C.c_int64, C.c_double, C.c_double,
                                                                          C.c_void_p, C.c_void_p, C.c_double] + \
                                          [C.c_void_p] * 8
        L.gorgo_oracle_replay_ex.restype = C.c_int
        L.gorgo_oracle_replay_ex.argtypes = [C.c_int64] + [C.c_void_p] * 5 + \
            [C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_double, C.c_double, C.c_void_p, C.c_void_p, C.c_double,
             C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_int32,
             C.c_uint64] + [C.c_void_p] * 11
        L.gorgo_oracle_replay_engine.restype = C.c_int
        L.gorgo_oracle_replay_engine.argtypes = [C.c_int64] + [C.c_void_p] * 5 + \
            [C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_double, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double,
             C.c_void_p, C.c_void_p, C.c_double,
             C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_int32,
             C.c_uint64] + [C.c_void_p] * 8
        L.gorgo_oracle_replay_proxy.restype = C.c_int
        L.gorgo_oracle_replay_proxy.argtypes = [C.c_int64] + [C.c_void_p] * 5 + \
            [C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_double, C.c_double, C.c_void_p, C.c_void_p, C.c_void_p,
             C.c_double, C.c_int32, C.c_int32, C.c_void_p, C.c_double, C.c_int64, C.c_void_p, C.c_double,
             C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double] + [C.c_void_p] * 11
        L.gorgo_oracle_philox4x32_10.restype = None
        L.gorgo_oracle_philox4x32_10.argtypes = [C.c_void_p] * 3
        L.gorgo_oracle_splitmix64_next.restype = C.c_uint64
        L.gorgo_oracle_splitmix64_next.argtypes = [C.c_uint64]
        L.gorgo_oracle_tuner_exp.restype = C.c_double
        L.gorgo_oracle_tuner_exp.argtypes = [C.c_double]
        L.gorgo_oracle_online_steps.restype = C.c_int64
        L.gorgo_oracle_online_steps.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class Replay:
    route: np.ndarray        # uint8 [N]
    hit_blocks: np.ndarray   # uint16 [N]
    ttft_ms: np.ndarray      # float64 [N]
    e2e_ms: np.ndarray       # float64 [N]
    p95_ttft_ms: float
    p95_e2e_ms: float
    score: Optional[np.ndarray] = None   # float64 [N,R]
    q: Optional[np.ndarray] = None       # int64 [N,R]
    size: Optional[np.ndarray] = None    # int64 [N]
    # online tuner (replay_online only)
    theta_step: Optional[np.ndarray] = None     # float64 [steps,3] weights in use after each step
    fitness_step: Optional[np.ndarray] = None   # float64 [steps] window p95 TTFT seen at each step
    theta_final: Optional[np.ndarray] = None    # float64 [3] parent weights after the last step
    sigma_final: float = 0.0
    steps: int = 0
    accepted: int = 0
    # imperfect proxy knowledge (replay_proxy only)
    rtt_est: Optional[np.ndarray] = None        # float64 [epochs,R] the proxy's smoothed round trip times
    believed_hit: Optional[np.ndarray] = None   # uint16 [N] blocks the proxy's index matched on the chosen replica


def p95(x) -> float:
    x = np.ascontiguousarray(x, dtype=np.float64)
    return float(lib().gorgo_oracle_p95(_p(x), x.shape[0]))


def replay(trace, *, R, batch, cache_blocks, prefill_ms_per_token, decode_ms_per_token, rtt_ms, w, scale=1.0,
           block_tokens=512, debug=False) -> Replay:
    """One sequential replay of `trace` (any object with ts_ms, in_len, out_len, blk_off, hash_ids)."""
    N = int(trace.ts_ms.shape[0])
    ts = np.ascontiguousarray(trace.ts_ms, dtype=np.int64)
    il = np.ascontiguousarray(trace.in_len, dtype=np.int32)
    ol = np.ascontiguousarray(trace.out_len, dtype=np.int32)
    bo = np.ascontiguousarray(trace.blk_off, dtype=np.int64)
    hi = np.ascontiguousarray(trace.hash_ids, dtype=np.int64)
    rtt = np.ascontiguousarray(rtt_ms, dtype=np.float64)
    wv = np.ascontiguousarray(w, dtype=np.float64)
    assert rtt.shape == (R,) and wv.shape == (3,) and bo.shape == (N + 1,)
    route = np.zeros(N, np.uint8)
    hit = np.zeros(N, np.uint16)
    ttft = np.zeros(N, np.float64)
    e2e = np.zeros(N, np.float64)
    p = np.zeros(2, np.float64)
    score = np.zeros((N, R), np.float64) if debug else None
    q = np.zeros((N, R), np.int64) if debug else None
    size = np.zeros(N, np.int64) if debug else None
    rc = lib().gorgo_oracle_replay(N, _p(ts), _p(il), _p(ol), _p(bo), _p(hi), block_tokens, R, batch,
                                   cache_blocks, prefill_ms_per_token, decode_ms_per_token, _p(rtt), _p(wv),
                                   float(scale), _p(route), _p(hit), _p(ttft), _p(e2e), _p(p), _p(score), _p(q),
                                   _p(size))
    if rc != 0:
        raise RuntimeError(f"gorgo_oracle_replay failed with code {rc}")
    return Replay(route, hit, ttft, e2e, float(p[0]), float(p[1]), score, q, size)


def replay_workload(wl, p: int, debug=False, trace=None) -> Replay:
    """Replay candidate p of a synth.tracegen.Workload."""
    return replay(trace if trace is not None else wl.trace, R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks,
                  prefill_ms_per_token=wl.prefill_ms_per_token, decode_ms_per_token=wl.decode_ms_per_token,
                  rtt_ms=wl.rtt_ms, w=wl.params[p], scale=wl.scale[p], block_tokens=wl.block_tokens, debug=debug)


def tuner_exp(x: float) -> float:
    return float(lib().gorgo_oracle_tuner_exp(float(x)))


def online_steps(N: int, window: int, hop: int) -> int:
    return int(lib().gorgo_oracle_online_steps(N, window, hop))


def philox4x32_10(ctr, key) -> np.ndarray:
    c, k = np.ascontiguousarray(ctr, np.uint32), np.ascontiguousarray(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().gorgo_oracle_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def splitmix64_next(x: int) -> int:
    return int(lib().gorgo_oracle_splitmix64_next(x & 0xFFFFFFFFFFFFFFFF))


POLICIES = {"cost-model": 0, "least-request": 1, "session-affinity": 2, "random": 3}


def _replay_ex(trace, R, batch, cache_blocks, prefill_ms_per_token, decode_ms_per_token, rtt_ms, w, scale,
               block_tokens, window, hop, schedule, z, lo, hi, sigma0, policy=0, seed=0, engine=None) -> Replay:
    N = int(trace.ts_ms.shape[0])
    ts = np.ascontiguousarray(trace.ts_ms, dtype=np.int64)
    il = np.ascontiguousarray(trace.in_len, dtype=np.int32)
    ol = np.ascontiguousarray(trace.out_len, dtype=np.int32)
    bo = np.ascontiguousarray(trace.blk_off, dtype=np.int64)
    hs = np.ascontiguousarray(trace.hash_ids, dtype=np.int64)
    rtt = np.ascontiguousarray(rtt_ms, dtype=np.float64)
    wv = np.ascontiguousarray(w, dtype=np.float64)
    steps = online_steps(N, window, hop)
    sched = None if schedule is None else np.ascontiguousarray(schedule, dtype=np.float64)
    zz = None if z is None else np.ascontiguousarray(z, dtype=np.float64)
    lov = None if lo is None else np.ascontiguousarray(lo, dtype=np.float64)
    hiv = None if hi is None else np.ascontiguousarray(hi, dtype=np.float64)
    assert rtt.shape == (R,) and wv.shape == (3,) and bo.shape == (N + 1,)
    assert sched is None or sched.shape == (steps, 3)
    assert zz is None or zz.shape == (steps, 3)
    route = np.zeros(N, np.uint8)
    hit = np.zeros(N, np.uint16)
    ttft = np.zeros(N, np.float64)
    e2e = np.zeros(N, np.float64)
    p = np.zeros(2, np.float64)
    theta_step = np.zeros((steps, 3), np.float64)
    fitness_step = np.zeros(steps, np.float64)
    fin = np.zeros(6, np.float64)
    if engine is None:
        rc = lib().gorgo_oracle_replay_ex(N, _p(ts), _p(il), _p(ol), _p(bo), _p(hs), block_tokens, R, batch,
                                          cache_blocks, prefill_ms_per_token, decode_ms_per_token, _p(rtt), _p(wv),
                                          float(scale), window, hop, _p(sched), _p(zz), _p(lov), _p(hiv),
                                          float(sigma0), int(policy), int(seed), _p(route), _p(hit), _p(ttft),
                                          _p(e2e), _p(p), None, None, None, _p(theta_step), _p(fitness_step), _p(fin))
    else:
        apf = np.ascontiguousarray(engine["prefill_ms_per_token"], dtype=np.float64)
        adec = np.ascontiguousarray(engine["decode_ms_per_token"], dtype=np.float64)
        kv = engine.get("kv_tokens")
        kv = None if kv is None else np.ascontiguousarray(kv, dtype=np.int64)
        assert apf.shape == (R,) and adec.shape == (R,) and (kv is None or kv.shape == (R,))
        rc = lib().gorgo_oracle_replay_engine(N, _p(ts), _p(il), _p(ol), _p(bo), _p(hs), block_tokens, R, batch,
                                              cache_blocks, prefill_ms_per_token, _p(apf), _p(adec), _p(kv),
                                              float(engine.get("slowdown", 0.0)), _p(rtt), _p(wv), float(scale),
                                              window, hop, _p(sched), _p(zz), _p(lov), _p(hiv), float(sigma0),
                                              int(policy), int(seed), _p(route), _p(hit), _p(ttft), _p(e2e), _p(p),
                                              _p(theta_step), _p(fitness_step), _p(fin))
    if rc != 0:
        raise RuntimeError(f"oracle replay failed with code {rc}")
    return Replay(route, hit, ttft, e2e, float(p[0]), float(p[1]), theta_step=theta_step, fitness_step=fitness_step,
                  theta_final=fin[:3].copy(), sigma_final=float(fin[3]), steps=int(fin[4]), accepted=int(fin[5]))


def replay_online(trace, *, R, batch, cache_blocks, prefill_ms_per_token, decode_ms_per_token, rtt_ms, theta0, z, lo,
                  hi, sigma0, window=128, hop=32, scale=1.0, block_tokens=512) -> Replay:
    """One replay with the online tuner: z[steps,3] are its standard normal draws."""
    return _replay_ex(trace, R, batch, cache_blocks, prefill_ms_per_token, decode_ms_per_token, rtt_ms, theta0, scale,
                      block_tokens, window, hop, None, z, lo, hi, sigma0)


def replay_schedule(trace, *, R, batch, cache_blocks, prefill_ms_per_token, decode_ms_per_token, rtt_ms, w, schedule,
                    window, hop, scale=1.0, block_tokens=512) -> Replay:
    """One replay whose weights are w, then schedule[h] after requests window + h * hop (no tuner)."""
    return _replay_ex(trace, R, batch, cache_blocks, prefill_ms_per_token, decode_ms_per_token, rtt_ms, w, scale,
                      block_tokens, window, hop, schedule, None, None, None, 0.0)


def replay_policy(trace, *, R, batch, cache_blocks, prefill_ms_per_token, decode_ms_per_token, rtt_ms, policy, seed=0,
                  scale=1.0, block_tokens=512) -> Replay:
    """One replay routed by a baseline policy ("least-request", "session-affinity", "random")."""
    return _replay_ex(trace, R, batch, cache_blocks, prefill_ms_per_token, decode_ms_per_token, rtt_ms, [0.0, 0.0, 0.0],
                      scale, block_tokens, 0, 0, None, None, None, None, 0.0, POLICIES[policy], seed)


def replay_engine(trace, *, R, batch, cache_blocks, prefill_ms_per_token, engine, rtt_ms, w=(0.0, 0.0, 0.0),
                  policy="cost-model", seed=0, scale=1.0, block_tokens=512, online=None) -> Replay:
    """One replay with the engine model of a replica.  engine = dict(prefill_ms_per_token=[R],
    decode_ms_per_token=[R], kv_tokens=[R] or None, slowdown=float); prefill_ms_per_token (the scalar) stays the
    cost model's rate.  online = dict(z=, lo=, hi=, sigma0=, window=, hop=) runs the tuner from weights w."""
    o = online or {}
    return _replay_ex(trace, R, batch, cache_blocks, prefill_ms_per_token, 0.0, rtt_ms, w, scale, block_tokens,
                      o.get("window", 0), o.get("hop", 0), None, o.get("z"), o.get("lo"), o.get("hi"),
                      o.get("sigma0", 0.0), POLICIES[policy], seed, engine=engine)


def replay_proxy(trace, *, R, batch, cache_blocks, prefill_ms_per_token, decode_ms_per_token=0.0, rtt_true, w,
                 probe_ms=30000, alpha=0.5, index_blocks=-1, engine=None, scale=1.0, block_tokens=512, online=None,
                 debug=False) -> Replay:
    """One replay with imperfect proxy knowledge: rtt_true[epochs,R] are the true round trip times per probe epoch,
    the cost model scores with their moving average; with index_blocks >= 0 it also takes its cached prefixes from
    an index of its own (an LRU of that many blocks per replica, 0 = it never forgets) instead of the replicas' caches.  engine / online as in replay_engine."""
    N = int(trace.ts_ms.shape[0])
    ts = np.ascontiguousarray(trace.ts_ms, dtype=np.int64)
    il = np.ascontiguousarray(trace.in_len, dtype=np.int32)
    ol = np.ascontiguousarray(trace.out_len, dtype=np.int32)
    bo = np.ascontiguousarray(trace.blk_off, dtype=np.int64)
    hs = np.ascontiguousarray(trace.hash_ids, dtype=np.int64)
    rt = np.ascontiguousarray(rtt_true, dtype=np.float64)
    wv = np.ascontiguousarray(w, dtype=np.float64)
    assert rt.ndim == 2 and rt.shape[1] == R and wv.shape == (3,) and bo.shape == (N + 1,)
    E = rt.shape[0]
    o = online or {}
    window, hop = o.get("window", 0), o.get("hop", 0)
    steps = online_steps(N, window, hop)
    zz = None if online is None else np.ascontiguousarray(o["z"], dtype=np.float64)
    lov = None if online is None else np.ascontiguousarray(o["lo"], dtype=np.float64)
    hiv = None if online is None else np.ascontiguousarray(o["hi"], dtype=np.float64)
    assert zz is None or zz.shape == (steps, 3)
    apf = adec = kv = None
    slow = 0.0
    if engine is not None:
        apf = np.ascontiguousarray(engine["prefill_ms_per_token"], dtype=np.float64)
        adec = np.ascontiguousarray(engine["decode_ms_per_token"], dtype=np.float64)
        kv = engine.get("kv_tokens")
        kv = None if kv is None else np.ascontiguousarray(kv, dtype=np.int64)
        slow = float(engine.get("slowdown", 0.0))
        assert apf.shape == (R,) and adec.shape == (R,) and (kv is None or kv.shape == (R,))
    route = np.zeros(N, np.uint8)
    hit = np.zeros(N, np.uint16)
    believed = np.zeros(N, np.uint16)
    ttft = np.zeros(N, np.float64)
    e2e = np.zeros(N, np.float64)
    p = np.zeros(2, np.float64)
    est = np.zeros((E, R), np.float64)
    score = np.zeros((N, R), np.float64) if debug else None
    theta_step = np.zeros((steps, 3), np.float64)
    fitness_step = np.zeros(steps, np.float64)
    fin = np.zeros(6, np.float64)
    rc = lib().gorgo_oracle_replay_proxy(N, _p(ts), _p(il), _p(ol), _p(bo), _p(hs), block_tokens, R, batch, cache_blocks,
                                         prefill_ms_per_token, decode_ms_per_token, _p(apf), _p(adec), _p(kv), slow,
                                         E, int(probe_ms), _p(rt), float(alpha), int(index_blocks), _p(wv),
                                         float(scale), window, hop, _p(zz), _p(lov), _p(hiv), float(o.get("sigma0", 0.0)),
                                         _p(route), _p(hit), _p(ttft), _p(e2e), _p(p), _p(score), _p(est), _p(believed),
                                         _p(theta_step), _p(fitness_step), _p(fin))
    if rc != 0:
        raise RuntimeError(f"oracle replay failed with code {rc}")
    return Replay(route, hit, ttft, e2e, float(p[0]), float(p[1]), score=score, theta_step=theta_step,
                  fitness_step=fitness_step, theta_final=fin[:3].copy(), sigma_final=float(fin[3]), steps=int(fin[4]),
                  accepted=int(fin[5]), rtt_est=est, believed_hit=believed)

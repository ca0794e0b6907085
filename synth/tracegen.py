"""Seeded synthetic workloads shaped like the paper's replay traces.

This module only manufactures INPUTS (a Mooncake-style request trace, replica
RTTs, service constants, candidate weight vectors, time scales).  It contains
none of the routing method's arithmetic: no score, no prefix match, no cache,
no queue, no percentile.  Both the CPU oracle's tests and the HIP path's tests
draw their inputs from here so that the two sides see identical bytes.

Trace shape (Sec. 3 "Dataset", Table 1, Appendix window statistics): multi-turn
conversations whose prompts grow turn by turn, so that ~90 % of a turn's
512-token blocks repeat the previous turn of the same user and almost nothing is
shared across users; long prompts; roughly 13-16 requests per user.  A trace
record carries a timestamp (integer ms), input/output token counts and one
integer hash id per 512-token prompt block (Mooncake FAST'25 layout, Sec. 1/3).

Five named workloads are provided (``config(1)`` .. ``config(5)``); each one
inherits every field it does not override from the previous one.
"""
from __future__ import annotations

import json
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

MASTER_SEED = 260211688
BLOCK_TOKENS = 512

# purposes of the independent random streams
_P_USERS, _P_TURNS, _P_FIRST, _P_NEW, _P_OUT, _P_ARRIVAL, _P_BURST, _P_RTT, _P_PARAMS, _P_THETA = range(10)


def _rng(config_index: int, purpose: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([MASTER_SEED + config_index, purpose])))


@dataclass
class Trace:
    ts_ms: np.ndarray      # int64 [N], non-decreasing
    in_len: np.ndarray     # int32 [N] input tokens
    out_len: np.ndarray    # int32 [N] output tokens (>= 1)
    blk_off: np.ndarray    # int64 [N+1] CSR offsets into hash_ids
    hash_ids: np.ndarray   # int64 [sum n_r]

    @property
    def N(self) -> int:
        return int(self.ts_ms.shape[0])

    def ids_of(self, r: int) -> np.ndarray:
        return self.hash_ids[self.blk_off[r]:self.blk_off[r + 1]]

    def head(self, n: int) -> "Trace":
        """First n requests as a trace of their own."""
        n = min(n, self.N)
        e = int(self.blk_off[n])
        return Trace(self.ts_ms[:n].copy(), self.in_len[:n].copy(), self.out_len[:n].copy(),
                     self.blk_off[:n + 1].copy(), self.hash_ids[:e].copy())

    def write_jsonl(self, path: str) -> None:
        """One JSON object per line: timestamp, input_length, output_length, hash_ids."""
        with open(path, "w") as f:
            for r in range(self.N):
                f.write(json.dumps({"timestamp": int(self.ts_ms[r]), "input_length": int(self.in_len[r]),
                                    "output_length": int(self.out_len[r]),
                                    "hash_ids": [int(x) for x in self.ids_of(r)]}) + "\n")


@dataclass
class Workload:
    name: str
    config_index: int
    trace: Trace
    R: int
    rtt_ms: np.ndarray            # float64 [R]
    batch: int                    # concurrent service slots per replica
    cache_blocks: int             # 0 = unbounded
    prefill_ms_per_token: float
    decode_ms_per_token: float
    params: Optional[np.ndarray]  # float64 [P,3] = (w_rtt, w_prefill, w_queue) per replay; None = from the ES
    scale: Optional[np.ndarray]   # float64 [P] time scale per replay
    es: dict = field(default_factory=dict)
    block_tokens: int = BLOCK_TOKENS
    notes: dict = field(default_factory=dict)

    @property
    def P(self) -> int:
        return 0 if self.params is None else int(self.params.shape[0])


def _expand_ranges(starts: np.ndarray, lens: np.ndarray) -> np.ndarray:
    """Concatenation of arange(starts[i], starts[i]+lens[i])."""
    total = int(lens.sum())
    off = np.cumsum(lens) - lens
    return np.repeat(starts - off, lens) + np.arange(total, dtype=np.int64)


def _poisson_timestamps(rng: np.random.Generator, N: int, rate_per_s: float) -> np.ndarray:
    gaps_ms = rng.exponential(1000.0 / rate_per_s, size=N)
    return np.floor(np.cumsum(gaps_ms)).astype(np.int64)


def _bursty_timestamps(rng_arr, rng_burst, N: int, base_rate_per_s: float, window_s: float = 10.0,
                       burst_prob: float = 0.25, lo: float = 2.0, hi: float = 5.0) -> np.ndarray:
    """Piecewise-constant-rate Poisson process: each window of `window_s` seconds is a burst with
    probability `burst_prob` (rate multiplied by U[lo,hi]) and runs at the base rate otherwise."""
    n_win = int(N / (base_rate_per_s * window_s)) + 64          # base-rate windows alone already suffice
    is_burst = rng_burst.random(n_win) < burst_prob
    mult = np.where(is_burst, rng_burst.uniform(lo, hi, n_win), 1.0)
    rate_per_ms = base_rate_per_s * mult / 1000.0
    win_ms = window_s * 1000.0
    cum = np.concatenate([[0.0], np.cumsum(rate_per_ms * win_ms)])   # expected arrivals up to each window edge
    s = np.cumsum(rng_arr.exponential(1.0, size=N))                  # unit-rate arrival epochs
    edges = np.arange(n_win + 1) * win_ms
    assert s[-1] < cum[-1]
    return np.floor(np.interp(s, cum, edges)).astype(np.int64)


def _build_trace(config_index: int, N: int, n_users: int, zipf: Optional[float], long_prompts: bool,
                 cap_blocks: int, bursty: bool, rate_per_s: float = 20.0) -> tuple[Trace, dict]:
    ru, rt, rf, rn = (_rng(config_index, p) for p in (_P_USERS, _P_TURNS, _P_FIRST, _P_NEW))
    if zipf is None:
        users = ru.integers(0, n_users, size=N)
        pop = None
    else:
        pop = np.arange(1, n_users + 1, dtype=np.float64) ** (-zipf)
        pop /= pop.sum()
        users = ru.choice(n_users, size=N, p=pop)
    turns_draw = rt.integers(1, 9, size=N)                       # U{1..8} turns per conversation
    if long_prompts:
        tok = np.exp(np.log(20000.0) + 0.75 * rf.standard_normal(N))
        first_draw = np.clip(np.ceil(tok / BLOCK_TOKENS), 1, cap_blocks).astype(np.int64)
        new_draw = None
    else:
        first_draw = rf.integers(1, 7, size=N)                   # U{1..6} blocks
        new_draw = rn.integers(1, 7, size=N)

    # conversation bookkeeping (structure only: which id ranges make up which request)
    turns_left = [0] * n_users
    conv_of_user = [-1] * n_users
    conv_nblk: list[int] = []
    conv_ranges: list[list[tuple[int, int]]] = []
    req_conv = np.empty(N, dtype=np.int64)
    req_nranges = np.empty(N, dtype=np.int64)
    req_nblk = np.empty(N, dtype=np.int64)
    counter = 1                                                  # ids come from one global counter from 1
    users_l, turns_l, first_l = users.tolist(), turns_draw.tolist(), first_draw.tolist()
    new_l = None if new_draw is None else new_draw.tolist()
    for r in range(N):
        u = users_l[r]
        if turns_left[u] == 0:
            c = len(conv_ranges)
            conv_of_user[u] = c
            turns_left[u] = turns_l[r]
            n = first_l[r]
            conv_ranges.append([(counter, n)])
            conv_nblk.append(n)
            counter += n
        else:
            c = conv_of_user[u]
            n_prev = conv_nblk[c]
            add = new_l[r] if new_l is not None else max(1, int(n_prev / 9.0 + 0.5))
            add = min(add, cap_blocks - n_prev)
            if add > 0:
                conv_ranges[c].append((counter, add))
                conv_nblk[c] = n_prev + add
                counter += add
        turns_left[u] -= 1
        req_conv[r] = c
        req_nranges[r] = len(conv_ranges[c])
        req_nblk[r] = conv_nblk[c]

    # flatten conversation ranges, then gather them per request
    conv_nr = np.array([len(x) for x in conv_ranges], dtype=np.int64)
    conv_roff = np.concatenate([[0], np.cumsum(conv_nr)])
    flat = np.array([p for x in conv_ranges for p in x], dtype=np.int64).reshape(-1, 2)
    rsel = _expand_ranges(conv_roff[req_conv], req_nranges)      # (request, range) pairs -> flat range index
    hash_ids = _expand_ranges(flat[rsel, 0], flat[rsel, 1])
    blk_off = np.concatenate([[0], np.cumsum(req_nblk)]).astype(np.int64)
    assert hash_ids.shape[0] == blk_off[-1]

    ro = _rng(config_index, _P_OUT)
    out_len = np.maximum(1, np.rint(np.exp(5.0 + 0.8 * ro.standard_normal(N)))).astype(np.int32)
    if bursty:
        ts = _bursty_timestamps(_rng(config_index, _P_ARRIVAL), _rng(config_index, _P_BURST), N, rate_per_s)
    else:
        ts = _poisson_timestamps(_rng(config_index, _P_ARRIVAL), N, rate_per_s)
    in_len = (req_nblk * BLOCK_TOKENS).astype(np.int32)
    notes = {"unique_ids": counter - 1, "conversations": len(conv_ranges),
             "mean_blocks": float(req_nblk.mean()), "max_blocks": int(req_nblk.max())}
    if pop is not None:
        top = max(1, n_users // 100)
        notes["top1pct_user_share"] = float((users < top).mean())
    return Trace(ts, in_len, out_len, blk_off, hash_ids), notes


def _log_uniform_rtt(config_index: int, R: int) -> np.ndarray:
    return 10.0 * 100.0 ** _rng(config_index, _P_RTT).random(R)


ES_DEFAULTS = {  # initial weights, ranges and step size of the tuner (Sec. 4 "Tuning and evaluation windows")
    "theta": [0.5, 1.0, 0.1], "sigma": 0.5, "lo": [0.05, 1.0, 0.05], "hi": [2.0, 1.0, 0.5],
}

_cache: dict = {}


def config(index: int, n_requests: Optional[int] = None) -> Workload:
    """Workload `index` (1..5).  `n_requests` truncates the trace to its first requests (parity-test sizes)."""
    key = (index, n_requests)
    if key in _cache:
        return _cache[key]
    svc = dict(batch=8, prefill_ms_per_token=0.05, decode_ms_per_token=20.0)
    if index == 1:
        tr, notes = _build_trace(1, 2000, 200, None, False, 1 << 30, False)
        params = _rng(1, _P_PARAMS).uniform(0.0, 2.0, size=(16, 3))
        w = Workload("tiny", 1, tr, 4, np.array([10.0, 40.0, 120.0, 300.0]), cache_blocks=0, params=params,
                     scale=np.ones(16), notes=notes, **svc)
    elif index == 2:
        tr, notes = _build_trace(2, 50000, 3000, None, True, 250, False)
        params = _rng(2, _P_PARAMS).uniform(0.0, 2.0, size=(64, 3))
        w = Workload("regional", 2, tr, 8, _log_uniform_rtt(2, 8), cache_blocks=4000, params=params,
                     scale=np.ones(64), notes=notes, **svc)
    elif index in (3, 4):
        base = _cache.get(("trace3",))
        if base is None:
            base = _build_trace(3, 200000, 12000, 1.1, True, 256, True)
            _cache[("trace3",)] = base
        tr, notes = base
        theta = _rng(3, _P_THETA).uniform(0.5, 1.5, size=3)
        params = theta + 0.1 * _rng(3, _P_PARAMS).standard_normal((256, 3))
        if index == 3:
            w = Workload("long-context", 3, tr, 16, _log_uniform_rtt(3, 16), cache_blocks=8000, params=params,
                         scale=np.ones(256), notes=dict(notes), **svc)
        else:
            scales = np.array([0.25, 0.5, 0.75, 1.0, 1.5, 2.0, 3.0, 4.0])
            w = Workload("saturation-sweep", 4, tr, 16, _log_uniform_rtt(3, 16), cache_blocks=8000,
                         params=np.tile(params[:128], (8, 1)), scale=np.repeat(scales, 128),
                         notes=dict(notes), **svc)
    elif index == 5:
        tr, notes = _build_trace(5, 1000000, 60000, 1.1, True, 256, False)
        w = Workload("large", 5, tr, 32, _log_uniform_rtt(5, 32), cache_blocks=16000, params=None, scale=None,
                     es=dict(ES_DEFAULTS, P=1024, seed=MASTER_SEED + 5, generations=10), notes=notes, **svc)
    else:
        raise ValueError("config index must be 1..5")
    if n_requests is not None:
        w.trace = w.trace.head(n_requests)
    _cache[key] = w
    return w


def random_small(seed: int, N: int, R: int, *, n_ids: int = 12, max_blocks: int = 5, consistent: bool = True,
                 gap_ms: int = 40, block_tokens: int = BLOCK_TOKENS) -> Trace:
    """Tiny random trace for brute-force and edge-case tests.  With consistent=False block ids are drawn
    independently per position, so one id can appear at several positions, under several predecessors, and
    twice inside one request."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([MASTER_SEED, 99, seed])))
    ts = np.cumsum(rng.integers(0, gap_ms + 1, size=N)).astype(np.int64)
    lists = []
    chains = [list(range(1 + c * max_blocks, 1 + (c + 1) * max_blocks)) for c in range(max(1, n_ids // max_blocks))]
    for _ in range(N):
        n = int(rng.integers(1, max_blocks + 1))
        if consistent:
            c = chains[int(rng.integers(0, len(chains)))]
            lists.append(c[:n])
        else:
            lists.append([int(x) for x in rng.integers(1, n_ids + 1, size=n)])
    nblk = np.array([len(x) for x in lists], dtype=np.int64)
    blk_off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64)
    ids = np.array([x for l in lists for x in l], dtype=np.int64)
    # input length: whole blocks, minus a random partial last block now and then
    in_len = (nblk * block_tokens - rng.integers(0, block_tokens // 2, size=N) * (rng.random(N) < 0.3)).astype(np.int32)
    out_len = rng.integers(1, 6, size=N).astype(np.int32)
    return Trace(ts, in_len, out_len, blk_off, ids)


def random_forest(seed: int, N: int, *, roots: int = 3, max_blocks: int = 40, grow: int = 6, gap_ms: int = 40,
                  block_tokens: int = BLOCK_TOKENS, keep: float = 0.0) -> Trace:
    """Random chain-consistent trace with branching: every request takes a prefix of an earlier request's blocks
    (cut anywhere) and, more often than not, appends fresh blocks to it, so paths share prefixes, fork in the
    middle of runs and end inside them.  Ids are fresh integers, so every id has one predecessor and position."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([MASTER_SEED, 98, seed])))
    ts = np.cumsum(rng.integers(0, gap_ms + 1, size=N)).astype(np.int64)
    nxt = 1
    paths, lists = [], []
    for _ in range(N):
        if len(paths) < roots or rng.random() < 0.02:
            base = []
        else:
            p = paths[int(rng.integers(0, len(paths)))]
            base = p if rng.random() < keep else p[:int(rng.integers(1, len(p) + 1))]   # keep: paths grow long
        add = int(rng.integers(0 if base else 1, grow + 1)) if rng.random() < 0.7 or not base else 0
        add = min(add, max_blocks - len(base))
        path = base + list(range(nxt, nxt + add))
        nxt += add
        paths.append(path)
        if len(paths) > 64:
            paths.pop(int(rng.integers(0, len(paths))))
        lists.append(path)
    nblk = np.array([len(x) for x in lists], dtype=np.int64)
    blk_off = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64)
    ids = np.array([x for l in lists for x in l], dtype=np.int64)
    in_len = (nblk * block_tokens - rng.integers(0, block_tokens // 2, size=N) * (rng.random(N) < 0.3)).astype(np.int32)
    out_len = rng.integers(1, 40, size=N).astype(np.int32)
    return Trace(ts, in_len, out_len, blk_off, ids)


def engine_recipe(wl: Workload, seed: int = 0, *, spread: float = 2.0, kv_requests: float = 4.0,
                  slowdown: float = 0.05) -> dict:
    """Seeded parameters of an uneven fleet for the engine model of a replica: replica i prefills and decodes at the
    workload's rates times spread^u, u uniform in (-1, 1), drawn independently for the two rates; every replica's KV
    budget is kv_requests times the tokens (input + output) of the largest request of the trace."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([MASTER_SEED, 97, wl.config_index, seed])))
    most = int((wl.trace.in_len.astype(np.int64) + wl.trace.out_len).max()) if wl.trace.N else 1
    return dict(prefill_ms_per_token=wl.prefill_ms_per_token * spread ** rng.uniform(-1.0, 1.0, wl.R),
                decode_ms_per_token=wl.decode_ms_per_token * spread ** rng.uniform(-1.0, 1.0, wl.R),
                kv_tokens=np.full(wl.R, int(kv_requests * most), np.int64), slowdown=float(slowdown))


def rtt_walk(wl: Workload, epochs: int, seed: int = 0, *, step: float = 0.15, pull: float = 0.9) -> np.ndarray:
    """Seeded true round trip times per probe epoch [epochs, R]: each replica's RTT starts at the workload's value and
    its logarithm wanders around it (x_e = pull * x_(e-1) + step * normal draw: deviations of about a third in the
    long run), rounded to 0.001 ms."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([MASTER_SEED, 96, wl.config_index, seed])))
    eps = step * rng.standard_normal((epochs, wl.R))
    x = np.zeros((epochs, wl.R))
    for e in range(1, epochs):
        x[e] = pull * x[e - 1] + eps[e]
    return np.round(wl.rtt_ms[None, :] * np.exp(x), 3)

"""Test-side helpers: golden-file loading and independent pure-Python models used to pin the oracle.

Nothing here is imported by the oracle or by the GPU library.
"""
import json
import os

import numpy as np

from synth.tracegen import Trace

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        g = json.load(f)
    reqs = g["requests"]
    nblk = np.array([len(q["hash_ids"]) for q in reqs], dtype=np.int64)
    tr = Trace(np.array([q["timestamp"] for q in reqs], dtype=np.int64),
               np.array([q["input_length"] for q in reqs], dtype=np.int32),
               np.array([q["output_length"] for q in reqs], dtype=np.int32),
               np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64),
               np.array([x for q in reqs for x in q["hash_ids"]], dtype=np.int64))
    return g, tr


def model_kwargs(g):
    m = g["model"]
    return dict(R=m["R"], batch=m["batch"], cache_blocks=m["cache_blocks"], block_tokens=m["block_tokens"],
                prefill_ms_per_token=m["prefill_ms_per_token"], decode_ms_per_token=m["decode_ms_per_token"],
                rtt_ms=g["rtt_ms"], w=g["w"], scale=g["scale"])


class ForcedRouteModel:
    """Independent pure-Python replay in which the ROUTE of every request is dictated from outside.

    For each request it reports the score every replica would have had (Eq. 3) given the state that the
    dictated predecessors induced; a route sequence is self-consistent when every dictated route is the
    lowest-index minimum of those scores.  The cache is a recency-ordered Python list (move-to-front,
    evict from the cold end), the in-flight set a plain list scanned at each request: different data
    structures from the oracle's on purpose.  `w` is one weight vector, or one per request (a weight
    schedule dictated from outside, like the routes).  `proxy` = dict(rtt_true=[epochs][R], probe_ms=, alpha=,
    index_blocks=) switches on imperfect proxy knowledge: round trip times per probe epoch (scored through their
    moving average), and, with index_blocks >= 0, scores that take their cached prefix from the proxy's own index
    of each replica (a recency list like the replica's, with that capacity; 0 = it never forgets).
    """

    def __init__(self, trace, R, batch, cache_blocks, block_tokens, a_pf, a_dec, rtt, w, scale, proxy=None):
        self.tr, self.R, self.B, self.C, self.bt = trace, R, batch, cache_blocks, block_tokens
        self.a_pf, self.a_dec, self.rtt, self.w, self.scale = a_pf, a_dec, list(rtt), list(w), scale
        self.proxy = proxy

    def run(self, routes):
        tr = self.tr
        lru = [[] for _ in range(self.R)]            # coldest first ... hottest last
        free = [[0.0] * self.B for _ in range(self.R)]
        inflight = [[] for _ in range(self.R)]       # (done, tokens)
        consistent = True
        out = dict(score=[], hit=[], ttft=[], e2e=[], q=[], done=[], cnt=[], believed=[])
        px = self.proxy
        seen = [[] for _ in range(self.R)]           # the proxy's own index: coldest first ... hottest last
        if px:
            true = [[float(x) for x in row] for row in px["rtt_true"]]
            est = [list(true[0])]
            for e in range(1, len(true)):
                est.append([px["alpha"] * true[e][i] + (1.0 - px["alpha"]) * est[e - 1][i] for i in range(self.R)])
        for r in range(tr.N):
            ids = [int(x) for x in tr.ids_of(r)]
            L, O = int(tr.in_len[r]), int(tr.out_len[r])
            t = float(int(tr.ts_ms[r])) * self.scale
            q = []
            for i in range(self.R):
                inflight[i] = [(d, tok) for (d, tok) in inflight[i] if not d <= t]
                q.append(sum(tok for _, tok in inflight[i]))
            scores, us, ms, seen_ms = [], [], [], []
            rtt_score, rtt_real = self.rtt, self.rtt
            if px:
                e = 0
                while e + 1 < len(true) and float((e + 1) * px["probe_ms"]) <= t:
                    e += 1
                rtt_score, rtt_real = est[e], true[e]
            for i in range(self.R):
                m = 0
                while m < len(ids) and ids[m] in lru[i]:
                    m += 1
                u = L - min(L, self.bt * m)
                ms_seen = m
                if px and px["index_blocks"] >= 0:
                    ms_seen = 0
                    while ms_seen < len(ids) and ids[ms_seen] in seen[i]:
                        ms_seen += 1
                pf = self.a_pf * float(L - min(L, self.bt * ms_seen))
                qd = self.a_pf * float(q[i])
                w = self.w[r] if isinstance(self.w[0], (list, tuple, np.ndarray)) else self.w
                scores.append((w[0] * rtt_score[i] + w[1] * pf) + w[2] * qd)
                us.append(u)
                ms.append(m)
                seen_ms.append(ms_seen)
            best = min(range(self.R), key=lambda i: (scores[i], i))
            i = routes[r]
            if i != best:
                consistent = False
            # cache: evict cold entries that are not part of this request, then touch deepest block first
            # so that the root ends up hottest
            def touch(lst, cap):
                mine = set(ids)
                if cap > 0:
                    n_new = len([x for x in mine if x not in lst])
                    excess = len(lst) + n_new - cap
                    keep = []
                    for x in lst:
                        if excess > 0 and x not in mine:
                            excess -= 1
                        else:
                            keep.append(x)
                    lst[:] = keep
                first_pos = {}
                for k, x in enumerate(ids):
                    first_pos.setdefault(x, k)
                for x in sorted(first_pos, key=lambda x: -first_pos[x]):
                    if x in lst:
                        lst.remove(x)
                    lst.append(x)
            touch(lru[i], self.C)
            if px and px["index_blocks"] >= 0:
                touch(seen[i], px["index_blocks"])
            half = 0.5 * rtt_real[i]
            a = t + half
            ks = min(range(self.B), key=lambda k: (free[i][k], k))
            s = max(a, free[i][ks])
            f = s + self.a_pf * float(us[i])
            e = f + self.a_dec * float(O)
            free[i][ks] = e
            done = e + half
            inflight[i].append((done, L))
            out["score"].append(scores)
            out["hit"].append(ms[i])
            out["believed"].append(seen_ms[i])
            out["ttft"].append((f + half) - t)
            out["e2e"].append(done - t)
            out["q"].append(q)
            out["cnt"].append([len(inflight[j]) - (1 if j == i else 0) for j in range(self.R)])   # before dispatch
            out["done"].append(done)
        out["consistent"] = consistent
        return out

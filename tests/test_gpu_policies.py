"""GPU parity of the baseline policies (Sec. 4 "Baseline policies") against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import paper_2602_11688_amd as g
from oracle import binding as ob
from synth import tracegen as tg
from tests.gpu_helpers import assert_replay_equal, gpu_eval, load

pytestmark = pytest.mark.gpu


def _model(wl, **over):
    kw = dict(R=wl.R, batch=wl.batch, cache_blocks=wl.cache_blocks, prefill_ms_per_token=wl.prefill_ms_per_token,
              decode_ms_per_token=wl.decode_ms_per_token)
    kw.update(over)
    return g.Model(**kw)


def _check(tr, model, rtt, policy, scales, seeds=None):
    import torch
    res = g.eval_policy(load(tr), model, rtt, policy, scales, seeds=seeds)
    torch.cuda.synchronize()
    got = dict(route=res.route.cpu().numpy(), hit=res.hit_blocks.cpu().numpy(), ttft=res.ttft_ms.cpu().numpy(),
               e2e=res.e2e_ms.cpu().numpy(), p95_ttft=res.p95_ttft_ms.cpu().numpy(), p95_e2e=res.p95_e2e_ms.cpu().numpy())
    for p, sc in enumerate(scales):
        ref = ob.replay_policy(tr, R=model.R, batch=model.batch, cache_blocks=model.cache_blocks,
                               prefill_ms_per_token=model.prefill_ms_per_token,
                               decode_ms_per_token=model.decode_ms_per_token, rtt_ms=rtt, policy=policy,
                               seed=0 if seeds is None else int(seeds[p]), scale=float(sc), block_tokens=model.block_tokens)
        assert_replay_equal(got, p, ref, policy)
    return got


@pytest.mark.parametrize("policy", ["least-request", "session-affinity", "random"])
def test_policies_on_saturated_and_idle_replicas(policy):
    wl = tg.config(1)
    seeds = np.array([1, 2, 2**40 + 7, 99], np.uint64) if policy == "random" else None
    got = _check(wl.trace, _model(wl), wl.rtt_ms, policy, [1.0, 2.0, 4.0, 0.5], seeds)
    assert len(set(got["route"][0].tolist())) == wl.R


@pytest.mark.parametrize("policy", ["least-request", "session-affinity", "random"])
def test_policies_with_bounded_caches(policy):
    wl = tg.config(2, 6000)
    seeds = np.array([5, 6], np.uint64) if policy == "random" else None
    _check(wl.trace, _model(wl), wl.rtt_ms, policy, [1.0, 1.5], seeds)


def test_policies_at_the_replica_and_slot_limits():
    tr = tg.random_small(9, 1500, 64, n_ids=400, max_blocks=6, consistent=True, gap_ms=3)
    rtt = np.linspace(5.0, 200.0, 64)
    for policy in ("least-request", "session-affinity", "random"):
        _check(tr, g.Model(64, 16, 40, 0.05, 20.0), rtt, policy, [1.0], np.array([3], np.uint64))
    _check(tr, g.Model(1, 64, 12, 0.05, 20.0), [9.0], "least-request", [1.0])


def test_special_case_weights_are_the_other_two_baselines():
    # prefix-cache = weights (0, 1, 0): every request goes to a replica with the longest cached prefix;
    # least-load from what the proxy tracks = weights (0, 0, 1)
    wl = tg.config(2, 3000)
    model = _model(wl)
    got = gpu_eval(wl.trace, model, wl.rtt_ms, [[0.0, 1.0, 0.0], [0.0, 0.0, 1.0]], 1.0)
    for p, w in enumerate(([0.0, 1.0, 0.0], [0.0, 0.0, 1.0])):
        ref = ob.replay(wl.trace, R=model.R, batch=model.batch, cache_blocks=model.cache_blocks,
                        prefill_ms_per_token=model.prefill_ms_per_token, decode_ms_per_token=model.decode_ms_per_token,
                        rtt_ms=wl.rtt_ms, w=w, debug=(p == 1))
        assert_replay_equal(got, p, ref, "special weights")
        if p == 1:
            assert all(ref.route[r] == int(np.argmin(ref.q[r])) for r in range(wl.trace.N))


def test_policy_arguments():
    wl = tg.config(1, 100)
    with pytest.raises(g.GorgoError):
        g.eval_policy(load(wl.trace), _model(wl), wl.rtt_ms, "random", [1.0])            # no seeds
    with pytest.raises(KeyError):
        g.eval_policy(load(wl.trace), _model(wl), wl.rtt_ms, "round-robin", [1.0])       # not a policy of Sec. 4

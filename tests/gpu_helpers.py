"""Shared pieces of the GPU parity tests: run the HIP library and the CPU oracle on the same inputs and
compare element by element.  Routes and hit counts must be bit-exact; latencies agree to 1e-9 relative."""
import contextlib

import numpy as np

import paper_2602_11688_amd as g
from oracle import binding as ob

RTOL = 1e-9      # stated tolerance for TTFT / E2E; both sides use the same fp64 operation order


def load(tr):
    return g.Trace.from_arrays(tr.ts_ms, tr.in_len, tr.out_len, tr.blk_off, tr.hash_ids)


PATH_NAMES = {0: "auto", 1: "block-tables", 2: "segment-rows"}


@contextlib.contextmanager
def formulation(path, table_factor_percent=None):
    """Calls inside run the given formulation of the cache state (1 = hashed block tables, 2 = dense segment rows),
    optionally with larger block tables, whatever the trace would get by itself."""
    before = g.default_options().table_factor_percent
    g.set_replay_path(path)
    if table_factor_percent is not None:
        g.set_table_factor_percent(table_factor_percent)
    try:
        yield
    finally:
        g.set_replay_path(0)
        g.set_table_factor_percent(before)


def gpu_eval(tr, model: g.Model, rtt, params, scale, handle=None, path=0, packing=True):
    import torch
    h = handle if handle is not None else load(tr)
    g.set_replay_path(path)
    g.set_replay_packing(1 if packing else 0)
    try:
        res = g.eval_population(h, model, rtt, params, scale)
        torch.cuda.synchronize()
    finally:
        g.set_replay_path(0)
        g.set_replay_packing(2)
    out = dict(route=res.route.cpu().numpy(), hit=res.hit_blocks.cpu().numpy(), ttft=res.ttft_ms.cpu().numpy(),
               e2e=res.e2e_ms.cpu().numpy(), p95_ttft=res.p95_ttft_ms.cpu().numpy(),
               p95_e2e=res.p95_e2e_ms.cpu().numpy())
    return out


def oracle_eval(tr, model: g.Model, rtt, w, scale):
    return ob.replay(tr, R=model.R, batch=model.batch, cache_blocks=model.cache_blocks,
                     prefill_ms_per_token=model.prefill_ms_per_token, decode_ms_per_token=model.decode_ms_per_token,
                     rtt_ms=rtt, w=w, scale=scale, block_tokens=model.block_tokens)


def assert_replay_equal(got, p, ref, label=""):
    bad = np.nonzero(got["route"][p] != ref.route)[0]
    assert bad.size == 0, f"{label} replay {p}: first route mismatch at request {bad[0]} ({bad.size} in all)"
    bad = np.nonzero(got["hit"][p] != ref.hit_blocks)[0]
    assert bad.size == 0, f"{label} replay {p}: first hit-count mismatch at request {bad[0]}"
    np.testing.assert_allclose(got["ttft"][p], ref.ttft_ms, rtol=RTOL, atol=0, err_msg=f"{label} ttft replay {p}")
    np.testing.assert_allclose(got["e2e"][p], ref.e2e_ms, rtol=RTOL, atol=0, err_msg=f"{label} e2e replay {p}")
    if ref.ttft_ms.size:
        assert abs(got["p95_ttft"][p] - ref.p95_ttft_ms) <= RTOL * abs(ref.p95_ttft_ms), f"{label} p95 ttft replay {p}"
        assert abs(got["p95_e2e"][p] - ref.p95_e2e_ms) <= RTOL * abs(ref.p95_e2e_ms), f"{label} p95 e2e replay {p}"


def check_population(tr, model, rtt, params, scale, replays=None, label="", paths=None):
    """Every formulation the trace admits (hashed block tables always, segment rows when the trace is
    chain-consistent) against the oracle.  Returns the outputs of the last formulation run."""
    params = np.asarray(params, np.float64)
    P = params.shape[0]
    scale = np.broadcast_to(np.asarray(scale, np.float64), (P,))
    h = load(tr)
    if paths is None:
        paths = [1, 2] if h.info()["chain_consistent"] else [1]
    which = list(range(P) if replays is None else replays)
    refs = {p: oracle_eval(tr, model, rtt, params[p], float(scale[p])) for p in which}
    got = None
    for path in paths:
        # segment rows: with two replays per wavefront pair where the shape allows it, and without
        for packing in ((False, True) if path == 2 else (True,)):
            par, sc = params, scale
            if packing and path == 2 and P % 2:      # pairs need an even number of replays: one more, not compared
                par, sc = np.concatenate([params, params[:1]]), np.concatenate([scale, scale[:1]])
            got = gpu_eval(tr, model, rtt, par, sc, handle=h, path=path, packing=packing)
            for p in which:
                assert_replay_equal(got, p, refs[p], f"{label} [{PATH_NAMES[path]}{'' if packing else ', unpacked'}]")
    return got

"""The entry point that allocates nothing (gorgo_eval_population_static) against gorgo_eval_population on the same
inputs: two calls in a row, the second with a smaller input, so that what the first call left in the library's
static scratch array is there when the second starts."""
import numpy as np
import pytest

import paper_2602_11688_amd as g
from paper_2602_11688_amd import binding
from synth import tracegen as tg

pytestmark = pytest.mark.gpu


def _both(wl, nreq_cache, P):
    import torch
    tr = g.Trace.from_arrays(wl.trace.ts_ms, wl.trace.in_len, wl.trace.out_len, wl.trace.blk_off, wl.trace.hash_ids)
    model = g.Model(wl.R, wl.batch, nreq_cache, wl.prefill_ms_per_token, wl.decode_ms_per_token)
    par, sc = wl.params[:P], wl.scale[:P]
    assert g.workspace_bytes(tr, model, P) <= binding.STATIC_SCRATCH_BYTES
    ref = g.eval_population(tr, model, wl.rtt_ms, par, sc)
    torch.cuda.synchronize()
    got = g.eval_population_static(tr, model, wl.rtt_ms, par, sc)
    torch.cuda.synchronize()
    for name in ("route", "hit_blocks"):
        a, b = getattr(got, name).cpu().numpy(), getattr(ref, name).cpu().numpy()
        assert np.array_equal(a, b), name
    for name in ("ttft_ms", "e2e_ms", "p95_ttft_ms", "p95_e2e_ms"):
        a, b = getattr(got, name).cpu().numpy(), getattr(ref, name).cpu().numpy()
        np.testing.assert_allclose(a, b, rtol=1e-9, atol=0, err_msg=name)
    return tr, model


def test_static_scratch_entry_point_matches_the_allocating_one_twice_in_a_row():
    _both(tg.config(2, 3000), 600, 8)        # 8 replays x 3,000 requests, bounded caches (evictions)
    _both(tg.config(1, 700), 0, 4)           # then a smaller input over the same scratch array


def test_static_scratch_entry_point_refuses_what_does_not_fit_and_a_trace_that_is_not_resident():
    wl = tg.config(2, 3000)
    tr = g.Trace.from_arrays(wl.trace.ts_ms, wl.trace.in_len, wl.trace.out_len, wl.trace.blk_off, wl.trace.hash_ids)
    model = g.Model(wl.R, wl.batch, 600, wl.prefill_ms_per_token, wl.decode_ms_per_token)
    import ctypes as C
    L = g.lib()
    m = model.c()
    P = 4
    par = np.ascontiguousarray(wl.params[:P], np.float64)
    sc = np.ascontiguousarray(wl.scale[:P], np.float64)
    rtt = np.ascontiguousarray(wl.rtt_ms, np.float64)
    import torch
    p95 = torch.empty((P,), dtype=torch.float64, device="cuda:0")
    o = binding._outputs_struct(p95_ttft_ms=p95)
    # not resident yet: no evaluation and no gorgo_trace_to_device has run on this handle
    rc = L.gorgo_eval_population_static(tr._h, C.byref(m), None, binding._ptr(rtt), binding._ptr(par), binding._ptr(sc), P,
                                        C.byref(o), None)
    assert rc == -1 and b"resident" in L.gorgo_last_error()
    assert L.gorgo_trace_to_device(tr._h) == 0
    big = 4096                                # far more replays than the static array holds
    parb = np.ascontiguousarray(np.tile(par, (big // P, 1)))
    scb = np.ascontiguousarray(np.tile(sc, big // P))
    p95b = torch.empty((big,), dtype=torch.float64, device="cuda:0")
    ob = binding._outputs_struct(p95_ttft_ms=p95b)
    assert g.workspace_bytes(tr, model, big) > binding.STATIC_SCRATCH_BYTES
    rc = L.gorgo_eval_population_static(tr._h, C.byref(m), None, binding._ptr(rtt), binding._ptr(parb), binding._ptr(scb), big,
                                        C.byref(ob), None)
    assert rc == -7 and b"static scratch" in L.gorgo_last_error()

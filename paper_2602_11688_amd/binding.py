"""ctypes binding of libgorgo.so: argument marshalling only -- every step of the evaluation runs in the
library's HIP kernels.  torch is used for device memory and streams, nothing else."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgorgo.so")
_lib = None


class GorgoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"gorgo error {code}: {msg}")
        self.code = code


class _Model(C.Structure):
    _fields_ = [("R", C.c_int32), ("batch", C.c_int32), ("block_tokens", C.c_int32), ("_pad", C.c_int32),
                ("cache_blocks", C.c_int64), ("prefill_ms_per_token", C.c_double),
                ("decode_ms_per_token", C.c_double)]


class _Outputs(C.Structure):
    _fields_ = [("route", C.c_void_p), ("hit_blocks", C.c_void_p), ("ttft_ms", C.c_void_p), ("e2e_ms", C.c_void_p),
                ("p95_ttft_ms", C.c_void_p), ("p95_e2e_ms", C.c_void_p)]


class _Online(C.Structure):
    _fields_ = [("window", C.c_int32), ("hop", C.c_int32), ("lo", C.c_double * 3), ("hi", C.c_double * 3),
                ("sigma0", C.c_double), ("z", C.c_void_p), ("theta_step", C.c_void_p), ("fitness_step", C.c_void_p),
                ("theta_final", C.c_void_p), ("sigma_final", C.c_void_p), ("accepted", C.c_void_p)]


class _Engine(C.Structure):
    _fields_ = [("prefill_ms_per_token", C.c_void_p), ("decode_ms_per_token", C.c_void_p), ("kv_tokens", C.c_void_p),
                ("decode_slowdown", C.c_double)]


class _Proxy(C.Structure):
    _fields_ = [("epochs", C.c_int32), ("probe_interval_ms", C.c_int32), ("rtt_true_ms", C.c_void_p),
                ("ewma_alpha", C.c_double), ("index_blocks", C.c_int64), ("rtt_tables", C.c_void_p),
                ("believed_hit_blocks", C.c_void_p)]


class Options(C.Structure):
    """gorgo_options: how an evaluation is carried out (no result depends on it), passed to the library with every
    call.  replay_path 0 automatic / 1 hashed block tables / 2 dense segment rows; replay_packing 0 never / 1 whenever
    the shape allows / 2 automatic; handover_poll_limit polls before a packed replay is given up;
    table_factor_percent 110..1600."""
    _fields_ = [("replay_path", C.c_int32), ("replay_packing", C.c_int32), ("handover_poll_limit", C.c_int32),
                ("table_factor_percent", C.c_int32)]


class EsState(C.Structure):
    _fields_ = [("theta", C.c_double * 3), ("sigma", C.c_double), ("lo", C.c_double * 3), ("hi", C.c_double * 3),
                ("seed", C.c_uint64), ("generation", C.c_int64), ("best_fitness", C.c_double),
                ("best_theta", C.c_double * 3)]


def lib():
    """Load the HIP library.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2602_11688_amd.build`")
        try:
            import torch  # noqa: F401  (loads the HIP runtime that the library shares with torch's allocator)
        except Exception:  # pragma: no cover
            pass
        L = C.CDLL(_LIB_PATH)
        vp, i32, i64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
        L.gorgo_last_error.restype = C.c_char_p
        L.gorgo_last_error.argtypes = []
        L.gorgo_load_trace.argtypes = [C.c_char_p, i32, C.POINTER(vp)]
        L.gorgo_load_trace_arrays.argtypes = [i64, vp, vp, vp, vp, vp, i32, C.POINTER(vp)]
        L.gorgo_trace_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32), C.POINTER(i64), C.POINTER(i32)]
        L.gorgo_free_trace.argtypes = [vp]
        L.gorgo_free_trace.restype = None
        L.gorgo_workspace_bytes.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), i32, C.POINTER(_Outputs), C.POINTER(C.c_size_t)]
        L.gorgo_eval_population.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), vp, vp, vp, i32, C.POINTER(_Outputs), vp,
                                            C.c_size_t, vp]
        L.gorgo_eval_population_sections.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), vp, vp, vp, i32, C.POINTER(_Outputs), vp,
                                                     C.c_size_t, vp, vp]
        L.gorgo_trace_to_device.argtypes = [vp]
        L.gorgo_eval_population_static.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), vp, vp, vp, i32, C.POINTER(_Outputs), vp]
        L.gorgo_online_steps.argtypes = [i64, i32, i32]
        L.gorgo_online_steps.restype = i64
        L.gorgo_eval_online.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), vp, vp, vp, i32, C.POINTER(_Online), C.POINTER(_Outputs),
                                        vp, C.c_size_t, vp]
        L.gorgo_eval_policy.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), vp, i32, vp, vp, i32, C.POINTER(_Outputs), vp, C.c_size_t, vp]
        L.gorgo_eval_engine.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), C.POINTER(_Engine), vp, i32, vp, vp, C.POINTER(_Online), vp,
                                        i32, C.POINTER(_Outputs), vp, C.c_size_t, vp]
        L.gorgo_eval_proxy.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), C.POINTER(_Proxy), C.POINTER(_Engine), vp, C.POINTER(_Online),
                                       vp, i32, C.POINTER(_Outputs), vp, C.c_size_t, vp]
        L.gorgo_es_init.argtypes = [C.POINTER(EsState), C.c_uint64]
        L.gorgo_es_sample.argtypes = [C.c_uint64, i64, i32, vp]
        L.gorgo_philox4x32_10.argtypes = [vp, vp, vp]
        L.gorgo_philox4x32_10.restype = None
        L.gorgo_es_propose.argtypes = [C.POINTER(EsState), vp, i32, vp]
        L.gorgo_es_update.argtypes = [vp, vp, i32, C.POINTER(EsState)]
        L.gorgo_es_workspace_bytes.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), i32, C.POINTER(C.c_size_t)]
        L.gorgo_es_step.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), vp, dbl, i32, C.POINTER(EsState), vp, vp, vp, C.c_size_t, vp]
        L.gorgo_query_replay_packing.argtypes = [vp, C.POINTER(_Model), C.POINTER(Options), i32, C.POINTER(i32)]
        L.gorgo_query_replay_path.argtypes = [vp, C.POINTER(Options), C.POINTER(i32), C.POINTER(i64), C.POINTER(i64)]
        L.gorgo_query_row_slots.argtypes = [vp, C.POINTER(i64)]
        L.gorgo_query_row_slots.restype = C.c_int
        L.gorgo_options_default.argtypes = [C.POINTER(Options)]
        L.gorgo_options_default.restype = None
        L.gorgo_last_eval_kernel_ms.argtypes = [C.POINTER(dbl)] * 3
        for name in ("gorgo_load_trace", "gorgo_load_trace_arrays", "gorgo_trace_info", "gorgo_workspace_bytes",
                     "gorgo_eval_population", "gorgo_eval_population_sections", "gorgo_trace_to_device", "gorgo_eval_population_static", "gorgo_eval_online", "gorgo_eval_policy", "gorgo_eval_engine", "gorgo_eval_proxy", "gorgo_es_init", "gorgo_es_sample", "gorgo_es_propose",
                     "gorgo_es_update", "gorgo_es_workspace_bytes", "gorgo_es_step",
                     "gorgo_last_eval_kernel_ms", "gorgo_query_replay_packing", "gorgo_query_replay_path"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise GorgoError(rc, lib().gorgo_last_error().decode())


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class Model:
    R: int
    batch: int
    cache_blocks: int
    prefill_ms_per_token: float
    decode_ms_per_token: float
    block_tokens: int = 512

    def c(self) -> _Model:
        return _Model(self.R, self.batch, self.block_tokens, 0, self.cache_blocks, self.prefill_ms_per_token,
                      self.decode_ms_per_token)


class Trace:
    """Handle of a loaded trace (gorgo_load_trace / gorgo_load_trace_arrays)."""

    def __init__(self, handle):
        self._h = handle

    @classmethod
    def from_jsonl(cls, path: str, block_tokens: int = 512) -> "Trace":
        h = C.c_void_p()
        _check(lib().gorgo_load_trace(os.fsencode(path), block_tokens, C.byref(h)))
        return cls(h)

    @classmethod
    def from_arrays(cls, ts_ms, in_len, out_len, blk_off, hash_ids, block_tokens: int = 512) -> "Trace":
        ts, il, ol = _np(ts_ms, np.int64), _np(in_len, np.int32), _np(out_len, np.int32)
        bo, hi = _np(blk_off, np.int64), _np(hash_ids, np.int64)
        if not (ts.shape == il.shape == ol.shape) or bo.shape != (ts.shape[0] + 1,) or (
                bo.shape[0] and hi.shape[0] < bo[-1]):
            raise ValueError("inconsistent trace array shapes")
        h = C.c_void_p()
        _check(lib().gorgo_load_trace_arrays(ts.shape[0], _ptr(ts), _ptr(il), _ptr(ol), _ptr(bo), _ptr(hi),
                                             block_tokens, C.byref(h)))
        return cls(h)

    def info(self) -> dict:
        n, tb, u = C.c_int64(), C.c_int64(), C.c_int64()
        mb, cc = C.c_int32(), C.c_int32()
        _check(lib().gorgo_trace_info(self._h, C.byref(n), C.byref(tb), C.byref(mb), C.byref(u), C.byref(cc)))
        return dict(N=n.value, total_blocks=tb.value, max_blocks=mb.value, unique_ids=u.value,
                    chain_consistent=bool(cc.value))

    def replay_path(self, options: Optional["Options"] = None) -> dict:
        """Formulation an evaluation would use under the options (1 = block tables, 2 = segment rows) and segment counts."""
        p, ns, nr = C.c_int32(), C.c_int64(), C.c_int64()
        _check(lib().gorgo_query_replay_path(self._h, _opt(options), C.byref(p), C.byref(ns), C.byref(nr)))
        return dict(path=p.value, n_segments=ns.value, segment_refs=nr.value)

    def row_slots(self) -> int:
        """Rows of cells a replay keeps in the segment formulation: the most segments in use at one time."""
        n = C.c_int64()
        _check(lib().gorgo_query_row_slots(self._h, C.byref(n)))
        return n.value

    @property
    def N(self) -> int:
        return self.info()["N"]

    def close(self):
        if self._h:
            lib().gorgo_free_trace(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# The library keeps no settings: every call carries its options.  For callers that want one choice for a whole
# script (tests, the benchmark), this module keeps a default Options object of its own, passed wherever a call
# gives none; the set_* functions below change it.
_default_options = None


def default_options() -> Options:
    """The Options passed when a call gives none (initially the library's defaults)."""
    global _default_options
    if _default_options is None:
        o = Options()
        lib().gorgo_options_default(C.byref(o))
        _default_options = o
    return _default_options


def _opt(options: Optional[Options]):
    return C.byref(options if options is not None else default_options())


def _set_default(field: str, value: int, lo: int, hi: int, what: str):
    if not lo <= int(value) <= hi:
        raise GorgoError(-1, f"{what} must be in {lo}..{hi}")
    setattr(default_options(), field, int(value))


def set_table_factor_percent(pct: int):
    _set_default("table_factor_percent", pct, 110, 1600, "table_factor_percent")


def set_replay_packing(mode: int) -> None:
    """Two replays per wavefront pair: 0 never, 1 whenever the shape allows it, 2 (default) when the replays would not
    all be resident at once otherwise; results do not depend on it."""
    _set_default("replay_packing", mode, 0, 2, "replay_packing")


def replay_packing(trace: "Trace", model: "Model", P: int, options: Optional[Options] = None) -> bool:
    """Whether eval_population with P replays would run two replays per wavefront pair under the options."""
    out = C.c_int32()
    m = model.c()
    _check(lib().gorgo_query_replay_packing(trace._h, C.byref(m), _opt(options), P, C.byref(out)))
    return bool(out.value)


def set_handover_poll_limit(polls: int):
    """Polls of a hand-over word before a packed replay is given up (default 2^24); for tests of that path."""
    _set_default("handover_poll_limit", polls, 0, 2**31 - 1, "handover_poll_limit")


def set_replay_path(mode: int):
    """0 = automatic, 1 = hashed block tables, 2 = dense segment rows."""
    _set_default("replay_path", mode, 0, 2, "replay_path")


def last_eval_kernel_ms() -> dict:
    """Device milliseconds of the stages of this thread's most recent evaluation (waits for it)."""
    a, b, c = C.c_double(), C.c_double(), C.c_double()
    _check(lib().gorgo_last_eval_kernel_ms(C.byref(a), C.byref(b), C.byref(c)))
    return dict(fill_ms=a.value, replay_ms=b.value, select_ms=c.value)


def _outputs_struct(route=None, hit_blocks=None, ttft_ms=None, e2e_ms=None, p95_ttft_ms=None, p95_e2e_ms=None):
    def dp(x):
        return None if x is None else C.c_void_p(x.data_ptr())
    return _Outputs(dp(route), dp(hit_blocks), dp(ttft_ms), dp(e2e_ms), dp(p95_ttft_ms), dp(p95_e2e_ms))


def workspace_bytes(trace: Trace, model: Model, P: int, outputs: Optional[_Outputs] = None, options: Optional[Options] = None) -> int:
    n = C.c_size_t()
    m = model.c()
    _check(lib().gorgo_workspace_bytes(trace._h, C.byref(m), _opt(options), P, None if outputs is None else C.byref(outputs),
                                       C.byref(n)))
    return n.value


@dataclass
class EvalResult:
    route: object = None
    hit_blocks: object = None
    ttft_ms: object = None
    e2e_ms: object = None
    p95_ttft_ms: object = None
    p95_e2e_ms: object = None
    workspace: object = None
    sections: object = None         # [P, 3, 12] int64 cycles per section (eval_population(sections=True) only)
    # online tuner (eval_online only)
    theta_step: object = None       # [P, steps, 3] weights in use after each step
    fitness_step: object = None     # [P, steps] window p95 TTFT seen at each step
    theta_final: object = None      # [P, 3]
    sigma_final: object = None      # [P]
    accepted: object = None         # [P] int32
    _z: object = None
    # imperfect proxy knowledge (eval_proxy only)
    rtt_est_ms: object = None           # [epochs, R] the proxy's smoothed round trip times
    believed_hit_blocks: object = None  # [P, N] uint16 blocks Eq. 3 took for cached on the chosen replica
    _tables: object = None


def eval_population(trace: Trace, model: Model, rtt_ms, params, scale, *, per_request: bool = True,
                    p95: bool = True, workspace=None, stream=None, device="cuda:0", sections: bool = False, options: Optional[Options] = None) -> EvalResult:
    """gorgo_eval_population with torch-allocated outputs.  Returns device tensors; asynchronous on `stream`
    (default: torch's current stream).  sections=True runs gorgo_eval_population_sections instead and adds
    `sections` [P, 3, 12] (cycles per section of the request loop: cache, queue and front-end wavefront) to the result."""
    import torch
    rtt = _np(rtt_ms, np.float64)
    par = _np(params, np.float64)
    P = par.shape[0]
    sc = _np(np.broadcast_to(np.asarray(scale, dtype=np.float64), (P,)), np.float64)
    if par.shape != (P, 3) or rtt.shape != (model.R,):
        raise ValueError("params must be [P,3] and rtt_ms [R]")
    N = trace.N
    dev = torch.device(device)
    res = EvalResult()
    if per_request:
        res.route = torch.empty((P, N), dtype=torch.uint8, device=dev)
        res.hit_blocks = torch.empty((P, N), dtype=torch.uint16, device=dev)
        res.ttft_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
        res.e2e_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
    if p95:
        res.p95_ttft_ms = torch.empty((P,), dtype=torch.float64, device=dev)
        res.p95_e2e_ms = torch.empty((P,), dtype=torch.float64, device=dev)
    o = _outputs_struct(res.route, res.hit_blocks, res.ttft_ms, res.e2e_ms, res.p95_ttft_ms, res.p95_e2e_ms)
    need = workspace_bytes(trace, model, P, o, options)
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
    res.workspace = workspace
    s = stream if stream is not None else torch.cuda.current_stream(dev)
    m = model.c()
    with torch.cuda.device(dev):
        if sections:
            res.sections = torch.zeros((P, 3, 12), dtype=torch.int64, device=dev)
            _check(lib().gorgo_eval_population_sections(trace._h, C.byref(m), _opt(options), _ptr(rtt), _ptr(par), _ptr(sc), P, C.byref(o),
                                                        C.c_void_p(workspace.data_ptr()), workspace.numel(),
                                                        C.c_void_p(s.cuda_stream), C.c_void_p(res.sections.data_ptr())))
        else:
            _check(lib().gorgo_eval_population(trace._h, C.byref(m), _opt(options), _ptr(rtt), _ptr(par), _ptr(sc), P, C.byref(o),
                                               C.c_void_p(workspace.data_ptr()), workspace.numel(),
                                               C.c_void_p(s.cuda_stream)))
    return res


STATIC_SCRATCH_BYTES = 64 << 20


def eval_population_static(trace: Trace, model: Model, rtt_ms, params, scale, *, per_request: bool = True,
                           p95: bool = True, stream=None, device="cuda:0", options: Optional[Options] = None) -> EvalResult:
    """gorgo_eval_population_static: as eval_population, with the library's static scratch array as the workspace
    (nothing is allocated by the library; the outputs are still torch tensors allocated here)."""
    import torch
    rtt = _np(rtt_ms, np.float64)
    par = _np(params, np.float64)
    P = par.shape[0]
    sc = _np(np.broadcast_to(np.asarray(scale, dtype=np.float64), (P,)), np.float64)
    if par.shape != (P, 3) or rtt.shape != (model.R,):
        raise ValueError("params must be [P,3] and rtt_ms [R]")
    N = trace.N
    dev = torch.device(device)
    res = EvalResult()
    if per_request:
        res.route = torch.empty((P, N), dtype=torch.uint8, device=dev)
        res.hit_blocks = torch.empty((P, N), dtype=torch.uint16, device=dev)
        res.ttft_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
        res.e2e_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
    if p95:
        res.p95_ttft_ms = torch.empty((P,), dtype=torch.float64, device=dev)
        res.p95_e2e_ms = torch.empty((P,), dtype=torch.float64, device=dev)
    o = _outputs_struct(res.route, res.hit_blocks, res.ttft_ms, res.e2e_ms, res.p95_ttft_ms, res.p95_e2e_ms)
    s = stream if stream is not None else torch.cuda.current_stream(dev)
    m = model.c()
    with torch.cuda.device(dev):
        _check(lib().gorgo_trace_to_device(trace._h))
        _check(lib().gorgo_eval_population_static(trace._h, C.byref(m), _opt(options), _ptr(rtt), _ptr(par), _ptr(sc), P, C.byref(o),
                                                  C.c_void_p(s.cuda_stream)))
    return res


POLICIES = {"least-request": 1, "session-affinity": 2, "random": 3}


def eval_policy(trace: Trace, model: Model, rtt_ms, policy: str, scale, *, seeds=None, per_request: bool = True,
                p95: bool = True, workspace=None, stream=None, device="cuda:0", options: Optional[Options] = None) -> EvalResult:
    """gorgo_eval_policy with torch-allocated outputs: one replay per entry of `scale`, routed by a baseline policy
    ("least-request", "session-affinity", "random"; prefix-cache and least-load are eval_population with weights
    (0,1,0) and (0,0,1)).  seeds [P] for the random policy."""
    import torch
    rtt = _np(rtt_ms, np.float64)
    sc = _np(np.atleast_1d(np.asarray(scale, dtype=np.float64)), np.float64)
    P = sc.shape[0]
    sd = None if seeds is None else _np(seeds, np.uint64)
    if rtt.shape != (model.R,) or (sd is not None and sd.shape != (P,)):
        raise ValueError("rtt_ms must be [R] and seeds [P]")
    N = trace.N
    dev = torch.device(device)
    res = EvalResult()
    if per_request:
        res.route = torch.empty((P, N), dtype=torch.uint8, device=dev)
        res.hit_blocks = torch.empty((P, N), dtype=torch.uint16, device=dev)
        res.ttft_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
        res.e2e_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
    if p95:
        res.p95_ttft_ms = torch.empty((P,), dtype=torch.float64, device=dev)
        res.p95_e2e_ms = torch.empty((P,), dtype=torch.float64, device=dev)
    o = _outputs_struct(res.route, res.hit_blocks, res.ttft_ms, res.e2e_ms, res.p95_ttft_ms, res.p95_e2e_ms)
    need = workspace_bytes(trace, model, P, o, options)
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
    res.workspace = workspace
    s = stream if stream is not None else torch.cuda.current_stream(dev)
    m = model.c()
    with torch.cuda.device(dev):
        _check(lib().gorgo_eval_policy(trace._h, C.byref(m), _opt(options), _ptr(rtt), POLICIES[policy], _ptr(sd), _ptr(sc), P, C.byref(o),
                                       C.c_void_p(workspace.data_ptr()), workspace.numel(), C.c_void_p(s.cuda_stream)))
    return res


def online_steps(N: int, window: int = 128, hop: int = 32) -> int:
    n = lib().gorgo_online_steps(N, window, hop)
    if n < 0:
        raise ValueError("window and hop must be >= 1")
    return n


def eval_online(trace: Trace, model: Model, rtt_ms, theta0, z, scale, *, lo, hi, sigma0, window: int = 128,
                hop: int = 32, per_request: bool = True, p95: bool = True, trajectory: bool = True, workspace=None,
                stream=None, device="cuda:0", options: Optional[Options] = None) -> EvalResult:
    """gorgo_eval_online with torch-allocated outputs: P replays, each tuning its weights online.  theta0 [P,3];
    z [P, steps, 3] standard normal draws (host array or device tensor)."""
    import torch
    rtt = _np(rtt_ms, np.float64)
    th0 = _np(theta0, np.float64)
    P = th0.shape[0]
    sc = _np(np.broadcast_to(np.asarray(scale, dtype=np.float64), (P,)), np.float64)
    if th0.shape != (P, 3) or rtt.shape != (model.R,):
        raise ValueError("theta0 must be [P,3] and rtt_ms [R]")
    N = trace.N
    steps = online_steps(N, window, hop)
    dev = torch.device(device)
    zt = z if isinstance(z, torch.Tensor) else torch.from_numpy(_np(z, np.float64))
    zt = zt.to(device=dev, dtype=torch.float64).contiguous()
    if tuple(zt.shape) != (P, steps, 3):
        raise ValueError(f"z must be [P, {steps}, 3]")
    res = EvalResult()
    if per_request:
        res.route = torch.empty((P, N), dtype=torch.uint8, device=dev)
        res.hit_blocks = torch.empty((P, N), dtype=torch.uint16, device=dev)
        res.ttft_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
        res.e2e_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
    if p95:
        res.p95_ttft_ms = torch.empty((P,), dtype=torch.float64, device=dev)
        res.p95_e2e_ms = torch.empty((P,), dtype=torch.float64, device=dev)
    if trajectory:
        res.theta_step = torch.empty((P, steps, 3), dtype=torch.float64, device=dev)
        res.fitness_step = torch.empty((P, steps), dtype=torch.float64, device=dev)
    res.theta_final = torch.empty((P, 3), dtype=torch.float64, device=dev)
    res.sigma_final = torch.empty((P,), dtype=torch.float64, device=dev)
    res.accepted = torch.empty((P,), dtype=torch.int32, device=dev)
    o = _outputs_struct(res.route, res.hit_blocks, res.ttft_ms, res.e2e_ms, res.p95_ttft_ms, res.p95_e2e_ms)

    def dp(x):
        return None if x is None else C.c_void_p(x.data_ptr())
    on = _Online(window, hop, (C.c_double * 3)(*[float(x) for x in lo]), (C.c_double * 3)(*[float(x) for x in hi]),
                 float(sigma0), dp(zt), dp(res.theta_step), dp(res.fitness_step), dp(res.theta_final),
                 dp(res.sigma_final), dp(res.accepted))
    need = workspace_bytes(trace, model, P, o, options)
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
    res.workspace = workspace
    s = stream if stream is not None else torch.cuda.current_stream(dev)
    m = model.c()
    with torch.cuda.device(dev):
        _check(lib().gorgo_eval_online(trace._h, C.byref(m), _opt(options), _ptr(rtt), _ptr(th0), _ptr(sc), P, C.byref(on), C.byref(o),
                                       C.c_void_p(workspace.data_ptr()), workspace.numel(), C.c_void_p(s.cuda_stream)))
    res._z = zt          # keep the draws alive until the stream has consumed them
    return res


@dataclass
class Engine:
    """Engine model of a replica (gorgo_engine): per-replica rates, KV budgets in tokens (None = no budget) and
    the decode slow-down per co-running request."""
    prefill_ms_per_token: Sequence[float]
    decode_ms_per_token: Sequence[float]
    kv_tokens: Optional[Sequence[int]] = None
    decode_slowdown: float = 0.0


def eval_engine(trace: Trace, model: Model, engine: Engine, rtt_ms, scale, *, params=None, policy: str = "cost-model",
                seeds=None, online: Optional[dict] = None, per_request: bool = True, p95: bool = True,
                workspace=None, stream=None, device="cuda:0", options: Optional[Options] = None) -> EvalResult:
    """gorgo_eval_engine with torch-allocated outputs.  policy "cost-model" routes by Eq. 3 with weights params
    [P,3] (and, with online = dict(z=[P,steps,3], lo=, hi=, sigma0=, window=, hop=), tunes them online); the
    baseline policies route as in eval_policy, one replay per entry of `scale`."""
    import torch
    rtt = _np(rtt_ms, np.float64)
    cost_model = policy == "cost-model"
    if cost_model:
        par = _np(params, np.float64)
        P = par.shape[0]
        if par.shape != (P, 3):
            raise ValueError("params must be [P,3]")
        sc = _np(np.broadcast_to(np.asarray(scale, dtype=np.float64), (P,)), np.float64)
    else:
        par = None
        sc = _np(np.atleast_1d(np.asarray(scale, dtype=np.float64)), np.float64)
        P = sc.shape[0]
    sd = None if seeds is None else _np(seeds, np.uint64)
    a_pf = _np(engine.prefill_ms_per_token, np.float64)
    a_dec = _np(engine.decode_ms_per_token, np.float64)
    kv = None if engine.kv_tokens is None else _np(engine.kv_tokens, np.int64)
    if rtt.shape != (model.R,) or a_pf.shape != (model.R,) or a_dec.shape != (model.R,) or \
            (kv is not None and kv.shape != (model.R,)) or (sd is not None and sd.shape != (P,)):
        raise ValueError("rtt_ms, the engine's rates and budgets must be [R], seeds [P]")
    eng = _Engine(_ptr(a_pf), _ptr(a_dec), _ptr(kv), float(engine.decode_slowdown))
    N = trace.N
    dev = torch.device(device)
    res = EvalResult()
    if per_request:
        res.route = torch.empty((P, N), dtype=torch.uint8, device=dev)
        res.hit_blocks = torch.empty((P, N), dtype=torch.uint16, device=dev)
        res.ttft_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
        res.e2e_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
    if p95:
        res.p95_ttft_ms = torch.empty((P,), dtype=torch.float64, device=dev)
        res.p95_e2e_ms = torch.empty((P,), dtype=torch.float64, device=dev)
    on = None
    if online is not None:
        window, hop = int(online.get("window", 128)), int(online.get("hop", 32))
        steps = online_steps(N, window, hop)
        z = online["z"]
        zt = z if isinstance(z, torch.Tensor) else torch.from_numpy(_np(z, np.float64))
        zt = zt.to(device=dev, dtype=torch.float64).contiguous()
        if tuple(zt.shape) != (P, steps, 3):
            raise ValueError(f"z must be [P, {steps}, 3]")
        res.theta_step = torch.empty((P, steps, 3), dtype=torch.float64, device=dev)
        res.fitness_step = torch.empty((P, steps), dtype=torch.float64, device=dev)
        res.theta_final = torch.empty((P, 3), dtype=torch.float64, device=dev)
        res.sigma_final = torch.empty((P,), dtype=torch.float64, device=dev)
        res.accepted = torch.empty((P,), dtype=torch.int32, device=dev)
        res._z = zt
        on = _Online(window, hop, (C.c_double * 3)(*[float(x) for x in online["lo"]]),
                     (C.c_double * 3)(*[float(x) for x in online["hi"]]), float(online["sigma0"]),
                     C.c_void_p(zt.data_ptr()), C.c_void_p(res.theta_step.data_ptr()),
                     C.c_void_p(res.fitness_step.data_ptr()), C.c_void_p(res.theta_final.data_ptr()),
                     C.c_void_p(res.sigma_final.data_ptr()), C.c_void_p(res.accepted.data_ptr()))
    o = _outputs_struct(res.route, res.hit_blocks, res.ttft_ms, res.e2e_ms, res.p95_ttft_ms, res.p95_e2e_ms)
    need = workspace_bytes(trace, model, P, o, options)
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
    res.workspace = workspace
    s = stream if stream is not None else torch.cuda.current_stream(dev)
    m = model.c()
    code = 0 if cost_model else POLICIES[policy]
    with torch.cuda.device(dev):
        _check(lib().gorgo_eval_engine(trace._h, C.byref(m), _opt(options), C.byref(eng), _ptr(rtt), code, _ptr(par), _ptr(sd),
                                       None if on is None else C.byref(on), _ptr(sc), P, C.byref(o),
                                       C.c_void_p(workspace.data_ptr()), workspace.numel(), C.c_void_p(s.cuda_stream)))
    return res


@dataclass
class Proxy:
    """Imperfect proxy knowledge (gorgo_proxy): true round trip times per probe epoch [epochs, R], the probe
    interval, the smoothing constant of the proxy's moving average, and the capacity of its own cache index in blocks
    per replica (0 = it never forgets, -1 = it sees the replicas' caches as they are)."""
    rtt_true_ms: Sequence[Sequence[float]]
    probe_interval_ms: int = 30000
    ewma_alpha: float = 0.5
    index_blocks: int = -1


def eval_proxy(trace: Trace, model: Model, proxy: Proxy, params, scale, *, engine: Optional[Engine] = None,
               online: Optional[dict] = None, per_request: bool = True, p95: bool = True, workspace=None, stream=None,
               device="cuda:0", options: Optional[Options] = None) -> EvalResult:
    """gorgo_eval_proxy with torch-allocated outputs: P replays under weights params [P,3] (tuned online when
    online = dict(z=, lo=, hi=, sigma0=, window=, hop=) is given) with imperfect proxy knowledge; replicas follow the
    engine model when `engine` is given, else the linear one."""
    import torch
    par = _np(params, np.float64)
    P = par.shape[0]
    if par.shape != (P, 3):
        raise ValueError("params must be [P,3]")
    sc = _np(np.broadcast_to(np.asarray(scale, dtype=np.float64), (P,)), np.float64)
    rt = _np(proxy.rtt_true_ms, np.float64)
    if rt.ndim != 2 or rt.shape[1] != model.R or rt.shape[0] < 1:
        raise ValueError("rtt_true_ms must be [epochs, R]")
    E = rt.shape[0]
    N = trace.N
    dev = torch.device(device)
    res = EvalResult()
    if per_request:
        res.route = torch.empty((P, N), dtype=torch.uint8, device=dev)
        res.hit_blocks = torch.empty((P, N), dtype=torch.uint16, device=dev)
        res.believed_hit_blocks = torch.empty((P, N), dtype=torch.uint16, device=dev)
        res.ttft_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
        res.e2e_ms = torch.empty((P, N), dtype=torch.float64, device=dev)
    if p95:
        res.p95_ttft_ms = torch.empty((P,), dtype=torch.float64, device=dev)
        res.p95_e2e_ms = torch.empty((P,), dtype=torch.float64, device=dev)
    tables = torch.empty((2, E, model.R), dtype=torch.float64, device=dev)
    res.rtt_est_ms = tables[1]
    px = _Proxy(E, int(proxy.probe_interval_ms), _ptr(rt), float(proxy.ewma_alpha), int(proxy.index_blocks),
                C.c_void_p(tables.data_ptr()),
                None if res.believed_hit_blocks is None else C.c_void_p(res.believed_hit_blocks.data_ptr()))
    eng = None
    if engine is not None:
        a_pf = _np(engine.prefill_ms_per_token, np.float64)
        a_dec = _np(engine.decode_ms_per_token, np.float64)
        kv = None if engine.kv_tokens is None else _np(engine.kv_tokens, np.int64)
        if a_pf.shape != (model.R,) or a_dec.shape != (model.R,) or (kv is not None and kv.shape != (model.R,)):
            raise ValueError("the engine's rates and budgets must be [R]")
        eng = _Engine(_ptr(a_pf), _ptr(a_dec), _ptr(kv), float(engine.decode_slowdown))
    on = None
    if online is not None:
        window, hop = int(online.get("window", 128)), int(online.get("hop", 32))
        steps = online_steps(N, window, hop)
        z = online["z"]
        zt = z if isinstance(z, torch.Tensor) else torch.from_numpy(_np(z, np.float64))
        zt = zt.to(device=dev, dtype=torch.float64).contiguous()
        if tuple(zt.shape) != (P, steps, 3):
            raise ValueError(f"z must be [P, {steps}, 3]")
        res.theta_step = torch.empty((P, steps, 3), dtype=torch.float64, device=dev)
        res.fitness_step = torch.empty((P, steps), dtype=torch.float64, device=dev)
        res.theta_final = torch.empty((P, 3), dtype=torch.float64, device=dev)
        res.sigma_final = torch.empty((P,), dtype=torch.float64, device=dev)
        res.accepted = torch.empty((P,), dtype=torch.int32, device=dev)
        res._z = zt
        on = _Online(window, hop, (C.c_double * 3)(*[float(x) for x in online["lo"]]),
                     (C.c_double * 3)(*[float(x) for x in online["hi"]]), float(online["sigma0"]),
                     C.c_void_p(zt.data_ptr()), C.c_void_p(res.theta_step.data_ptr()),
                     C.c_void_p(res.fitness_step.data_ptr()), C.c_void_p(res.theta_final.data_ptr()),
                     C.c_void_p(res.sigma_final.data_ptr()), C.c_void_p(res.accepted.data_ptr()))
    o = _outputs_struct(res.route, res.hit_blocks, res.ttft_ms, res.e2e_ms, res.p95_ttft_ms, res.p95_e2e_ms)
    need = workspace_bytes(trace, model, P, o, options)
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
    res.workspace = workspace
    s = stream if stream is not None else torch.cuda.current_stream(dev)
    m = model.c()
    with torch.cuda.device(dev):
        _check(lib().gorgo_eval_proxy(trace._h, C.byref(m), _opt(options), C.byref(px), None if eng is None else C.byref(eng), _ptr(par),
                                      None if on is None else C.byref(on), _ptr(sc), P, C.byref(o),
                                      C.c_void_p(workspace.data_ptr()), workspace.numel(), C.c_void_p(s.cuda_stream)))
    res._tables = tables
    return res


# ------------------------------------------------------------------------------------------------ tuner

def es_init(seed: int) -> EsState:
    s = EsState()
    _check(lib().gorgo_es_init(C.byref(s), seed))
    return s


def philox4x32_10(ctr, key) -> np.ndarray:
    c, k = _np(ctr, np.uint32), _np(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().gorgo_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def es_sample(seed: int, generation: int, P: int) -> np.ndarray:
    z = np.zeros((P, 3), np.float64)
    _check(lib().gorgo_es_sample(seed, generation, P, _ptr(z)))
    return z


def es_propose(state: EsState, z) -> np.ndarray:
    z = _np(z, np.float64)
    out = np.zeros_like(z)
    _check(lib().gorgo_es_propose(C.byref(state), _ptr(z), z.shape[0], _ptr(out)))
    return out


def es_update(state: EsState, params, fitness) -> EsState:
    par, fit = _np(params, np.float64), _np(fitness, np.float64)
    _check(lib().gorgo_es_update(_ptr(par), _ptr(fit), par.shape[0], C.byref(state)))
    return state


def es_workspace_bytes(trace: Trace, model: Model, P: int, options: Optional[Options] = None) -> int:
    n = C.c_size_t()
    m = model.c()
    _check(lib().gorgo_es_workspace_bytes(trace._h, C.byref(m), _opt(options), P, C.byref(n)))
    return n.value


def es_step(trace: Trace, model: Model, rtt_ms, scale: float, P: int, state: EsState, *, workspace=None,
            stream=None, device="cuda:0", options: Optional[Options] = None):
    """gorgo_es_step.  Returns (params[P,3], fitness[P], workspace); `state` is updated in place."""
    import torch
    rtt = _np(rtt_ms, np.float64)
    dev = torch.device(device)
    need = es_workspace_bytes(trace, model, P, options)
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
    par = np.zeros((P, 3), np.float64)
    fit = np.zeros(P, np.float64)
    s = stream if stream is not None else torch.cuda.current_stream(dev)
    m = model.c()
    with torch.cuda.device(dev):
        _check(lib().gorgo_es_step(trace._h, C.byref(m), _opt(options), _ptr(rtt), float(scale), P, C.byref(state), _ptr(par),
                                   _ptr(fit), C.c_void_p(workspace.data_ptr()), workspace.numel(),
                                   C.c_void_p(s.cuda_stream)))
    return par, fit, workspace

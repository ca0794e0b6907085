"""MI355X-native batched routing-fitness evaluation (replay of a request trace under a population of
cost-model weight vectors).  The compute lives in libgorgo.so (hand-written HIP for gfx950); this package
is the thin ctypes binding."""
from .binding import (Engine, GorgoError, Model, Options, Proxy, Trace, default_options, es_init, es_propose, es_sample, es_step, es_update,  # noqa: F401
                      es_workspace_bytes, eval_engine, eval_online, eval_proxy, eval_policy, eval_population, eval_population_static, last_eval_kernel_ms, lib, online_steps,
                      philox4x32_10, replay_packing, set_handover_poll_limit, set_replay_packing, set_replay_path, set_table_factor_percent, workspace_bytes)

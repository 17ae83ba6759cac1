"""MI355X-native batched evaluation of the DiSCo dispatch and migration
policies (arXiv 2502.11417).  The work is done by ``libdisco.so`` (HIP,
gfx950); this package is its ctypes binding."""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    ACC, DevicePolicies, MIG_BUFFER, MIG_LAG, MIG_NONE, MODE_D, MODE_S, MODE_STOCH_D, MODE_STOCH_S, PARAM_BETA, PARAM_L_TH, PARAM_W_TAIL, DiscoError, Policy, Trace,
    accum_to_host, disco_average_runs, disco_budget_search, disco_solve_policy, solve_to_host,
    disco_device_profile, disco_fit_lognormal, disco_ingest_trace, fit_to_host, disco_eval_dispatch, disco_eval_dispatch_static, disco_eval_migration, disco_gen_trace,
    disco_reduce_stats, disco_policy_type, disco_read_probe, disco_validate_trace, disco_time_token_walk, disco_workspace_bytes, policies_to_host, search_to_host, stats_to_host,
    prepare_policies, prepare_specs, upload_trace, workspace,
)

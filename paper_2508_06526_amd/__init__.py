"""MI355X (gfx950) implementation of PiKV's routed sharded-KV decode path.

The work is done by hand-written HIP kernels in ``libpikv.so`` behind the C ABI declared
in ``include/pikv.h``; this package is the thin ctypes binding (argument marshalling only).
There is no CPU or eager fallback: if the library is missing, calls raise.
"""
from .binding import (  # noqa: F401
    COMBINE_LOCAL, COMBINE_LSE, PENALTY_CACHE_AWARE, PENALTY_LOAD_BALANCE, PENALTY_ENTROPY, DESC_VALUE_BIAS, PikvRouterFeedback,
    make_router_feedback, POLICY_H2O, POLICY_LRU,
    POLICY_LRU_PLUS, POLICY_SL, PikvDesc, PikvError, PikvPolicyArgs, make_policy_args, pikv_decode_step_policy, library_path, load_library, make_desc,
    pikv_append, pikv_attn_workspace_bytes, pikv_compress, pikv_router_penalty, pikv_decode_step, pikv_evict, pikv_route, pikv_route_round_robin, pikv_sharded_attn, pikv_sharded_attn_noalloc, NOALLOC_SCRATCH_BYTES,
    pikv_policy_compact, pikv_policy_stamp, pikv_policy_utility, pikv_set_attn_split, pikv_set_profile_events, pikv_strerror,
    pikv_stream_read_probe, pikv_update_utility, pikv_update_utility_tracked, pikv_version, shard_table)

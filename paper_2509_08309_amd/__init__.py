"""MI355X-native head-subset decode Attention over a block-paged KV cache.

The product is the HIP library built from csrc/ (C ABI in include/hetis_attn.h and
include/hetis_kv.h);
`binding` exposes it under the same names, `workloads` draws seeded inputs.
Importing this package loads nothing; the library is loaded on first call and
its absence is an error, never a fallback.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    HetisError, check, hetis_attn_decode, hetis_attn_decode_pairs, hetis_attn_decode_split,
    hetis_attn_decode_static, hetis_attn_decode_step, hetis_attn_decode_step_ws, hetis_attn_decode_ws, hetis_attn_decode_pairs_ws, hetis_attn_decode_pairs_step, hetis_attn_decode_pairs_step_ws, hetis_attn_decode_split_ws,
    hetis_attn_decode_workspace_bytes, hetis_attn_decode_pairs_workspace_bytes,
    hetis_attn_workspace_init, hetis_attn_workspace_status, hetis_attn_reserve_workspace,
    hetis_attn_validate_pairs, hetis_attn_merge, hetis_attn_profile_events,
    hetis_attn_release_workspace, hetis_attn_shape, hetis_attn_split_num_chunks,
    hetis_attn_split_workspace_bytes, hetis_attn_status_string, hetis_attn_validate,
    hetis_attn_version, hetis_dispatch_device, hetis_dispatch_solve, hetis_kv_append, hetis_kv_append_pairs, hetis_kv_copy_tiles, hetis_kv_fetch, hetis_kv_pool,
    hetis_kv_profile_events, hetis_kv_store, hetis_profiler_fit, hetis_profiler_fit_nonneg, hetis_profiler_predict, make_pool,
    make_shape,
)

"""MI355X (gfx950) KVSlimmer KV-cache merge step: HIP kernels behind a C ABI, plus a thin binding.

    from paper_2603_00907_amd import Problem, kvs_step, kvs_workspace_size

The compute lives in libkvs.so (csrc/*.hip, declared in include/kvs.h).  Build it with
`python -m paper_2603_00907_amd.build`.
"""

from .binding import (  # noqa: F401
    EXPORTS,
    KVS_BF16,
    KVS_ERR_ALIAS,
    KVS_ERR_BUDGET,
    KVS_ERR_DEVICE,
    KVS_ERR_DTYPE,
    KVS_ERR_INVALID_ARG,
    KVS_ERR_WORKSPACE,
    KVS_F32,
    KVS_OK,
    KvsError,
    Problem,
    kvs_decode_attention,
    kvs_decode_workspace_size,
    kvs_merge_compact,
    kvs_merge_compact_counts,
    kvs_merge_compact_norms,
    kvs_merge_compact_norms_counts,
    kvs_per_query_workspace_size,
    kvs_score,
    kvs_score_counts,
    kvs_select,
    kvs_sensitivity,
    kvs_sensitivity_counts,
    kvs_step,
    kvs_step_counts,
    kvs_step_per_query,
    kvs_step_per_query_counts,
    kvs_step_static,
    kvs_debug_set,
    kvs_debug_get,
    DEBUG_SWITCHES,
    STATIC_SCRATCH_BYTES,
    kvs_version,
    kvs_workspace_size,
    load_library,
    status_str,
)

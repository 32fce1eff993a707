"""MI355X-native fork-tree paged-KV decode attention (APAR hot path).

Thin ctypes binding over libapar.so (see include/apar.h): argument marshalling
only - every step of the path runs in the library's HIP kernels.  There is no
CPU fallback: importing the binding without a built library raises.
"""
from .binding import (  # noqa: F401
    APAR_BF16,
    APAR_F32,
    AparError,
    AparPlanInfo,
    AparPoolConfig,
    AparProfile,
    AparStats,
    Pool,
    apar_append_kv,
    apar_append_kv_batch,
    apar_block_refcount,
    apar_decode_attention,
    apar_decode_attention_spec,
    apar_fork,
    apar_free_thread,
    apar_last_plan_export,
    apar_last_plan_info,
    APAR_PLAN_WORKGROUPS,
    APAR_PLAN_TILES,
    APAR_PLAN_DFS_THREADS,
    APAR_PLAN_PATH_OFS,
    APAR_PLAN_PATH_IDS,
    APAR_PLAN_GEOMETRY,
    apar_pool_create,
    apar_pool_destroy,
    apar_pool_stats,
    apar_profile_enable,
    apar_profile_read,
    apar_read_kv_rows,
    apar_set_chunk_blocks,
    apar_status_string,
    apar_thread_block_table,
    apar_thread_create,
    apar_thread_len,
    exported_symbols,
    library_path,
)

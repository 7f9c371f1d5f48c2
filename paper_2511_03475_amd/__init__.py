"""MI355X (gfx950) extend attention over a paged prefix cache: Python binding of the C ABI."""
from .binding import (  # noqa: F401
    CP_ERR_ALIGN, CP_ERR_LAUNCH, CP_ERR_LENGTHS, CP_ERR_NULL, CP_ERR_TABLE, CP_ERR_SHAPE, CP_ERR_WORKSPACE, CP_OK, EXPORTS, ContextIndex, CpError, Shape,
    Conversation, cp_dedup_chunks, cp_dedup_hash, cp_index_distinct, cp_index_schedule,
    cp_check_tables, cp_set_debug_validate, cp_plan_kind, PLAN_KERNELS,
    cp_context_distance, cp_extend_attention, cp_extend_attention_noalloc, cp_noalloc_scratch_bytes, cp_num_splits, cp_shape, cp_status_string, cp_workspace_bytes,
    cp_probe_mfma, cp_probe_mix, cp_probe_copy, cp_probe_fill_lds, cp_probe_mfma_flops, cp_probe_mfma_sink_floats, cp_write_kv, load_library,
)
from .build import LIB_PATH, build  # noqa: F401

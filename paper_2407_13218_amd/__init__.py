"""MI355X-native exhaustive filtered top-k retrieval (the data-parallel hot path of
LiNR, arXiv 2407.13218, Sec. 3.1): HIP kernels behind a C ABI, with a thin ctypes
binding.  Every step of a search runs in the HIP library; there is no CPU fallback."""
from .binding import (  # noqa: F401
    F32, BF16, I8, BITS, NO_ID, MAX_K, MAX_M,
    SRC_HOST, SRC_DEVICE_COPY, SRC_DEVICE_BORROW, FILTERS_ON_DEVICE, FILTERS_ON_HOST, PLAN_MASKING, PLAN_PREFILTER, STRATEGY_MASKING, STRATEGY_PREFILTER, plan_filtered,
    LinrError, lib_path, load_library,
    index_create, index_load_fp32, index_load_bf16, index_load_int8, index_info, index_destroy,
    search_workspace_bytes, search_filtered, search_filtered_timed, set_tuning, strerror,
    events_create, events_destroy, events_elapsed_ms, MAX_STAGES, STAGE_NAMES,
    index_build_bits, index_load_bits, quantize_queries, search_bits_workspace_bytes, search_bits, search_bits_timed,
    select_bits_workspace_bytes, select_bits,
    search_two_stage_workspace_bytes, search_two_stage,
    index_enable_updates, index_upsert, index_delete, index_sync_updates,
    index_load_clauses, search_clauses_workspace_bytes, search_clauses, search_clauses_timed,
    search_clauses_prefilter, index_upsert_clauses, search_prefilter_workspace_bytes, search_filtered_prefilter,
    search_filtered_noalloc, NOALLOC_SCRATCH_BYTES,
    Index,
)

"""MI355X-native CItruS chunk-eviction hot path: HIP kernels behind a C ABI
(include/citrus.h) and this thin ctypes binding."""

from .binding import (  # noqa: F401
    BF16, F32, CACHE_DUAL, CACHE_INSTR, CACHE_SHARED, CACHE_STANDARD, LM_EVICT_THEN_APPEND, LM_SCORE_AFTER_APPEND, SCORE_ACCUMULATED, SCORE_PER_STEP,
    SELECT_PER_KV_HEAD, SELECT_PER_LAYER,
    CitrusError, Config, DocumentState, SideStream, abi_version, alloc_workspace, citrus_cache_score, citrus_chunk_attn, citrus_decode_step, citrus_evict_cache, citrus_evict_cache_static, citrus_instr_score,
    citrus_kv_compact, citrus_process_document, citrus_rope, citrus_score_accumulate, citrus_score_gather,
    citrus_topk_select, resident_doc, static_scratch_bytes, status_string, workspace_bytes,
)

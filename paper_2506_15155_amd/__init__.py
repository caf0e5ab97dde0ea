"""MI355X-native chunk-backed KV tensors, KV append and batched GQA decode attention
(the data-parallel hot path of the eLLM elastic memory framework, arXiv 2506.15155).

This package is a thin ctypes binding over libellm.so (hand-written HIP for gfx950). It only
marshals arguments; every step of the path runs in the library. Importing it without a built
library raises: there is no fallback path.
"""
from .binding import (  # noqa: F401
    EllmError, ERR, LIB_PATH, lib,
    ellm_pool_create, ellm_pool_destroy, ellm_tensor_create, ellm_tensor_destroy,
    ellm_tensor_map_chunks, ellm_tensor_unmap_chunks, ellm_pool_transfer, ellm_pool_set_act_busy,
    ellm_kv_append, ellm_decode_attention, ellm_kv_append_decode, ellm_tensor_release, ellm_tensor_acquire,
    ellm_tensor_is_released, ellm_kv_premap_next, ellm_pool_flush_tables, ellm_pool_set_logical_host_slots,
    ellm_pool_get_logical_host_slots, ellm_pool_slo_configure, ellm_pool_slo_observe, ellm_chunk_deflate_to_host, ellm_chunk_inflate_from_host,
    ellm_pool_sync, ellm_pool_get_geometry, ellm_tensor_get_table, ellm_pool_get_owner_state,
    ellm_pool_get_host_slots, ellm_decode_plan, ellm_pool_set_split_tokens, ellm_pool_self_check,
    ellm_pool_profile_enable, ellm_pool_profile_stride, ellm_pool_profile_collect,
    ellm_debug_set_waves, ellm_debug_vmm_latency, ellm_debug_vmm_buffer_create, ellm_debug_vmm_buffer_destroy, ellm_debug_copy, ellm_debug_stream_read, ellm_debug_kv_stream_read,
    ellm_last_error,
    ELLM_OWNER_KV, ELLM_OWNER_ACT, ELLM_CHUNK_FREE, ELLM_CHUNK_MAPPED, ELLM_CHUNK_BUSY,
    ELLM_MAP_ALLOW_INFLATE, ELLM_POOL_METADATA_ONLY, ELLM_BF16,
)

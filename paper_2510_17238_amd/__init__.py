"""Streaming-constrained attention for MI355X (gfx950): thin Python binding over libst.so.

Every step of the path runs in the HIP kernels of the C-ABI library; this package only
marshals arguments (torch tensors -> device pointers, the current HIP stream).  There is
no CPU or PyTorch fallback: importing the binding without a built library raises.
"""
from .binding import (  # noqa: F401
    ST_SOURCE, ST_REASONING, ST_F32, ST_BF16, ST_FP8_E4M3, ST_BLOCK_SS, ST_BLOCK_RS, ST_BLOCK_RR,
    ST_TILE_SKIP, ST_TILE_FULL, ST_TILE_PARTIAL, PAGE,
    StError, Plan, KVCache, DualCache, library_path, load_library, load_probe_library,
    st_version, st_last_error, st_profile_enable, st_profile_repeat, st_profile_wave_trace, st_profile_read, st_probe_paged_read, st_probe_mfma_bf16, ST_PROF_PREFILL_ATTN, ST_PROF_DECODE_SPLIT, ST_PROF_BWD_DQ, ST_PROF_BWD_DKV, ST_PROF_TILE_PACK, ST_PROF_SOURCE_CHUNK, st_rope_apply, st_rope_apply_qk, st_plan_workspace_bytes, st_plan_create,
    st_prefill_workspace_bytes, st_attn_prefill, st_attn_prefill_rope, st_attn_prefill_ids, st_attn_prefill_bwd, st_kv_append, st_kv_append_rope, st_attn_decode_dual_append, st_decode_workspace_bytes,
    st_attn_decode_dual, st_attn_decode_dual_static, st_decode_static_scratch_bytes, st_attn_decode_dual_rope, st_source_chunk_workspace_bytes, st_attn_source_chunk, st_attn_source_chunk_rope, k_pool_to_logical, v_pool_to_logical, k_pool8_to_logical, scale_to_logical, k_pool_from_logical,
    v_pool_from_logical, ST_SCHED_STREAMING, ST_SCHED_SERIAL, ST_SCHED_BATCH, st_stream_timeline, st_stream_run,
)

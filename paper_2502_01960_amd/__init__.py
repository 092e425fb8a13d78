"""Python binding of libmpic (selective-recompute prefill on one MI355X).

Argument marshalling only: every step of the path runs in the HIP library.
"""
from .binding import (  # noqa: F401
    MpicError, Context, Plan, Store, ChunkSources, lib_path, load_library,
    mpic_create, mpic_destroy, mpic_set_option, MPIC_OPT_ATTN_BLOCK_KEYS, mpic_plan_create, mpic_plan_get, mpic_plan_get_rope, mpic_plan_get_fresh_rope,
    mpic_plan_destroy, mpic_assemble_kv, mpic_assemble_kv_parts, mpic_selective_attn, mpic_selective_attn_link_next, mpic_selective_attn_in_place, mpic_decode_attn_in_place, mpic_decode_attn, mpic_decode_attn_static, mpic_k_distance, mpic_rank_tokens, mpic_strerror, mpic_last_error,
    mpic_store_create, mpic_store_destroy, mpic_store_put, mpic_store_move, mpic_store_expire, mpic_store_drop,
    mpic_store_lookup, mpic_store_layer, mpic_prefill_layers,
    MPIC_TIER_MISSING, MPIC_TIER_HBM, MPIC_TIER_HOST, MPIC_TIER_DISK, MPIC_ERR_IO, MPIC_ERR_CACHE_MISS,
    MPIC_F32, MPIC_BF16, MPIC_PART_CACHED, MPIC_PART_FRESH, MPIC_PART_BACKGROUND, MPIC_K_LISTED, MPIC_SRC_DEVICE, MPIC_SRC_HOST_STAGED, MPIC_SRC_HOST_MAPPED, PLAN_FIELDS,
)

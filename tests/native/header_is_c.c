/* The public header must be plain C: compiled with gcc -std=c99 -pedantic -Werror by
 * tests/test_planner_host.py.  Every declared entry point is referenced once so that a
 * missing or C++-only declaration fails the build. */
#include "mpic.h"

static void* use[] = {
    (void*)mpic_create,          (void*)mpic_destroy,        (void*)mpic_plan_create,  (void*)mpic_plan_create_selected,
    (void*)mpic_plan_get,        (void*)mpic_plan_get_rope,  (void*)mpic_plan_get_fresh_rope,
    (void*)mpic_plan_destroy,    (void*)mpic_assemble_kv,    (void*)mpic_assemble_kv_parts,
    (void*)mpic_selective_attn,  (void*)mpic_decode_attn,  (void*)mpic_decode_attn_static, (void*)mpic_selective_attn_in_place, (void*)mpic_decode_attn_in_place,  (void*)mpic_k_distance,   (void*)mpic_rank_tokens,
    (void*)mpic_store_create,    (void*)mpic_store_destroy,  (void*)mpic_store_put,    (void*)mpic_store_move,
    (void*)mpic_store_expire,    (void*)mpic_store_drop,     (void*)mpic_store_lookup, (void*)mpic_store_layer,
    (void*)mpic_prefill_layers,  (void*)mpic_selective_attn_link_next, (void*)mpic_set_option,  (void*)mpic_strerror,       (void*)mpic_last_error};

int main(void) {
  mpic_config c;
  mpic_segment s;
  mpic_chunk_src src;
  c.n_q_heads = 4; c.n_kv_heads = 4; c.head_dim = 64; c.dtype = MPIC_F32; c.rope_theta = 1e4;
  c.rope_interleaved = 0; c.page_size = 0; c.fresh_pre_rope = 0; c.lazy_rope = 0;
  s.kind = 1; s.len = 4; s.chunk = 0; s.k = MPIC_K_LISTED;
  src.k = 0; src.v = 0; src.len = 4; src.on_host = MPIC_SRC_HOST_MAPPED;
  return (int)(sizeof(use) / sizeof(use[0])) + c.head_dim + s.k + src.on_host + MPIC_PART_BACKGROUND + MPIC_PLAN_ATTN_TILES + MPIC_TIER_DISK +
             MPIC_ERR_CACHE_MISS == 0;
}

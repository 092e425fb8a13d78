/*
 * libmpic -- selective-recompute prefill for position-independent multimodal
 * context caching, for one AMD MI355X (gfx950).
 *
 * The library implements the data-parallel hot path of the method: the linker
 * that joins stored per-image KV caches and freshly computed rows into one
 * request context (Sec. 3.1 item 5, Sec. 4.1, Fig. 7 steps 1-2), and selective
 * attention of the recomputed tokens over that linked cache (Fig. 7 step 3,
 * App. A).  The paper leaves positional embedding out of Fig. 7; here a stored key
 * that was computed at chunk-local position t is moved to its global position by
 * a rotary shift of its chunk's offset in the request.
 *
 * General conventions
 *   - Plain C ABI.  Every call returns an int: MPIC_OK (0) or a negative
 *     mpic_status.  Nothing throws or aborts across the boundary.
 *   - All arguments are validated on the host first; a call that fails enqueues
 *     no GPU work.
 *   - Tensors are token-major, innermost dimension contiguous:
 *     [tokens][heads][head_dim], element type given by mpic_config.dtype.
 *   - The caller owns every data buffer and must keep it alive and unchanged
 *     until the work enqueued on `stream` has completed.  The library owns what it
 *     creates (context, plans, staging buffers, its side stream and events).
 *   - `stream` arguments are hipStream_t values passed as void* (NULL = the
 *     default stream).  Calls are stream-ordered and return without waiting.
 *   - Pointers documented "device" must be device-accessible on the GPU that is
 *     current when the call is made; pointers documented "host" are ordinary host
 *     memory unless "pinned" is stated.
 *   - A context and its plans may be used from one host thread at a time.
 */
#ifndef MPIC_H
#define MPIC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mpic_ctx mpic_ctx;   /* opaque: configuration, side stream, events, staging */
typedef struct mpic_plan mpic_plan; /* opaque: host and device copies of the integer plan   */
typedef struct mpic_store mpic_store; /* opaque: library of stored chunk caches in three tiers */

typedef enum mpic_status {
  MPIC_OK = 0,
  MPIC_ERR_INVALID = -1,     /* an argument violates the documented contract   */
  MPIC_ERR_UNSUPPORTED = -2, /* valid request that this build has no kernel for */
  MPIC_ERR_OOM = -3,         /* host or device allocation failed                */
  MPIC_ERR_HIP = -4,         /* a HIP runtime call failed (see mpic_last_error) */
  MPIC_ERR_IO = -5,          /* a file of the disk tier could not be written     */
  MPIC_ERR_CACHE_MISS = -6   /* a stored cache the plan reads is missing or its  */
                             /* load failed: plan those chunks as recomputed     */
} mpic_status;

typedef enum mpic_dtype { MPIC_F32 = 0, MPIC_BF16 = 1 } mpic_dtype;

typedef struct mpic_config {
  int32_t n_q_heads;        /* query heads Hq                                        */
  int32_t n_kv_heads;       /* key/value heads Hkv; Hq % Hkv == 0 (grouped queries)  */
  int32_t head_dim;         /* D; F32: 64 or 128, BF16: 128                          */
  int32_t dtype;            /* mpic_dtype of Q, K, V, the context and the output     */
  double rope_theta;        /* rotary base; pair i turns by shift * theta^(-2i/D)    */
  int32_t rope_interleaved; /* 0: pairs (i, i+D/2) "rotate-half"; 1: pairs (2i,2i+1) */
  int32_t page_size;        /* 0: contiguous context; >0: tokens per physical page   */
  int32_t fresh_pre_rope;   /* 0: fresh Q and K already carry their positions;       */
                            /* 1: they come straight from the projections and the    */
                            /*    library rotates them (K while linking, Q while     */
                            /*    attending) by the position id of their token, the  */
                            /*    positional step that Fig. 7 leaves out             */
  int32_t lazy_rope;        /* 0: stored keys are rotated to their global position   */
                            /*    while they are linked (the context holds final     */
                            /*    keys);                                             */
                            /* 1: stored keys are never rewritten: linking copies    */
                            /*    them as stored (or does not touch them at all, see */
                            /*    mpic_selective_attn_in_place) and the attention    */
                            /*    kernels turn the query back by the shift of each   */
                            /*    chunk instance instead, <Rot(-s) q, k> =           */
                            /*    <q, Rot(s) k> (Sec. 4.1: single-step linking that  */
                            /*    only joins caches; Fig. 7 step 2)                  */
} mpic_config;

/* One segment of a request, in prompt order. */
typedef struct mpic_segment {
  int32_t kind;  /* 0 = text (always recomputed), 1 = cached chunk                       */
  int32_t len;   /* tokens, >= 0                                                         */
  int32_t chunk; /* kind 1: index into the srcs[] array given to mpic_assemble_kv        */
  int32_t k;     /* kind 1: tokens recomputed at the head of the chunk; -1 = default_k;  */
                 /*         >= len recomputes the whole chunk (a cache that is missing   */
                 /*         or failed to load, Sec. 3.2); MPIC_K_LISTED: the tokens are  */
                 /*         named one by one (mpic_plan_create_selected only)            */
} mpic_segment;
#define MPIC_K_LISTED (-2)

/* Stored cache of one chunk for the layer being assembled. */
typedef struct mpic_chunk_src {
  const void* k;   /* [len][Hkv][D], keys already rotated for chunk-local positions 0..len-1 */
  const void* v;   /* [len][Hkv][D]                                                          */
  int32_t len;     /* must equal the len of every segment that refers to this source         */
  int32_t on_host; /* where the cache lives, see below                                        */
} mpic_chunk_src;
enum {
  MPIC_SRC_DEVICE = 0,      /* device memory, read in place                                        */
  MPIC_SRC_HOST_STAGED = 1, /* pinned host memory: copied by the DMA engines on the library's side  */
                            /* stream into library staging, then linked (uses no compute unit while */
                            /* in flight, so it overlaps with whatever the GPU computes)            */
  MPIC_SRC_HOST_MAPPED = 2  /* pinned host memory that the GPU can address (hipHostMalloc): the     */
                            /* linking kernel reads it in place over the bus -- no staging, no     */
                            /* copies, higher bus throughput; the launch lasts as long as the      */
                            /* transfer, so issue it (mpic_assemble_kv_parts, MPIC_PART_CACHED) on */
                            /* another stream than the computation it should overlap with          */
};

/* Selectors for mpic_plan_get.  All arrays are int32. */
enum {
  MPIC_PLAN_CTX_OFF = 0,  /* [B+1]  prefix sums of request context lengths N_b               */
  MPIC_PLAN_Q_OFF = 1,    /* [B+1]  prefix sums of recompute-set sizes Nq_b                  */
  MPIC_PLAN_Q_POS = 2,    /* [Nq]   position id (inside its request) of each fresh row       */
  MPIC_PLAN_Q_REQ = 3,    /* [Nq]   request of each fresh row                                */
  MPIC_PLAN_SLOT_MAP = 4, /* [Nq]   physical context slot each fresh row is written to       */
  MPIC_PLAN_SRC_INST = 5, /* [N]    chunk instance that feeds a position, -1 = fresh row     */
  MPIC_PLAN_SRC_ROW = 6,  /* [N]    row inside that chunk, or index of the fresh row         */
  MPIC_PLAN_DST_SLOT = 7, /* [N]    physical context slot of a position                      */
  MPIC_PLAN_INST_SRC = 8, /* [n_inst] srcs[] index of each chunk instance                    */
  MPIC_PLAN_INST_DELTA = 9,  /* [n_inst] rotary shift = position of the instance's first token */
  MPIC_PLAN_INST_LEN = 10,   /* [n_inst] tokens                                                */
  MPIC_PLAN_INST_K = 11,     /* [n_inst] effective k = min(k, len); listed set: its leading run */
  MPIC_PLAN_INST_REQ = 12,   /* [n_inst] owning request                                        */
  MPIC_PLAN_RUNS = 13,       /* [n_runs][4] (request, first fresh row, length, first position) */
  MPIC_PLAN_LAUNCH_ESTIMATE = 15, /* [4] the planner's simulation of the attention launch: its  */
                             /* duration and the compute-unit time it leaves idle (summed over */
                             /* the chip), both in 64-key blocks of one tile; 1 if a launch    */
                             /* can carry the linking of the next layer                        */
                             /* (mpic_selective_attn_link_next); 1 if that is also predicted   */
                             /* to pay (the linking fits into the idle time, or the launch is  */
                             /* too short for a second stream to help)                         */
  MPIC_PLAN_KEY_BLOCKS_32 = 16, /* lazy_rope contexts: [n_blocks][4] (first position, keys,    */
  MPIC_PLAN_KEY_BLOCKS_64 = 17, /* chunk instance or -1 = fresh rows, request): the keys of    */
  MPIC_PLAN_KEY_BLOCKS_96 = 18, /* every request cut into blocks of at most 32 / 64 / 96 keys  */
                             /* that never straddle a change of source; request after request, */
                             /* inside a request the blocks of fresh rows first, then those of */
                             /* stored rows, each part in position order.  The decode kernel   */
                             /* walks the first list, the two shapes of the attention kernel   */
                             /* the others                                                     */
  MPIC_PLAN_LAZY_TILES_64 = 19, /* lazy_rope contexts: [n_tiles][4] for every entry of         */
  MPIC_PLAN_LAZY_TILES_96 = 20, /* MPIC_PLAN_ATTN_TILES the blocks it visits, as (f0, f1, s0,  */
                             /* s1): fresh blocks f0..f1-1 and stored blocks s0..s1-1 of its   */
                             /* request, counted inside their parts                            */
  MPIC_PLAN_KEY_BLOCK_PARTS_32 = 21, /* lazy_rope contexts: [B][3] (first fresh block, first   */
  MPIC_PLAN_KEY_BLOCK_PARTS_64 = 22, /* stored block, end) of every request in the list above  */
  MPIC_PLAN_KEY_BLOCK_PARTS_96 = 23,
  MPIC_PLAN_ATTN_TILES = 14  /* [n_tiles][8] launch order of the attention kernel: (request,   */
                             /* kv head, first flattened row, rows, end key, first key, slot   */
                             /* of the partial result or -1, 0); flattened row = (fresh row -  */
                             /* q_off[request]) * (Hq/Hkv) + head in group.  A tile visits     */
                             /* keys first..end-1; tiles whose first key is > 0 or whose slot  */
                             /* is >= 0 are pieces of one tile cut along the keys, merged by a */
                             /* second kernel                                                  */
};

/*
 * Create a context.  Host only: no GPU call is made until the first
 * mpic_assemble_kv / mpic_selective_attn, which binds the context to the GPU that
 * is current at that moment.
 * Errors: MPIC_ERR_INVALID (null pointer, non-positive sizes, Hq % Hkv != 0, odd
 * head_dim, theta <= 0, page_size < 0, flags other than 0 / 1), MPIC_ERR_UNSUPPORTED
 * (dtype / head_dim).
 */
int mpic_create(mpic_ctx** out, const mpic_config* config);

/*
 * Options of a context.
 *   MPIC_OPT_ATTN_BLOCK_KEYS  keys per LDS block of the bf16 attention kernel: 64, 96, or 0 =
 *     the library chooses (default).  96 is the faster shape when the launch has the chip to
 *     itself; 64 uses fewer registers and leaves room on every SIMD for a wave of another
 *     kernel, which is what linking on a second stream (MPIC_PART_BACKGROUND,
 *     MPIC_SRC_HOST_MAPPED) needs to overlap with the attention.  With 0 a context uses 96 until
 *     it has linked that way once, then 64; mpic_prefill_layers picks per call.
 * Errors: INVALID (unknown option or value).
 */
enum { MPIC_OPT_ATTN_BLOCK_KEYS = 1 };
int mpic_set_option(mpic_ctx* ctx, int32_t option, int64_t value);

/* Destroy a context after all of its plans.  Waits for the side stream.  NULL is allowed. */
void mpic_destroy(mpic_ctx* ctx);

/*
 * Build the integer plan of a batch of requests (Sec. 4.2: the recompute set is
 * every text token plus the first k tokens of every chunk; Fig. 7 step 2: those
 * rows replace the stored ones, every other row comes from its chunk).  Host only.
 *
 *   n_requests        B >= 1
 *   seg_off  [B+1]    host; request b owns segs[seg_off[b] .. seg_off[b+1])
 *   segs              host; see mpic_segment
 *   default_k         >= 0
 *   page_table        host; may be NULL when config.page_size == 0 or no request holds
 *                     a token.  Physical page ids
 *                     (0 <= id < n_pool_pages), all requests concatenated.
 *   page_table_off [B+1]  host; request b owns page_table[off[b] .. off[b+1]), which
 *                     must cover ceil(N_b / page_size) pages.  No page id may be used
 *                     twice inside the batch.
 *   n_pool_pages      pages in the pool the tables index (ignored when contiguous)
 *
 * Contiguous layout: the context buffers hold the requests one after the other,
 * request b at slots ctx_off[b] .. ctx_off[b+1).  Paged layout: position p of
 * request b lives at slot table_b[p / page_size] * page_size + p % page_size.
 * The plan can be reused for every layer of the batch.
 * Errors: MPIC_ERR_INVALID for any violation above (negative len, bad kind, chunk
 * index < 0, table too short, duplicate or out-of-range page id, totals >= 2^31).
 */
int mpic_plan_create(mpic_ctx* ctx, int32_t n_requests, const int32_t* seg_off,
                     const mpic_segment* segs, int32_t default_k, const int32_t* page_table,
                     const int32_t* page_table_off, int64_t n_pool_pages, mpic_plan** out);

/*
 * The same plan for recompute sets chosen by another policy than "the first k tokens"
 * (Sec. 4.2 derives that rule from a ranking of tokens by K distance; Sec. 5.1 compares with
 * recomputing the tokens of largest deviation): a chunk segment whose k is MPIC_K_LISTED
 * recomputes exactly the chunk-local tokens sel_idx[sel_off[s] .. sel_off[s+1]), s being
 * the segment's index in segs (any order, duplicates allowed, each 0 <= index < len; an
 * empty range recomputes nothing).  Other segments follow their k as in mpic_plan_create.
 * Text tokens are always recomputed.  sel_off [n_segs + 1] and sel_idx are host arrays and
 * may be NULL when no segment is listed.
 * Errors: as mpic_plan_create; MPIC_ERR_INVALID for a listed token outside its chunk or a
 * listed segment without sel_off.
 */
int mpic_plan_create_selected(mpic_ctx* ctx, int32_t n_requests, const int32_t* seg_off,
                              const mpic_segment* segs, int32_t default_k, const int32_t* sel_off,
                              const int32_t* sel_idx, const int32_t* page_table,
                              const int32_t* page_table_off, int64_t n_pool_pages, mpic_plan** out);

/* Borrow one host array of the plan; valid until mpic_plan_destroy. */
int mpic_plan_get(const mpic_plan* plan, int32_t what, const int32_t** host_ptr, size_t* n);

/*
 * Borrow the rotary tables of the plan: cos and sin of shift * theta^(-2i/D),
 * [n_inst][D/2] floats each, evaluated in double precision and rounded once.
 */
int mpic_plan_get_rope(const mpic_plan* plan, const float** cos_tab, const float** sin_tab,
                       size_t* n);

/*
 * Borrow the rotary tables of the fresh rows (contexts created with fresh_pre_rope = 1;
 * otherwise *n_rows = 0): table_row [Nq] gives, for every fresh row, its row in cos_tab /
 * sin_tab, which hold cos and sin of position * theta^(-2i/D) as [n_rows][D/2] floats, one
 * row per distinct position id of the batch.
 */
int mpic_plan_get_fresh_rope(const mpic_plan* plan, const int32_t** table_row, const float** cos_tab,
                             const float** sin_tab, size_t* n_rows);

/* Destroy a plan (device copies included).  The caller must have synchronised every
 * stream that still uses it.  NULL is allowed. */
void mpic_plan_destroy(mpic_plan* plan);

/*
 * Link one layer's context (Sec. 3.1 item 5; Fig. 7 step 2; parallel transfer of
 * Sec. 3.2 for sources that are not on the GPU).
 * For every context position exactly one of:
 *   - position in the recompute set:  K_ctx[slot] = fresh_k[row], V_ctx[slot] = fresh_v[row]
 *   - otherwise (row t of chunk instance c): V_ctx[slot] = V_c[t] and
 *     K_ctx[slot] = K_c[t] rotated head by head by the instance's shift
 *     (pair (x, y) -> (x cos - y sin, x sin + y cos)), computed in fp32 and rounded
 *     once to the storage type.
 * Slots that belong to no position (tail of a last page, unused pool pages) are not
 * touched.  On a context with lazy_rope = 1 stored keys are copied as stored, bit for bit
 * (K_ctx[slot] = K_c[t]); mpic_selective_attn and mpic_decode_attn then apply the shift on
 * the query side.
 *
 *   srcs [n_srcs]     host array; every chunk index used by the plan must be < n_srcs
 *                     and srcs[i].len must match.  k / v: device, or pinned host memory
 *                     according to on_host (MPIC_SRC_*).
 *   fresh_k, fresh_v  device [n_fresh_rows][Hkv][D]; may be NULL only if the plan
 *                     has no fresh row.  Keys already carry their global position,
 *                     unless the context was created with fresh_pre_rope = 1: then each
 *                     fresh key is rotated by its position id on its way into K_ctx
 *                     (fp32 arithmetic, one rounding), like a stored key by its shift.
 *   n_fresh_rows      must equal the plan's total recompute-set size
 *   k_ctx, v_ctx      device [n_ctx_slots][Hkv][D], written
 *   n_ctx_slots       slots in k_ctx / v_ctx; must cover every slot of the plan
 *                     (contiguous: >= total N; paged: >= n_pool_pages * page_size)
 * Errors: MPIC_ERR_INVALID, MPIC_ERR_OOM (staging), MPIC_ERR_HIP.
 */
int mpic_assemble_kv(mpic_ctx* ctx, mpic_plan* plan, const mpic_chunk_src* srcs, int32_t n_srcs,
                     const void* fresh_k, const void* fresh_v, int64_t n_fresh_rows, void* k_ctx,
                     void* v_ctx, int64_t n_ctx_slots, void* stream);

/*
 * The same linking in two parts, for callers that overlap it with other work (Sec. 3.2:
 * preparing the stored caches proceeds concurrently with computation).  MPIC_PART_CACHED
 * links every row that comes from a stored chunk -- it needs only the plan and the chunk
 * sources, so it can run ahead, e.g. on another stream while the previous layer computes;
 * MPIC_PART_FRESH writes the rows of the recompute set once the model has produced them.
 * The two parts write disjoint rows and may run in either order or concurrently; with
 * both bits the call equals mpic_assemble_kv.  With MPIC_PART_CACHED alone fresh_k, fresh_v
 * and n_fresh_rows are ignored; with MPIC_PART_FRESH alone srcs and n_srcs are ignored.
 * MPIC_PART_BACKGROUND may be added to either part: it tells the library that the call runs
 * beside other GPU work on another stream, and the linking kernel is then held to a small grid
 * that strides over the rows, so that it takes a few wave slots for longer instead of the
 * whole chip for a moment (alone it would run several times slower).
 * Errors: as mpic_assemble_kv; MPIC_ERR_INVALID for an empty or unknown `parts`.
 */
enum { MPIC_PART_CACHED = 1, MPIC_PART_FRESH = 2, MPIC_PART_BACKGROUND = 4 };
int mpic_assemble_kv_parts(mpic_ctx* ctx, mpic_plan* plan, const mpic_chunk_src* srcs,
                           int32_t n_srcs, const void* fresh_k, const void* fresh_v,
                           int64_t n_fresh_rows, void* k_ctx, void* v_ctx, int64_t n_ctx_slots,
                           uint32_t parts, void* stream);

/*
 * Selective attention (Fig. 7 step 3; App. A): for every fresh row r at position p
 * of its request and every query head h (kv head h / (Hq/Hkv)):
 *   s_j = softmax_scale * <fresh_q[r][h], K_ctx[slot(j)][kv]>   for positions j = 0..p
 *   out[r][h] = sum_j softmax(s)_j * V_ctx[slot(j)][kv]
 *   lse[r][h] = log sum_j exp(s_j)                               (optional)
 * BF16: products on the matrix cores with fp32 accumulation, softmax in fp32,
 * probabilities rounded to bf16 before the second product, one final rounding of
 * out.  F32: fp32 throughout.
 *
 *   fresh_q           device [n_fresh_rows][Hq][D], already rotated for its position;
 *                     with fresh_pre_rope = 1 not yet rotated: the kernel rotates each
 *                     row by its position id as it loads it (fp32 arithmetic, rounded
 *                     once to the storage type before the first product)
 *   k_ctx, v_ctx      device [n_ctx_slots][Hkv][D] as written by mpic_assemble_kv
 *   softmax_scale     finite, > 0 (1/sqrt(D) for the definition of App. A)
 *   out               device [n_fresh_rows][Hq][D], written
 *   lse               device float [n_fresh_rows][Hq], written; may be NULL
 * A plan with no fresh row is a no-op that returns MPIC_OK.
 * Small and medium batches are cut along the keys as well as along the rows (see
 * MPIC_PLAN_ATTN_TILES); the partial results live in a workspace owned by the context,
 * allocated on first use and grown (with a device synchronisation) when a later call needs
 * more, so calls of one context that use it must not overlap on different streams.
 * Errors: MPIC_ERR_INVALID, MPIC_ERR_OOM (workspace), MPIC_ERR_HIP.
 */
int mpic_selective_attn(mpic_ctx* ctx, mpic_plan* plan, const void* fresh_q, int64_t n_fresh_rows,
                        const void* k_ctx, const void* v_ctx, int64_t n_ctx_slots,
                        double softmax_scale, void* out, float* lse, void* stream);

/*
 * Selective attention over caches that are linked by reference (contexts created with
 * lazy_rope = 1; Sec. 4.1: the linker joins the stored caches in a single step; Fig. 7 steps
 * 2-3).  Same result as mpic_assemble_kv followed by mpic_selective_attn, but no stored row is
 * copied or rewritten: the kernel reads the rows of every chunk instance where its cache is
 * stored (srcs, device memory) and turns the query back by the instance's shift; only the rows
 * of the recompute set are read from k_ctx / v_ctx, where mpic_assemble_kv_parts with
 * MPIC_PART_FRESH has put them (the other slots of the context are never touched and may hold
 * anything).  Per layer the linking traffic drops from 4 * N * Hkv * D * elem bytes to
 * 4 * Nq * Hkv * D * elem, and caches of chunks shared by several requests exist once.
 *   srcs [n_srcs]     as for mpic_assemble_kv; every source the plan reads must be
 *                     MPIC_SRC_DEVICE (copy host-resident caches to the GPU first, or use
 *                     mpic_assemble_kv + mpic_selective_attn, which on these contexts copies
 *                     stored keys unrotated)
 * BF16: at most 128 chunk instances per plan (their addresses travel as kernel arguments).
 * Errors: as mpic_selective_attn; INVALID on a context without lazy_rope or for a source that
 * is not in device memory; UNSUPPORTED beyond 128 instances.
 */
int mpic_selective_attn_in_place(mpic_ctx* ctx, mpic_plan* plan, const void* fresh_q, int64_t n_fresh_rows,
                                 const mpic_chunk_src* srcs, int32_t n_srcs, const void* k_ctx,
                                 const void* v_ctx, int64_t n_ctx_slots, double softmax_scale, void* out,
                                 float* lse, void* stream);

/*
 * mpic_selective_attn of one layer and, in the same launch, the stored rows of the next
 * layer's context (what mpic_assemble_kv_parts with MPIC_PART_CACHED writes): workgroups
 * that follow the attention tiles in the grid link them while the attention drains, on
 * the compute units its last tiles leave idle (Sec. 3.2: preparing the next KV cache and
 * computing proceed concurrently; here without a second stream).
 *   next_srcs[n_srcs]        chunk caches of the next layer, as for mpic_assemble_kv
 *   next_k_ctx, next_v_ctx   device, n_ctx_slots rows each, written; must not overlap
 *                            k_ctx / v_ctx
 * The fused launch needs bf16, device-resident sources, at most 128 chunk instances in
 * the plan and Hkv * D / 16 dividing 512; otherwise (and when the recompute set is empty)
 * the call does the same work with a launch of its own after the attention.  Whether
 * fusing pays depends on how much of the chip the attention tiles leave idle at the end:
 * MPIC_PLAN_LAUNCH_ESTIMATE holds the planner's prediction (a batch whose tiles fill the
 * chip evenly is better served by MPIC_PART_CACHED | MPIC_PART_BACKGROUND on a second
 * stream).  The fresh rows of the next layer are not touched: link them
 * (MPIC_PART_FRESH) before that layer's attention.
 * Errors: as mpic_selective_attn and mpic_assemble_kv; INVALID if the buffers overlap.
 */
int mpic_selective_attn_link_next(mpic_ctx* ctx, mpic_plan* plan, const void* fresh_q, int64_t n_fresh_rows,
                                  const void* k_ctx, const void* v_ctx, int64_t n_ctx_slots,
                                  double softmax_scale, void* out, float* lse,
                                  const mpic_chunk_src* next_srcs, int32_t n_srcs, void* next_k_ctx,
                                  void* next_v_ctx, void* stream);

/*
 * Decode-step attention over a linked context (App. A, autoregressive generation: the
 * query of the next token attends to every cached position and, its key and value being
 * appended to the cache, to itself).  For every request b of the plan and query head h
 * (kv head h / (Hq/Hkv)), with N_b the request's context length:
 *   s_j    = softmax_scale * <q[b][h], K_ctx[slot(j)][kv]>      for positions j = 0..N_b-1
 *   s_self = softmax_scale * <q[b][h], new_k[b][kv]>            (when new_k is given)
 *   out[b][h] = softmax-weighted sum of V_ctx[slot(j)][kv] and new_v[b][kv]
 *   lse[b][h] = log of the softmax denominator                  (optional)
 * BF16: products on the matrix cores with fp32 accumulation, probabilities rounded to bf16
 * before the second product, one final rounding of out; the new token's own term is
 * computed in fp32.  F32: fp32 throughout.
 *
 *   q                 device [B][Hq][D], rotated for position N_b by the caller (also on
 *                     fresh_pre_rope contexts: the plan holds no angle for that position)
 *   new_k, new_v      device [B][Hkv][D], key (rotated for position N_b) and value of the new
 *                     token; both NULL to attend to the linked context only
 *   k_ctx, v_ctx      device [n_ctx_slots][Hkv][D] as written by mpic_assemble_kv
 *   out               device [B][Hq][D], written; a request with no key at all (N_b = 0 and
 *                     no new_k) gets zeros and lse = -infinity
 *   lse               device float [B][Hq], written; may be NULL
 * Partial results of the key splits live in a workspace owned by the context, allocated on
 * the first call and grown (with a device synchronisation) when a later call needs more;
 * calls on one context must therefore not overlap on different streams.
 * Errors: MPIC_ERR_INVALID, MPIC_ERR_OOM (workspace), MPIC_ERR_HIP.
 */
int mpic_decode_attn(mpic_ctx* ctx, mpic_plan* plan, const void* q, const void* new_k,
                     const void* new_v, const void* k_ctx, const void* v_ctx, int64_t n_ctx_slots,
                     double softmax_scale, void* out, float* lse, void* stream);

/*
 * mpic_decode_attn over caches linked by reference (lazy_rope contexts): stored rows are read
 * in their caches (srcs: device memory, as for mpic_selective_attn_in_place), rows of the
 * recompute set in k_ctx / v_ctx.  Same arguments otherwise, same result.
 * Errors: as mpic_decode_attn and mpic_selective_attn_in_place.
 */
int mpic_decode_attn_in_place(mpic_ctx* ctx, mpic_plan* plan, const void* q, const void* new_k,
                              const void* new_v, const mpic_chunk_src* srcs, int32_t n_srcs,
                              const void* k_ctx, const void* v_ctx, int64_t n_ctx_slots,
                              double softmax_scale, void* out, float* lse, void* stream);

/*
 * mpic_decode_attn for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * result, but the partial results of the key splits live in a file-scope device array of the
 * library (8 MiB per GPU, held until the process ends) instead of the context's workspace,
 * and the call makes no hipMalloc, hipFree or other allocating call:
 *   - the context must be bound to the current GPU and the plan already uploaded to it, which
 *     any earlier GPU call with this plan does (mpic_assemble_kv, mpic_selective_attn,
 *     mpic_decode_attn); otherwise MPIC_ERR_INVALID;
 *   - a batch whose partial results ([B][Hq][splits][D+1] floats; splits is chosen so that
 *     B * Hkv * splits is about 256, and is 1 for larger batches) exceed 8 MiB is rejected
 *     with MPIC_ERR_UNSUPPORTED before anything is enqueued;
 *   - the first call on a GPU looks the array's device address up (no allocation).
 * All calls on one GPU share the array, whatever their context: calls that may overlap (on
 * different streams, or from different host threads) race.  The kernels write every partial
 * they later read, so nothing needs clearing between calls.
 * Errors: as mpic_decode_attn without OOM; INVALID / UNSUPPORTED as above.
 */
int mpic_decode_attn_static(mpic_ctx* ctx, mpic_plan* plan, const void* q, const void* new_k,
                            const void* new_v, const void* k_ctx, const void* v_ctx, int64_t n_ctx_slots,
                            double softmax_scale, void* out, float* lse, void* stream);

/*
 * K distance of every token of a chunk (Sec. 4.2: the L1 distance between the token's K
 * tensors in two caches of the same image computed at different positions):
 *   dist[t] = sum over kv heads and coordinates of |k_a[t] - k_b[t]|, fp32 accumulation.
 *   k_a, k_b          device [n_tokens][Hkv][D] in the context's dtype, 16-byte aligned
 *   dist              device float [n_tokens], written
 * Errors: MPIC_ERR_INVALID, MPIC_ERR_HIP.
 */
int mpic_k_distance(mpic_ctx* ctx, const void* k_a, const void* k_b, int64_t n_tokens, float* dist,
                    void* stream);

/*
 * Host only: the n_top tokens of largest distance (Sec. 4.2 ranks the tokens of every layer
 * this way and keeps the first 50), as ascending chunk-local indices ready for
 * mpic_plan_create_selected.  Of two tokens with the same distance the lower index ranks
 * higher; NaN ranks last.  n_top is clipped to n_tokens.
 *   dist              host float [n_tokens]
 *   idx               host int32 [min(n_top, n_tokens)], written
 * Errors: MPIC_ERR_INVALID, MPIC_ERR_OOM.
 */
int mpic_rank_tokens(const float* dist, int64_t n_tokens, int64_t n_top, int32_t* idx);

/* ---- library of stored caches and the layer pipeline (Sec. 3.1 items 2-3, Sec. 3.2, Fig. 6) ----
 *
 * A store keeps the KV cache of uploaded items, all layers of an item under one 64-bit
 * id, in one of three places: GPU memory, pinned CPU memory, or a file (Sec. 3.2 names
 * the three).  With a disk directory every stored cache also has its file, as in the
 * serving workflow of Sec. 3.1 (kept for serving, copied to disk, deleted on expiry).
 * A cache is bytes: what comes back is what went in, or the cache is reported missing.
 *
 * File <disk_dir>/<id as 16 hex digits>.mpickv, little endian:
 *     0  "MPICKV01"    8  u64 id      16  i32 len   20  i32 n_layers   24  i32 n_kv_heads
 *    28  i32 head_dim  32  i32 dtype  36  i32 0     40  u64 block_bytes = len*Hkv*D*elem
 *    48  u64 payload_off (multiple of 4096)          56  u64 checksum of bytes [0, 56)
 *    64  u64 x 2 x n_layers: checksum of the K block and of the V block of each layer
 *    payload_off: K block of layer 0, V block of layer 0, K block of layer 1, ...
 * checksum of n 8-byte words w_i: (n + sum_i w_i * P^(i+1)) mod 2^64, P = 0x9E3779B97F4A7C15.
 *
 * A store and the context it was made from are used by one host thread at a time; the
 * store's own reader threads are internal.  The caller must not move, replace, expire
 * or destroy a cache while GPU work that reads it is still enqueued.
 */
enum { MPIC_TIER_MISSING = 0, MPIC_TIER_HBM = 1, MPIC_TIER_HOST = 2, MPIC_TIER_DISK = 3 };

/*
 * Create a store for caches of ctx's shape (Hkv, D, dtype) with n_layers layers each.
 * disk_dir: directory of the disk tier (must exist), or NULL for none; files already
 * there whose header fits the shape are registered in tier DISK (a restarted server
 * finds its caches; they do not expire until put again).  io_threads: reader threads
 * of the disk tier (<= 0: 4).  Host only; GPU and pinned memory are touched by put /
 * move into those tiers.
 * Errors: INVALID (null pointer, n_layers < 1, directory missing), OOM.
 */
int mpic_store_create(mpic_ctx* ctx, int32_t n_layers, const char* disk_dir, int32_t io_threads,
                      mpic_store** out);

/* Destroy a store (before its context): waits for the device, frees both memory tiers,
 * keeps the files.  NULL is allowed. */
void mpic_store_destroy(mpic_store* store);

/*
 * Store (or replace) the cache of item `id`: k, v host pointers, [n_layers][len][Hkv][D],
 * copied before the call returns.  tier: where it is kept (HBM / HOST / DISK).  With a
 * disk tier the file is written in every case.  expires_at: time (caller's unit) at
 * which mpic_store_expire deletes it; < 0 = never.
 * Errors: INVALID (null, len < 1, unknown tier, DISK without disk_dir), OOM (device or
 * pinned allocation), IO (file could not be written; the store is unchanged), HIP.
 */
int mpic_store_put(mpic_store* store, uint64_t id, int32_t len, const void* k, const void* v,
                   int32_t tier, int64_t expires_at);

/*
 * Move a cache to another tier (promotion before use, demotion under memory pressure).
 * Into DISK the memory copy is freed (needs the disk tier); out of DISK the file is read
 * and verified.  Waits for the device before freeing memory.
 * Errors: INVALID (unknown id or tier), CACHE_MISS (the file is gone or damaged; the
 * cache is dropped from the store), OOM, HIP.
 */
int mpic_store_move(mpic_store* store, uint64_t id, int32_t tier);

/* Delete every cache with 0 <= expires_at <= now from all tiers, its file included
 * (Sec. 3.1: deleted after the expiration of its timeframe).  n_removed may be NULL. */
int mpic_store_expire(mpic_store* store, int64_t now, int32_t* n_removed);

/* Delete one cache from all tiers; unknown ids are ignored. */
int mpic_store_drop(mpic_store* store, uint64_t id);

/*
 * Where are these caches (Sec. 3.2: the lookup at the beginning of processing)?  tier[i]
 * receives MPIC_TIER_*, len[i] (may be NULL) the token count or 0.  A cache of tier DISK
 * whose file has disappeared or changed size is dropped and reported missing.
 */
int mpic_store_lookup(mpic_store* store, const uint64_t* ids, int32_t n, int32_t* tier, int32_t* len);

/*
 * Pointers to one layer of a cache held in HBM or HOST, for use with mpic_assemble_kv
 * (on_host is set to MPIC_SRC_DEVICE or MPIC_SRC_HOST_STAGED; HOST memory comes from
 * hipHostMalloc, so MPIC_SRC_HOST_MAPPED may be chosen instead).  Valid until the cache
 * is moved, replaced, expired or the store destroyed.
 * Errors: INVALID (unknown id, layer out of range, cache is in tier DISK).
 */
int mpic_store_layer(mpic_store* store, uint64_t id, int32_t layer, mpic_chunk_src* out);

/*
 * Selective-recompute prefill of n_layers layers of one batch, caches fetched from the
 * store while earlier layers compute (Sec. 3.2 / Fig. 6: transfer and computation run
 * concurrently; layer by layer, as the layer-wise transfer that Sec. 3.2 calls orthogonal).
 * ids[s] = store id of chunk source s of the plan (n_srcs entries; sources the plan does
 * not read may carry any id).  Per layer l the call does what mpic_assemble_kv followed
 * by mpic_selective_attn do with that layer's slices:
 *   fresh_q[l], fresh_k[l], fresh_v[l]  device, [n_fresh_rows][H][D]
 *   k_ctx[l], v_ctx[l]                  device, n_ctx_slots rows; the same buffer may be
 *                                       given to several layers (the library orders the
 *                                       linking of a later layer after the attention of
 *                                       the earlier one), distinct buffers let linking
 *                                       run further ahead
 *   out[l], lse[l]                      device; lse or lse[l] may be NULL
 * Schedule: the stored part of layer l is linked on a library stream (host and disk
 * tiers: the kernel reads pinned memory in place over the bus, held to a few workgroups
 * so that it runs beside the attention of earlier layers -- or, when the batch uses its
 * caches more than 1.25 times on average, staged copies that fetch each cache once;
 * disk: read and verified by the reader threads into a ring of pinned buffers, one
 * layer ahead of the linking),
 * fresh rows and attention run on `stream`, joined by events.  When every cache the plan
 * reads is in GPU memory there is nothing to fetch ahead: the stored rows of layer l+1 are
 * then linked by the attention launch of layer l (mpic_selective_attn_link_next), all on
 * `stream`.  On a lazy_rope context such caches are not linked at all but read in place
 * (mpic_selective_attn_in_place): the context buffers then receive the fresh rows only;
 * caches of the other tiers are linked as stored.  The call returns when everything is enqueued; the host thread waits only for
 * file reads.
 * failed: [n_srcs] or NULL; on MPIC_ERR_CACHE_MISS failed[s] = 1 for every source whose
 * cache is missing from the store or failed to load.  Missing caches and unreadable or
 * mis-sized files are found before anything is enqueued; a damaged block is found when
 * its layer is read: the call then stops enqueuing, earlier layers still complete, and
 * the cache is dropped from the store.  In both cases the caller plans those chunks
 * with k >= len and calls again (Sec. 3.2: fall back to computing without the cache).
 * Errors: INVALID (as mpic_assemble_kv / mpic_selective_attn; store of another context;
 * n_layers beyond the store's), CACHE_MISS, OOM, HIP.
 */
int mpic_prefill_layers(mpic_ctx* ctx, mpic_plan* plan, mpic_store* store, const uint64_t* ids,
                        int32_t n_srcs, int32_t n_layers, const void* const* fresh_q,
                        const void* const* fresh_k, const void* const* fresh_v, int64_t n_fresh_rows,
                        void* const* k_ctx, void* const* v_ctx, int64_t n_ctx_slots, double softmax_scale,
                        void* const* out, float* const* lse, void* stream, int32_t* failed);

/* Static description of a status code. */
const char* mpic_strerror(int status);

/* Detail of the last failing call on this context (empty string if none).  The
 * pointer stays valid until the next call on the context. */
const char* mpic_last_error(const mpic_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* MPIC_H */

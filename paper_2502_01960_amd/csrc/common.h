// Internal declarations shared by the translation units of libmpic.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "mpic.h"

namespace mpic {

// One attention work item, as laid out in MPIC_PLAN_ATTN_TILES (8 int32).
struct AttnTile {
  int32_t req;      // request b
  int32_t kv_head;  // key/value head g
  int32_t row0;     // first flattened row: (fresh row - q_off[b]) * G + head-in-group
  int32_t n_rows;   // rows in this tile (0 = padding entry, the workgroup exits)
  int32_t n_keys;   // keys key0..n_keys-1 are visited (at most the largest position in the tile + 1)
  int32_t key0;     // first key (a multiple of 64); > 0 only for pieces of a tile cut along the keys
  int32_t part;     // -1: the tile writes the output; >= 0: slot of its partial result
  int32_t pad;
};
static_assert(sizeof(AttnTile) == 32, "tile layout is part of the ABI");

// Rows whose keys were cut into several tiles: their partial results are merged afterwards.
struct AttnMerge {
  int32_t req, kv_head, row0, n_rows;
  int32_t first_part, n_parts;  // partial slots first_part .. first_part + n_parts - 1, in key order
  int32_t pad[2];
};
static_assert(sizeof(AttnMerge) == 32, "merge item layout");

// Contexts with lazy_rope: the keys of a request, cut into blocks that never straddle a change
// of source (a chunk instance, or a run of fresh rows).  Inside a block all keys come from
// consecutive rows of one source and lack the same position shift, so a kernel can turn the
// query back once per block instead of turning every key forward (Sec. 4.1: the linker joins
// caches and touches nothing else).  A block holds n_valid <= BN keys at positions pos0 ..
// pos0 + n_valid - 1; the rest of its BN slots are padding that the kernels mask.
struct KeyBlock {
  int32_t pos0;     // position (inside its request) of the block's first key
  int32_t n_valid;  // keys in the block, 1 .. BN
  int32_t inst;     // chunk instance that stores the keys (they lack its shift), -1 = fresh rows
  int32_t req;      // owning request
};
static_assert(sizeof(KeyBlock) == 16, "key block layout");
constexpr int kNumBlockSizes = 3;
constexpr int kBlockSizes[kNumBlockSizes] = {32, 64, 96};  // decode kernel, attention kernel shapes
inline int block_size_index(int bn) { return bn == 32 ? 0 : bn == 64 ? 1 : 2; }

// Device-resident copy of a plan.
struct PlanDevice {
  int32_t* src_inst = nullptr;
  int32_t* src_row = nullptr;
  int32_t* dst_slot = nullptr;
  int32_t* fresh_pos = nullptr;  // batch-flattened context position of every fresh row
  uint32_t* kv_off16 = nullptr;  // dst_slot * (bytes of a context row / 16): row offset in 16-byte units
  int32_t* q_pos = nullptr;
  int32_t* q_off = nullptr;
  int32_t* ctx_off = nullptr;
  float* rope_cos = nullptr;
  float* rope_sin = nullptr;
  int32_t* fresh_rot = nullptr;  // row of fresh_cos / fresh_sin for every fresh row (null: rows arrive rotated)
  float* fresh_cos = nullptr;
  float* fresh_sin = nullptr;
  AttnTile* tiles = nullptr;
  AttnMerge* merges = nullptr;
  // lazy_rope contexts, one set per block size (kBlockSizes)
  KeyBlock* kblk[kNumBlockSizes] = {};
  int32_t* kblk_first[kNumBlockSizes] = {};   // [B+1] first block of each request
  uint32_t* voff_ctx[kNumBlockSizes] = {};    // [n_blocks * BN + pad] row offsets (16-byte units), every row in the context
  uint32_t* voff_ref[kNumBlockSizes] = {};    // the same with stored rows addressed inside their source
  int32_t* kblk_mid[kNumBlockSizes] = {};     // [B] first stored block of each request
  int32_t* lazy_range[kNumBlockSizes] = {};   // [n_tiles][4] block ranges of every tile: fresh [f0, f1), stored [s0, s1)
  void* block = nullptr;  // the single allocation all of the above point into
  int device = -1;
};

}  // namespace mpic

struct mpic_ctx {
  mpic_config cfg{};
  int group = 1;  // Hq / Hkv
  std::string last_error;
  // GPU side, created on first use
  int device = -1;
  hipStream_t side_stream = nullptr;
  // Device staging for host-resident chunks, double buffered: the copies of one call may
  // run while the kernels of the previous call (linking and whatever the caller enqueued
  // after it) still read the other buffer.
  void* staging[2] = {nullptr, nullptr};
  size_t staging_bytes[2] = {0, 0};
  hipEvent_t ev_done[2] = {nullptr, nullptr};  // recorded after the last kernel that reads staging[i]
  bool ev_done_valid[2] = {false, false};
  int next_staging = 0;
  std::vector<hipEvent_t> ev_copy;             // one per transfer group
  // layer pipeline: stream on which stored rows are linked ahead of the computation, and the
  // events that order it against the caller's stream (two per layer in flight)
  hipStream_t link_stream = nullptr;
  std::vector<hipEvent_t> ev_layer;
  // shape of the bf16 attention kernel: 0 = the library chooses (96 keys per block, 64 once the
  // context has linked in the background: only that shape leaves registers for a wave of the
  // linking kernel beside it); 64 / 96 = fixed by mpic_set_option
  int32_t attn_block_keys = 0;
  int32_t attn_ablate = 0;  // probe builds only, see kAblate*
  bool background_seen = false;
  // partial results of the decode step (one per key split), grown on demand
  void* decode_ws = nullptr;
  size_t decode_ws_bytes = 0;
  // partial results of prefill tiles that were cut along the keys, grown on demand
  void* attn_ws = nullptr;
  size_t attn_ws_bytes = 0;
};

struct mpic_plan {
  mpic_ctx* ctx = nullptr;
  int32_t n_requests = 0;
  int64_t n_ctx = 0;      // total context positions of the batch
  int64_t n_q = 0;        // total fresh rows
  int64_t max_slot = -1;  // largest physical slot used
  int32_t max_src = -1;   // largest srcs[] index used
  std::vector<int32_t> ctx_off, q_off, q_pos, q_req, slot_map, src_inst, src_row, dst_slot;
  std::vector<int32_t> inst_src, inst_delta, inst_len, inst_k, inst_req, runs;
  std::vector<int32_t> inst_cached;  // rows each chunk instance actually takes from its stored cache
  std::vector<mpic::AttnTile> tiles;
  std::vector<mpic::AttnMerge> merges;  // tiles cut along the keys
  int32_t n_parts = 0;                  // partial-result slots those tiles use
  // the planner's simulation of the attention launch, in 64-key blocks of one tile: when the
  // last workgroup ends, and the compute-unit time left idle until then (summed over the chip)
  int64_t est_makespan_blocks = 0;
  int64_t est_idle_blocks = 0;
  std::vector<int32_t> launch_est;  // MPIC_PLAN_LAUNCH_ESTIMATE
  std::vector<float> rope_cos, rope_sin;
  // contexts with lazy_rope only: key blocks per block size, first block of every request,
  // attention tiles in block indices (empty for the decode block size)
  std::vector<mpic::KeyBlock> kblk[mpic::kNumBlockSizes];
  std::vector<int32_t> kblk_first[mpic::kNumBlockSizes];
  std::vector<int32_t> kblk_mid[mpic::kNumBlockSizes];    // [B] first stored block of every request (its fresh blocks come first)
  std::vector<int32_t> lazy_range[mpic::kNumBlockSizes];  // [n_tiles][4] fresh blocks [f0, f1) and stored blocks [s0, s1) of every tile
  std::vector<int32_t> kblk_flat[mpic::kNumBlockSizes];   // the blocks as int32 quadruples, for mpic_plan_get
  std::vector<int32_t> kblk_parts[mpic::kNumBlockSizes];  // [B][3] first fresh block, first stored block, end, for mpic_plan_get
  std::vector<int32_t> fresh_rot;            // contexts with fresh_pre_rope only
  std::vector<float> fresh_cos, fresh_sin;   // one row per distinct position id
  mpic::PlanDevice dev;
};

namespace mpic {

int fail(mpic_ctx* ctx, int code, const std::string& msg);
int fail_hip(mpic_ctx* ctx, hipError_t e, const char* what);

#define MPIC_HIP(ctx, call)                                  \
  do {                                                       \
    hipError_t e_ = (call);                                  \
    if (e_ != hipSuccess) return mpic::fail_hip(ctx, e_, #call); \
  } while (0)

// Implementations behind mpic_assemble_kv_parts / mpic_selective_attn (same arguments and
// checks); they may throw std::bad_alloc, which the extern "C" entry points turn into
// MPIC_ERR_OOM.  bind_device ties the context to the current GPU on first use.
int bind_device(mpic_ctx* ctx);
int assemble_parts(mpic_ctx* ctx, mpic_plan* plan, const mpic_chunk_src* srcs, int32_t n_srcs,
                   const void* fresh_k, const void* fresh_v, int64_t n_fresh_rows, void* k_ctx,
                   void* v_ctx, int64_t n_ctx_slots, uint32_t parts, void* stream);
// Stored rows of the next layer's context, to be linked along with an attention call.
struct NextLink {
  const mpic_chunk_src* srcs;
  int32_t n_srcs;
  void* k_ctx;
  void* v_ctx;
};
// refs non-null (lazy_rope contexts): stored rows are read in place in these chunk caches.
struct SrcRefs {
  const mpic_chunk_src* srcs;
  int32_t n_srcs;
};
int attend(mpic_ctx* ctx, mpic_plan* plan, const void* fresh_q, int64_t n_fresh_rows,
           const void* k_ctx, const void* v_ctx, int64_t n_ctx_slots, double softmax_scale, void* out,
           float* lse, void* stream, const NextLink* next, int32_t block_keys = 0, const SrcRefs* refs = nullptr);

// Rows of the attention tile handled by one workgroup of the bf16 kernel.
constexpr int kAttnTileRows = 256;

// ---- kernel launchers (each validates nothing: callers have done so) ----

struct AssembleArgs {
  const int32_t* src_inst;
  const int32_t* src_row;
  const int32_t* dst_slot;
  const float* rope_cos;
  const float* rope_sin;
  const int32_t* fresh_rot;  // non-null: fresh keys are rotated with row fresh_rot[r] of fresh_cos / fresh_sin
  const float* fresh_cos;
  const float* fresh_sin;
  const void* fresh_k;
  const void* fresh_v;
  void* k_ctx;
  void* v_ctx;
  int64_t pos_begin, pos_end;  // batch-flattened context positions handled by this launch
  int32_t inst_base;           // first chunk instance present in src_k / src_v
  int32_t n_inst;              // entries in src_k / src_v
  int32_t n_kv_heads, head_dim, interleaved;
  int32_t skip_fresh;          // 1: leave rows of the recompute set alone
  const int32_t* pos_list;     // non-null: the launch visits pos_list[pos_begin .. pos_end) instead of a range
  int32_t grid_limit;          // > 0: at most this many workgroups, which stride over the work
};
constexpr int kMaxInstPerLaunch = 128;
struct AssembleSrcTable {
  const void* k[kMaxInstPerLaunch];
  const void* v[kMaxInstPerLaunch];
};
hipError_t launch_assemble(int dtype, const AssembleArgs& a, const AssembleSrcTable& t,
                           hipStream_t stream);

struct AttnArgs {
  const AttnTile* tiles;
  int32_t n_tiles;
  const int32_t* q_pos;
  const int32_t* q_off;
  const int32_t* ctx_off;
  const int32_t* dst_slot;
  const uint32_t* kv_off16;
  const void* q;
  const void* k_ctx;
  const void* v_ctx;
  void* out;
  float* lse;
  float scale;
  int32_t n_q_heads, n_kv_heads, head_dim;
  int32_t n_requests;
  float* ws_o;    // [n_parts][kAttnTileRows][D] normalised partial outputs of cut tiles
  float* ws_lse;  // [n_parts][kAttnTileRows] their log-sum-exp (-inf: the row saw no key of the piece)
  const AttnMerge* merges;
  int32_t n_merges;
  int32_t block_keys;    // keys per LDS block of the bf16 kernel: 64 or 96
  const int32_t* q_rot;  // non-null: queries are rotated with row q_rot[r] of q_cos / q_sin on load
  const float* q_cos;
  const float* q_sin;
  int32_t interleaved;
  // lazy_rope contexts, fp32 kernel: source of every position and the rotary tables of the instances
  const int32_t* src_inst;
  const int32_t* src_row;
  const float* rope_cos;
  const float* rope_sin;
  int32_t ablate;  // probe builds only (kAblate*): parts of the bf16 kernel's inner loop that a timing run leaves out
};
// Timing-only variants of the bf16 attention kernel.  They exist only in the probe library
// (built with -DMPIC_PROBE_BUILD next to the product library, which has none of them) and
// compute nothing meaningful: each leaves one part of the inner loop out, with every access
// still in bounds, so that the cost of that part can be read off the difference in run time.
enum { kAblateLoads = 1,     // K/V blocks are staged only until every ring slot holds rows once
       kAblateLdsReads = 2,  // operand fragments are taken from registers instead of LDS
       kAblateSoftmax = 4,   // no exponentials, sums or conversions between the two products
       kAblateSameRows = 8,  // every block is staged from the rows of the tile's first block (the loads are issued, their
                             // data come from the nearest cache)
       kAblateNoLoadWaits = 32,    // no wait for staged blocks inside the loop (only with kAblateLdsReads)
       kAblateAddressesOnly = 64 };// the addresses of the direct loads are formed, the loads are not issued
constexpr int kProbeOptionAblate = 1000;  // mpic_set_option of the probe library: value = mask of kAblate*
// Contexts with lazy_rope: stored keys are never turned to their global position.  The kernel
// walks the request's key blocks (KeyBlock: all keys of a block come from consecutive rows of
// one source and lack the same shift) and turns its *queries* back by that shift whenever the
// source changes, <Rot(-s) q, k> = <q, Rot(s) k>.  Each block is staged from the base address of
// its source: the context buffers for fresh rows (and for stored rows that were copied there),
// or the chunk's cache itself when the caches are linked by reference.
struct LazyRefs {
  const KeyBlock* blocks;  // key blocks of the batch for this kernel's block size
  const int32_t* first;    // [B+1] first block of every request (its fresh blocks, then its stored blocks)
  const int32_t* mid;      // [B] first stored block of every request
  const int32_t* range;    // [n_tiles][4] attention kernel: fresh blocks [f0, f1) and stored blocks [s0, s1) of every tile
  const uint32_t* voff;    // [n_blocks][BN] row offsets (16-byte units) from the block's base
  const float* rope_cos;   // [n_inst][D/2] cos / sin of every instance's shift
  const float* rope_sin;
  int32_t by_ref;          // 0: every block is staged from the context buffers (the tables below are unused);
                           // 1: stored rows are read in their caches, at the addresses below
  int32_t pad;
  const void* k[kMaxInstPerLaunch];  // base of the rows of every chunk instance
  const void* v[kMaxInstPerLaunch];
};
// `next` / `next_tab` non-null: workgroups after the attention tiles link those rows (stored
// rows of the next layer's context; device-resident sources only, at most kMaxInstPerLaunch).
// `lazy` non-null: the lazy_rope kernel (a.tiles then counts in key blocks); not combined with `next`.
hipError_t launch_attn_bf16(const AttnArgs& a, const AssembleArgs* next, const AssembleSrcTable* next_tab,
                            const LazyRefs* lazy, hipStream_t stream);

// Keys of a decode split are a multiple of this (four wavefronts x 32-key blocks).
constexpr int kDecodeBlockKeys = 128;
struct DecodeArgs {
  const int32_t* ctx_off;
  const int32_t* dst_slot;
  const uint32_t* kv_off16;
  const void* q;
  const void* new_k;  // null: the new token does not attend to itself
  const void* new_v;
  const void* k_ctx;
  const void* v_ctx;
  void* out;
  float* lse;
  float* ws_o;    // [B][Hq][n_splits][D] normalised partial outputs
  float* ws_lse;  // [B][Hq][n_splits] their log-sum-exp
  float scale;
  int32_t n_q_heads, n_kv_heads, head_dim, n_requests;
  int32_t n_splits, keys_per_split;
  int32_t max_ctx;  // longest context of the batch
  // lazy_rope contexts: keys_per_split and max_ctx then count 32-key slots of the request's key
  // blocks (KeyBlock list for 32 keys); the fp32 kernel uses the per-position maps instead
  int32_t interleaved;
  const int32_t* blk_first;  // [B+1] first 32-key block of each request (bf16), null otherwise
  const int32_t* src_inst;
  const int32_t* src_row;
  const float* rope_cos;
  const float* rope_sin;
};
// `lazy` non-null: the lazy_rope kernels.
hipError_t launch_decode(int dtype, const DecodeArgs& a, const LazyRefs* lazy, hipStream_t stream);
// Device address and size of the file-scope scratch array of the decode kernels on the
// current GPU (looked up once per device; allocates nothing).
hipError_t decode_static_scratch(float** ptr, size_t* bytes);
// `lazy` non-null (lazy_rope contexts): stored keys are turned to their position as they are read.
hipError_t launch_attn_f32(const AttnArgs& a, int64_t n_q, const LazyRefs* lazy, hipStream_t stream);


// Can the attention launch of this plan carry the linking of the next layer (device-resident
// sources assumed)?  The trailing workgroups of 512 threads give every thread one unit pair of a row.
inline bool can_link_in_attention(const mpic_ctx* ctx, const mpic_plan* plan) {
  const int pairs_per_row = ctx->cfg.n_kv_heads * (ctx->cfg.head_dim / 16);
  return ctx->cfg.dtype == MPIC_BF16 && plan->inst_src.size() <= static_cast<size_t>(kMaxInstPerLaunch) &&
         !plan->tiles.empty() && pairs_per_row <= 512 && 512 % pairs_per_row == 0;
}
// ... and does it pay?  Yes when the linking is predicted to fit into the time the launch leaves
// idle (a 64-key block of a 256-row tile takes about 2.1 us; a linking launch of its own moves
// about 6 TB/s), and for short launches in any case: there the events of a two-stream schedule
// cost more than the linking itself (2.6K-token request: 59 us per layer against 100 us).
inline bool link_fits_attention_tail(const mpic_ctx* ctx, const mpic_plan* plan) {
  int64_t rows = 0;
  for (int32_t r : plan->inst_cached) rows += r;
  const double row_bytes = static_cast<double>(ctx->cfg.n_kv_heads) * ctx->cfg.head_dim * (ctx->cfg.dtype == MPIC_F32 ? 4 : 2);
  const double link_us = 4.0 * static_cast<double>(rows) * row_bytes / 6.0e6;
  const double idle_us = static_cast<double>(plan->est_idle_blocks) * 2.1 / 256.0;
  const double launch_us = static_cast<double>(plan->est_makespan_blocks) * 2.1;
  return link_us <= idle_us || launch_us < 500.0;
}

}  // namespace mpic

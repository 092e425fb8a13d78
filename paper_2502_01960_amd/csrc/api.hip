// GPU-facing entry points of libmpic: argument validation, device copies of the
// plan, the side-stream transfer of host-resident chunk caches (Sec. 3.2: transfer
// and linking proceed concurrently) and the kernel launches.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <string>

#include "common.h"

namespace mpic {

int bind_device(mpic_ctx* ctx) {
  int dev = -1;
  MPIC_HIP(ctx, hipGetDevice(&dev));
  if (ctx->device < 0) {
    ctx->device = dev;
    MPIC_HIP(ctx, hipStreamCreateWithFlags(&ctx->side_stream, hipStreamNonBlocking));
    MPIC_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_done[0], hipEventDisableTiming));
    MPIC_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_done[1], hipEventDisableTiming));
  } else if (ctx->device != dev) {
    return fail(ctx, MPIC_ERR_INVALID, "context is bound to another GPU than the current one");
  }
  return MPIC_OK;
}

namespace {

constexpr size_t kTablePad = 128;

// Copy the integer maps, rotary tables and tile list to the GPU (once per plan): the tables
// are packed into one host image that crosses the bus in a single copy into a single
// allocation.  May throw std::bad_alloc (host image); the entry points catch it.
int upload_plan(mpic_ctx* ctx, mpic_plan* p) {
  if (p->dev.block) {
    if (p->dev.device != ctx->device) return fail(ctx, MPIC_ERR_INVALID, "plan lives on another GPU");
    return MPIC_OK;
  }
  const size_t n = p->n_ctx, nq = p->n_q, B = p->n_requests;
  // byte offset of every context row in 16-byte units (saves the attention kernel a
  // 64-bit multiply per staged row); fits 32 bits for context buffers below 64 GiB
  const uint64_t units = static_cast<uint64_t>(ctx->cfg.n_kv_heads) * ctx->cfg.head_dim *
                         (ctx->cfg.dtype == MPIC_F32 ? 4 : 2) / 16;
  if (static_cast<uint64_t>(p->max_slot + 1) * units > 0xffffffffull)
    return fail(ctx, MPIC_ERR_UNSUPPORTED, "context buffers of 64 GiB or more are not supported");
  // kTablePad entries follow the table: the attention kernels fetch offsets eight at a
  // time and may run up to one key block past the last key of a tile.  They repeat the
  // last row of the batch, so that what is staged beyond a request's end is always a
  // linked row (its weight is zero, but 0 x NaN from an untouched slot would not be)
  std::vector<uint32_t> off(n + kTablePad, 0u);
  for (size_t i = 0; i < n; ++i) off[i] = static_cast<uint32_t>(static_cast<uint64_t>(p->dst_slot[i]) * units);
  for (size_t i = n; i < off.size() && n > 0; ++i) off[i] = off[n - 1];
  std::vector<int32_t> fp(nq);  // batch-flattened context position of every fresh row
  for (size_t r = 0; r < nq; ++r) fp[r] = p->ctx_off[p->q_req[r]] + p->q_pos[r];

  std::vector<char> image;
  auto put = [&](const void* src, size_t bytes) -> size_t {
    const size_t at = image.size();
    image.resize(at + (bytes + 255) / 256 * 256, 0);
    if (bytes) std::memcpy(image.data() + at, src, bytes);
    return at;
  };
  const size_t o_src_inst = put(p->src_inst.data(), n * 4);
  const size_t o_src_row = put(p->src_row.data(), n * 4);
  const size_t o_dst_slot = put(p->dst_slot.data(), n * 4);
  const size_t o_kv_off16 = put(off.data(), off.size() * 4);
  const size_t o_fresh_pos = put(fp.data(), nq * 4);
  const size_t o_q_pos = put(p->q_pos.data(), nq * 4);
  const size_t o_q_off = put(p->q_off.data(), (B + 1) * 4);
  const size_t o_ctx_off = put(p->ctx_off.data(), (B + 1) * 4);
  const size_t o_rope_cos = put(p->rope_cos.data(), p->rope_cos.size() * 4);
  const size_t o_rope_sin = put(p->rope_sin.data(), p->rope_sin.size() * 4);
  const size_t o_fresh_rot = put(p->fresh_rot.data(), p->fresh_rot.size() * 4);
  const size_t o_fresh_cos = put(p->fresh_cos.data(), p->fresh_cos.size() * 4);
  const size_t o_fresh_sin = put(p->fresh_sin.data(), p->fresh_sin.size() * 4);
  const size_t o_tiles = put(p->tiles.data(), p->tiles.size() * sizeof(AttnTile));
  const size_t o_merges = put(p->merges.data(), p->merges.size() * sizeof(AttnMerge));
  // lazy_rope contexts: key blocks, their row-offset tables in both views, tiles in block indices
  size_t o_kblk[kNumBlockSizes] = {}, o_first[kNumBlockSizes] = {}, o_mid[kNumBlockSizes] = {}, o_vctx[kNumBlockSizes] = {},
         o_vref[kNumBlockSizes] = {}, o_range[kNumBlockSizes] = {};
  const bool lazy = ctx->cfg.lazy_rope != 0;
  if (lazy) {
    for (int s = 0; s < kNumBlockSizes; ++s) {
      const size_t bn = kBlockSizes[s];
      const std::vector<KeyBlock>& blocks = p->kblk[s];
      // slots past n_valid repeat the block's last row: what is staged there is masked, but it
      // must be a row that exists (in-place reads must stay inside their source)
      std::vector<uint32_t> vctx(blocks.size() * bn + kTablePad, 0u), vref(vctx.size(), 0u);
      for (size_t t = 0; t < blocks.size(); ++t) {
        const KeyBlock& kb = blocks[t];
        const size_t ctx0 = p->ctx_off[kb.req];
        for (size_t i = 0; i < bn; ++i) {
          const size_t pos = ctx0 + kb.pos0 + std::min<size_t>(i, kb.n_valid - 1);
          vctx[t * bn + i] = off[pos];
          vref[t * bn + i] = kb.inst < 0 ? off[pos] : static_cast<uint32_t>(static_cast<uint64_t>(p->src_row[pos]) * units);
        }
      }
      o_kblk[s] = put(blocks.data(), blocks.size() * sizeof(KeyBlock));
      o_first[s] = put(p->kblk_first[s].data(), p->kblk_first[s].size() * 4);
      o_vctx[s] = put(vctx.data(), vctx.size() * 4);
      o_vref[s] = put(vref.data(), vref.size() * 4);
      o_mid[s] = put(p->kblk_mid[s].data(), p->kblk_mid[s].size() * 4);
      o_range[s] = put(p->lazy_range[s].data(), p->lazy_range[s].size() * 4);
    }
  }
  image.resize(image.size() + 256, 0);

  char* base = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&base), image.size()) != hipSuccess) {
    (void)hipGetLastError();
    return fail(ctx, MPIC_ERR_OOM, "device allocation of the plan failed");
  }
  const hipError_t e = hipMemcpy(base, image.data(), image.size(), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(base);
    return fail_hip(ctx, e, "upload of the plan");
  }
  PlanDevice d;
  d.src_inst = reinterpret_cast<int32_t*>(base + o_src_inst);
  d.src_row = reinterpret_cast<int32_t*>(base + o_src_row);
  d.dst_slot = reinterpret_cast<int32_t*>(base + o_dst_slot);
  d.kv_off16 = reinterpret_cast<uint32_t*>(base + o_kv_off16);
  d.fresh_pos = reinterpret_cast<int32_t*>(base + o_fresh_pos);
  d.q_pos = reinterpret_cast<int32_t*>(base + o_q_pos);
  d.q_off = reinterpret_cast<int32_t*>(base + o_q_off);
  d.ctx_off = reinterpret_cast<int32_t*>(base + o_ctx_off);
  d.rope_cos = reinterpret_cast<float*>(base + o_rope_cos);
  d.rope_sin = reinterpret_cast<float*>(base + o_rope_sin);
  if (!p->fresh_rot.empty()) {  // null pointers tell the kernels that fresh rows arrive rotated
    d.fresh_rot = reinterpret_cast<int32_t*>(base + o_fresh_rot);
    d.fresh_cos = reinterpret_cast<float*>(base + o_fresh_cos);
    d.fresh_sin = reinterpret_cast<float*>(base + o_fresh_sin);
  }
  d.tiles = reinterpret_cast<AttnTile*>(base + o_tiles);
  d.merges = reinterpret_cast<AttnMerge*>(base + o_merges);
  if (lazy) {
    for (int s = 0; s < kNumBlockSizes; ++s) {
      d.kblk[s] = reinterpret_cast<KeyBlock*>(base + o_kblk[s]);
      d.kblk_first[s] = reinterpret_cast<int32_t*>(base + o_first[s]);
      d.voff_ctx[s] = reinterpret_cast<uint32_t*>(base + o_vctx[s]);
      d.voff_ref[s] = reinterpret_cast<uint32_t*>(base + o_vref[s]);
      d.kblk_mid[s] = reinterpret_cast<int32_t*>(base + o_mid[s]);
      d.lazy_range[s] = reinterpret_cast<int32_t*>(base + o_range[s]);
    }
  }
  d.block = base;
  d.device = ctx->device;
  p->dev = d;
  return MPIC_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// lazy_rope contexts: what the kernels need to walk the plan's key blocks of `bn` keys.  With
// `refs` the stored rows are read in place in the chunk caches (validated here), else in the
// context buffers, where mpic_assemble_kv copied them unrotated.
int fill_lazy_refs(mpic_ctx* ctx, const mpic_plan* plan, int bn, const SrcRefs* refs, const char* who, LazyRefs* out) {
  const int s = block_size_index(bn);
  LazyRefs r{};
  r.blocks = plan->dev.kblk[s];
  r.first = plan->dev.kblk_first[s];
  r.mid = plan->dev.kblk_mid[s];
  r.range = plan->dev.lazy_range[s];
  r.voff = refs ? plan->dev.voff_ref[s] : plan->dev.voff_ctx[s];
  r.rope_cos = plan->dev.rope_cos;
  r.rope_sin = plan->dev.rope_sin;
  r.by_ref = refs ? 1 : 0;
  if (refs) {
    const size_t n_inst = plan->inst_src.size();
    if (n_inst > static_cast<size_t>(kMaxInstPerLaunch))
      return fail(ctx, MPIC_ERR_UNSUPPORTED, std::string(who) + ": more than 128 chunk instances cannot be read in place");
    if (n_inst > 0 && (!refs->srcs || refs->n_srcs <= plan->max_src))
      return fail(ctx, MPIC_ERR_INVALID, std::string(who) + ": srcs does not cover every chunk index of the plan");
    for (size_t i = 0; i < n_inst; ++i) {
      const mpic_chunk_src& sc = refs->srcs[plan->inst_src[i]];
      if (sc.len != plan->inst_len[i]) return fail(ctx, MPIC_ERR_INVALID, std::string(who) + ": chunk source length differs from its segment");
      if (plan->inst_cached[i] > 0) {
        if (sc.on_host != MPIC_SRC_DEVICE) return fail(ctx, MPIC_ERR_INVALID, std::string(who) + ": a cache that is read in place must be in device memory");
        if (!sc.k || !sc.v || !aligned16(sc.k) || !aligned16(sc.v))
          return fail(ctx, MPIC_ERR_INVALID, std::string(who) + ": chunk source pointer missing or not 16-byte aligned");
      }
      r.k[i] = sc.k;
      r.v[i] = sc.v;
    }
  }
  *out = r;
  return MPIC_OK;
}

}  // namespace
}  // namespace mpic

using mpic::fail;

extern "C" void mpic_destroy(mpic_ctx* ctx) {
  if (!ctx) return;
  if (ctx->device >= 0) {
    int cur = -1;
    (void)hipGetDevice(&cur);
    (void)hipSetDevice(ctx->device);
    if (ctx->side_stream) {
      (void)hipStreamSynchronize(ctx->side_stream);
      (void)hipStreamDestroy(ctx->side_stream);
    }
    if (ctx->link_stream) {
      (void)hipStreamSynchronize(ctx->link_stream);
      (void)hipStreamDestroy(ctx->link_stream);
    }
    for (hipEvent_t ev : ctx->ev_layer) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : ctx->ev_done)
      if (ev) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : ctx->ev_copy) (void)hipEventDestroy(ev);
    for (void* buf : ctx->staging)
      if (buf) (void)hipFree(buf);
    if (ctx->decode_ws) (void)hipFree(ctx->decode_ws);
    if (ctx->attn_ws) (void)hipFree(ctx->attn_ws);
    if (cur >= 0) (void)hipSetDevice(cur);
  }
  delete ctx;
}

extern "C" void mpic_plan_destroy(mpic_plan* plan) {
  if (!plan) return;
  if (plan->dev.block) {
    int cur = -1;
    (void)hipGetDevice(&cur);
    (void)hipSetDevice(plan->dev.device);
    (void)hipFree(plan->dev.block);
    if (cur >= 0) (void)hipSetDevice(cur);
  }
  delete plan;
}

extern "C" int mpic_assemble_kv(mpic_ctx* ctx, mpic_plan* plan, const mpic_chunk_src* srcs,
                                int32_t n_srcs, const void* fresh_k, const void* fresh_v,
                                int64_t n_fresh_rows, void* k_ctx, void* v_ctx, int64_t n_ctx_slots,
                                void* stream_) {
  return mpic_assemble_kv_parts(ctx, plan, srcs, n_srcs, fresh_k, fresh_v, n_fresh_rows, k_ctx, v_ctx,
                                n_ctx_slots, MPIC_PART_CACHED | MPIC_PART_FRESH, stream_);
}

int mpic::assemble_parts(mpic_ctx* ctx, mpic_plan* plan, const mpic_chunk_src* srcs,
                                  int32_t n_srcs, const void* fresh_k, const void* fresh_v,
                                  int64_t n_fresh_rows, void* k_ctx, void* v_ctx,
                                  int64_t n_ctx_slots, uint32_t parts, void* stream_) {
  if (!ctx) return MPIC_ERR_INVALID;
  const bool background = parts & MPIC_PART_BACKGROUND;
  if (background) ctx->background_seen = true;
  parts &= ~static_cast<uint32_t>(MPIC_PART_BACKGROUND);
  if (parts == 0 || (parts & ~static_cast<uint32_t>(MPIC_PART_CACHED | MPIC_PART_FRESH)))
    return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: parts must be MPIC_PART_CACHED, MPIC_PART_FRESH or both");
  const bool do_cached = parts & MPIC_PART_CACHED, do_fresh = parts & MPIC_PART_FRESH;
  if (!plan || plan->ctx != ctx) return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: plan does not belong to this context");
  if (do_fresh && n_fresh_rows != plan->n_q) return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: n_fresh_rows differs from the plan's recompute set");
  if (do_fresh && plan->n_q > 0 && (!fresh_k || !fresh_v)) return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: fresh_k / fresh_v missing");
  if (plan->n_ctx == 0) return MPIC_OK;
  if (!k_ctx || !v_ctx) return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: k_ctx / v_ctx missing");
  if (n_ctx_slots <= plan->max_slot) return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: context buffers smaller than the plan's largest slot");
  if ((do_fresh && (!mpic::aligned16(fresh_k) || !mpic::aligned16(fresh_v))) || !mpic::aligned16(k_ctx) || !mpic::aligned16(v_ctx))
    return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: buffers must be 16-byte aligned");
  const size_t n_inst = do_cached ? plan->inst_src.size() : 0;  // chunk sources are only looked at for the cached part
  if (n_inst > 0 && (!srcs || n_srcs <= plan->max_src)) return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: srcs does not cover every chunk index of the plan");
  bool any_host = false, any_mapped = false;
  for (size_t i = 0; i < n_inst; ++i) {
    const mpic_chunk_src& s = srcs[plan->inst_src[i]];
    if (s.len != plan->inst_len[i]) return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: chunk source length differs from its segment");
    if (s.on_host < MPIC_SRC_DEVICE || s.on_host > MPIC_SRC_HOST_MAPPED) return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: unknown on_host value");
    if (plan->inst_cached[i] > 0) {  // some rows are actually read
      if (!s.k || !s.v || !mpic::aligned16(s.k) || !mpic::aligned16(s.v))
        return fail(ctx, MPIC_ERR_INVALID, "assemble_kv: chunk source pointer missing or not 16-byte aligned");
      any_host = any_host || s.on_host == MPIC_SRC_HOST_STAGED;
      any_mapped = any_mapped || s.on_host == MPIC_SRC_HOST_MAPPED;
    }
  }
  if (any_mapped) ctx->background_seen = true;  // a launch that lasts as long as the transfer runs beside others
  int rc = mpic::bind_device(ctx);
  if (rc != MPIC_OK) return rc;
  rc = mpic::upload_plan(ctx, plan);
  if (rc != MPIC_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const mpic_config& c = ctx->cfg;
  const size_t elem = c.dtype == MPIC_F32 ? 4 : 2;
  const size_t row_bytes = static_cast<size_t>(c.n_kv_heads) * c.head_dim * elem;

  // ---- host-resident sources: where each lands in device staging ----
  // Only rows that some instance actually reuses cross the bus: rows below the smallest
  // effective k of the source's instances are replaced by fresh rows anyway.
  constexpr int kGroup = 4;  // sources per transfer group (one event each)
  std::vector<int32_t> host_srcs;              // distinct host sources in order of first use
  std::vector<size_t> stage_off(n_srcs > 0 ? n_srcs : 0, SIZE_MAX);
  std::vector<int32_t> first_row(n_srcs > 0 ? n_srcs : 0, INT32_MAX);
  size_t need = 0;
  char* staging = nullptr;
  int buf = 0;
  if (any_host) {
    for (size_t i = 0; i < n_inst; ++i) {
      const int32_t s = plan->inst_src[i];
      if (srcs[s].on_host == MPIC_SRC_HOST_STAGED && plan->inst_cached[i] > 0)
        first_row[s] = std::min(first_row[s], plan->inst_k[i]);
    }
    for (size_t i = 0; i < n_inst; ++i) {
      const int32_t s = plan->inst_src[i];
      if (srcs[s].on_host == MPIC_SRC_HOST_STAGED && plan->inst_cached[i] > 0 && stage_off[s] == SIZE_MAX) {
        stage_off[s] = need;  // room for the whole chunk keeps row addressing trivial
        need += 2 * static_cast<size_t>(srcs[s].len) * row_bytes;
        host_srcs.push_back(s);
      }
    }
    buf = ctx->next_staging;
    ctx->next_staging ^= 1;
    if (need > ctx->staging_bytes[buf]) {
      // growing a staging area is rare (first calls / larger batch): drain and reallocate
      MPIC_HIP(ctx, hipStreamSynchronize(ctx->side_stream));
      MPIC_HIP(ctx, hipStreamSynchronize(stream));
      if (ctx->ev_done_valid[buf]) MPIC_HIP(ctx, hipEventSynchronize(ctx->ev_done[buf]));
      if (ctx->staging[buf]) MPIC_HIP(ctx, hipFree(ctx->staging[buf]));
      ctx->staging[buf] = nullptr;
      ctx->staging_bytes[buf] = 0;
      hipError_t e = hipMalloc(&ctx->staging[buf], need);
      if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, MPIC_ERR_OOM, "assemble_kv: device staging allocation failed");
      }
      ctx->staging_bytes[buf] = need;
    }
    staging = static_cast<char*>(ctx->staging[buf]);
    const size_t n_groups = (host_srcs.size() + kGroup - 1) / kGroup;
    while (ctx->ev_copy.size() < n_groups) {
      hipEvent_t ev;
      MPIC_HIP(ctx, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
      ctx->ev_copy.push_back(ev);
    }
    // this staging buffer may still be read by the linking kernels of the call before last
    if (ctx->ev_done_valid[buf]) MPIC_HIP(ctx, hipStreamWaitEvent(ctx->side_stream, ctx->ev_done[buf], 0));
    for (size_t i = 0; i < host_srcs.size(); ++i) {
      const int32_t si = host_srcs[i];
      const mpic_chunk_src& s = srcs[si];
      const size_t skip = static_cast<size_t>(first_row[si]) * row_bytes;
      const size_t bytes = static_cast<size_t>(s.len) * row_bytes;
      char* dst = staging + stage_off[si];
      if (static_cast<const char*>(s.v) == static_cast<const char*>(s.k) + bytes) {
        // keys and values lie back to back (the layout of the cache library): one transfer,
        // the skipped head of V rides along
        MPIC_HIP(ctx, hipMemcpyAsync(dst + skip, static_cast<const char*>(s.k) + skip, 2 * bytes - skip,
                                     hipMemcpyHostToDevice, ctx->side_stream));
      } else {
        MPIC_HIP(ctx, hipMemcpyAsync(dst + skip, static_cast<const char*>(s.k) + skip, bytes - skip,
                                     hipMemcpyHostToDevice, ctx->side_stream));
        MPIC_HIP(ctx, hipMemcpyAsync(dst + bytes + skip, static_cast<const char*>(s.v) + skip, bytes - skip,
                                     hipMemcpyHostToDevice, ctx->side_stream));
      }
      if ((i + 1) % kGroup == 0 || i + 1 == host_srcs.size())
        MPIC_HIP(ctx, hipEventRecord(ctx->ev_copy[i / kGroup], ctx->side_stream));
    }
  }

  mpic::AssembleArgs a{};
  a.src_inst = plan->dev.src_inst;
  a.src_row = plan->dev.src_row;
  a.dst_slot = plan->dev.dst_slot;
  // (lazy_rope: stored keys are copied as stored, the shift is applied on the query side)
  a.rope_cos = ctx->cfg.lazy_rope ? nullptr : plan->dev.rope_cos;
  a.rope_sin = ctx->cfg.lazy_rope ? nullptr : plan->dev.rope_sin;
  a.fresh_rot = plan->dev.fresh_rot;
  a.fresh_cos = plan->dev.fresh_cos;
  a.fresh_sin = plan->dev.fresh_sin;
  a.fresh_k = fresh_k;
  a.fresh_v = fresh_v;
  a.k_ctx = k_ctx;
  a.v_ctx = v_ctx;
  a.n_kv_heads = c.n_kv_heads;
  a.head_dim = c.head_dim;
  a.interleaved = c.rope_interleaved;

  if (!do_cached) {
    // fresh rows only: one launch over the list of their positions
    mpic::AssembleSrcTable none{};
    a.pos_list = plan->dev.fresh_pos;
    a.pos_begin = 0;
    a.pos_end = plan->n_q;
    a.inst_base = 0;
    a.n_inst = 0;
    a.skip_fresh = 0;
    MPIC_HIP(ctx, mpic::launch_assemble(c.dtype, a, none, stream));
    return MPIC_OK;
  }
  auto inst_first_pos = [&](size_t i) -> int64_t {
    return static_cast<int64_t>(plan->ctx_off[plan->inst_req[i]]) + plan->inst_delta[i];
  };
  // Pass 1: fresh rows and device-resident chunks, at most kMaxInstPerLaunch instances per
  // launch (their source pointers travel as kernel arguments).  Host-resident instances
  // have a null entry and are skipped here.
  for (size_t i0 = 0; i0 == 0 || i0 < n_inst; i0 += mpic::kMaxInstPerLaunch) {
    const size_t i1 = std::min(n_inst, i0 + mpic::kMaxInstPerLaunch);
    mpic::AssembleSrcTable tab{};
    for (size_t i = i0; i < i1; ++i) {
      const mpic_chunk_src& s = srcs[plan->inst_src[i]];
      const bool deferred = s.on_host == MPIC_SRC_HOST_STAGED && plan->inst_cached[i] > 0;
      tab.k[i - i0] = deferred ? nullptr : s.k;
      tab.v[i - i0] = deferred ? nullptr : s.v;
    }
    a.pos_begin = i0 == 0 ? 0 : inst_first_pos(i0);
    a.pos_end = i1 < n_inst ? inst_first_pos(i1) : plan->n_ctx;
    a.inst_base = static_cast<int32_t>(i0);
    a.n_inst = static_cast<int32_t>(i1 - i0);
    a.skip_fresh = do_fresh ? 0 : 1;
    // Launches meant to run beside other work are held to a small grid that strides.
    // Chunks read in place over the bus: 64 workgroups keep the bus busy (52 GB/s measured)
    // and leave the wave slots and registers of the chip to a concurrent kernel; with 128 or
    // more the attention of the previous layer no longer overlaps (measured: 3.3 ms per step
    // at 128, 2.8 ms at 64, 2.9 ms at 16).  Background linking from device memory: one
    // workgroup per 5 MB of traffic, at least 64, so that the launch lasts about a quarter of
    // a millisecond alone whatever the batch (18K-token batch of 4, 325 MB: whole step 1.151 ms
    // at 64, 1.159 at 256, 1.179 unlimited; a batch whose linking moves 1.1 GB would make a
    // 64-workgroup launch the bottleneck of a 1.1 ms step).
    if (any_mapped) {
      a.grid_limit = 64;
    } else if (background) {
      const int64_t bytes = 4 * (a.pos_end - a.pos_begin) * static_cast<int64_t>(row_bytes);
      a.grid_limit = static_cast<int32_t>(std::max<int64_t>(64, bytes / (5 << 20)));
    } else {
      a.grid_limit = 0;
    }
    MPIC_HIP(ctx, mpic::launch_assemble(c.dtype, a, tab, stream));
  }
  a.grid_limit = 0;
  // Pass 2: one launch per chunk instance fed from staging, as soon as its transfer group
  // has landed.  Only that instance's rows are touched.
  if (any_host) {
    std::vector<int32_t> group_of(n_srcs, -1);
    for (size_t i = 0; i < host_srcs.size(); ++i) group_of[host_srcs[i]] = static_cast<int32_t>(i / kGroup);
    // instances ordered by the transfer group of their source
    std::vector<size_t> order;
    for (size_t i = 0; i < n_inst; ++i) {
      const int32_t s = plan->inst_src[i];
      if (srcs[s].on_host == MPIC_SRC_HOST_STAGED && plan->inst_cached[i] > 0) order.push_back(i);
    }
    std::stable_sort(order.begin(), order.end(), [&](size_t x, size_t y) {
      return group_of[plan->inst_src[x]] < group_of[plan->inst_src[y]];
    });
    int32_t waited = -1;
    for (size_t i : order) {
      const int32_t s = plan->inst_src[i];
      if (group_of[s] > waited) {
        waited = group_of[s];
        MPIC_HIP(ctx, hipStreamWaitEvent(stream, ctx->ev_copy[waited], 0));
      }
      mpic::AssembleSrcTable tab{};
      const size_t bytes = static_cast<size_t>(srcs[s].len) * row_bytes;
      tab.k[0] = staging + stage_off[s];
      tab.v[0] = staging + stage_off[s] + bytes;
      a.pos_begin = inst_first_pos(i) + plan->inst_k[i];
      a.pos_end = inst_first_pos(i) + plan->inst_len[i];
      a.inst_base = static_cast<int32_t>(i);
      a.n_inst = 1;
      a.skip_fresh = 1;
      MPIC_HIP(ctx, mpic::launch_assemble(c.dtype, a, tab, stream));
    }
    MPIC_HIP(ctx, hipEventRecord(ctx->ev_done[buf], stream));
    ctx->ev_done_valid[buf] = true;
  }
  return MPIC_OK;
}

int mpic::attend(mpic_ctx* ctx, mpic_plan* plan, const void* fresh_q,
                               int64_t n_fresh_rows, const void* k_ctx, const void* v_ctx,
                               int64_t n_ctx_slots, double softmax_scale, void* out, float* lse,
                               void* stream_, const mpic::NextLink* next, int32_t block_keys, const mpic::SrcRefs* refs) {
  if (!ctx) return MPIC_ERR_INVALID;
  const bool lazy = ctx->cfg.lazy_rope != 0;
  if (refs && !lazy) return fail(ctx, MPIC_ERR_INVALID, "selective_attn_in_place: the context was not created with lazy_rope");
  if (!plan || plan->ctx != ctx) return fail(ctx, MPIC_ERR_INVALID, "selective_attn: plan does not belong to this context");
  if (n_fresh_rows != plan->n_q) return fail(ctx, MPIC_ERR_INVALID, "selective_attn: n_fresh_rows differs from the plan's recompute set");
  if (!(softmax_scale > 0.0) || !std::isfinite(softmax_scale)) return fail(ctx, MPIC_ERR_INVALID, "selective_attn: softmax_scale must be finite and positive");
  if (plan->n_q == 0) {
    if (next)  // no attention to ride along with
      return mpic::assemble_parts(ctx, plan, next->srcs, next->n_srcs, nullptr, nullptr, 0, next->k_ctx, next->v_ctx,
                                  n_ctx_slots, MPIC_PART_CACHED, stream_);
    return MPIC_OK;
  }
  if (!fresh_q || !k_ctx || !v_ctx || !out) return fail(ctx, MPIC_ERR_INVALID, "selective_attn: null buffer");
  if (n_ctx_slots <= plan->max_slot) return fail(ctx, MPIC_ERR_INVALID, "selective_attn: context buffers smaller than the plan's largest slot");
  if (!mpic::aligned16(fresh_q) || !mpic::aligned16(k_ctx) || !mpic::aligned16(v_ctx) || !mpic::aligned16(out))
    return fail(ctx, MPIC_ERR_INVALID, "selective_attn: buffers must be 16-byte aligned");
  bool fuse_next = false;
  if (next) {
    // the stored rows of the next layer, linked by the same launch when the sources allow it
    const size_t n_inst = plan->inst_src.size();
    if (!next->k_ctx || !next->v_ctx || !mpic::aligned16(next->k_ctx) || !mpic::aligned16(next->v_ctx))
      return fail(ctx, MPIC_ERR_INVALID, "selective_attn: next layer's context buffers missing or not 16-byte aligned");
    const size_t bytes = static_cast<size_t>(n_ctx_slots) * ctx->cfg.n_kv_heads * ctx->cfg.head_dim * (ctx->cfg.dtype == MPIC_F32 ? 4 : 2);
    auto overlap = [&](const void* x, const void* y) {
      const char* a0 = static_cast<const char*>(x);
      const char* b0 = static_cast<const char*>(y);
      return a0 < b0 + bytes && b0 < a0 + bytes;
    };
    if (overlap(next->k_ctx, k_ctx) || overlap(next->k_ctx, v_ctx) || overlap(next->v_ctx, k_ctx) || overlap(next->v_ctx, v_ctx))
      return fail(ctx, MPIC_ERR_INVALID, "selective_attn: the next layer's context must not overlap the one being read");
    if (n_inst > 0 && (!next->srcs || next->n_srcs <= plan->max_src))
      return fail(ctx, MPIC_ERR_INVALID, "selective_attn: next layer's srcs does not cover every chunk index of the plan");
    fuse_next = mpic::can_link_in_attention(ctx, plan) && !lazy;  // (the lazy kernel carries no linking)
    for (size_t i = 0; i < n_inst; ++i) {
      const mpic_chunk_src& sc = next->srcs[plan->inst_src[i]];
      if (sc.len != plan->inst_len[i]) return fail(ctx, MPIC_ERR_INVALID, "selective_attn: next layer's chunk source length differs from its segment");
      if (sc.on_host < MPIC_SRC_DEVICE || sc.on_host > MPIC_SRC_HOST_MAPPED) return fail(ctx, MPIC_ERR_INVALID, "selective_attn: unknown on_host value");
      if (plan->inst_cached[i] > 0) {
        if (!sc.k || !sc.v || !mpic::aligned16(sc.k) || !mpic::aligned16(sc.v))
          return fail(ctx, MPIC_ERR_INVALID, "selective_attn: next layer's chunk source pointer missing or not 16-byte aligned");
        if (sc.on_host != MPIC_SRC_DEVICE) fuse_next = false;  // host memory: the separate, slower launch
      }
    }
  }
  int rc = mpic::bind_device(ctx);
  if (rc != MPIC_OK) return rc;
  rc = mpic::upload_plan(ctx, plan);
  if (rc != MPIC_OK) return rc;
  const mpic_config& c = ctx->cfg;
  mpic::AttnArgs a{};
  a.tiles = plan->dev.tiles;
  a.n_tiles = static_cast<int32_t>(plan->tiles.size());
  a.q_pos = plan->dev.q_pos;
  a.q_off = plan->dev.q_off;
  a.ctx_off = plan->dev.ctx_off;
  a.dst_slot = plan->dev.dst_slot;
  a.kv_off16 = plan->dev.kv_off16;
  a.q = fresh_q;
  a.k_ctx = k_ctx;
  a.v_ctx = v_ctx;
  a.out = out;
  a.lse = lse;
  a.scale = static_cast<float>(softmax_scale);
  a.n_q_heads = c.n_q_heads;
  a.n_kv_heads = c.n_kv_heads;
  a.head_dim = c.head_dim;
  a.n_requests = plan->n_requests;
  if (c.dtype == MPIC_BF16 && plan->n_parts > 0) {
    const size_t slots = static_cast<size_t>(plan->n_parts) * mpic::kAttnTileRows;
    const size_t need = slots * (c.head_dim + 1) * sizeof(float);
    if (need > ctx->attn_ws_bytes) {
      // growing the workspace is rare (first call / larger batch): drain what may still read it
      MPIC_HIP(ctx, hipDeviceSynchronize());
      if (ctx->attn_ws) MPIC_HIP(ctx, hipFree(ctx->attn_ws));
      ctx->attn_ws = nullptr;
      ctx->attn_ws_bytes = 0;
      if (hipMalloc(&ctx->attn_ws, need) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, MPIC_ERR_OOM, "selective_attn: workspace allocation failed");
      }
      ctx->attn_ws_bytes = need;
    }
    a.ws_o = static_cast<float*>(ctx->attn_ws);
    a.ws_lse = a.ws_o + slots * c.head_dim;
    a.merges = plan->dev.merges;
    a.n_merges = static_cast<int32_t>(plan->merges.size());
  }
  a.block_keys = block_keys ? block_keys : ctx->attn_block_keys ? ctx->attn_block_keys : ctx->background_seen ? 64 : 96;
  a.q_rot = plan->dev.fresh_rot;
  a.q_cos = plan->dev.fresh_cos;
  a.q_sin = plan->dev.fresh_sin;
  a.interleaved = c.rope_interleaved;
  a.ablate = ctx->attn_ablate;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (lazy) {
    mpic::LazyRefs lr;
    rc = mpic::fill_lazy_refs(ctx, plan, c.dtype == MPIC_F32 ? 32 : a.block_keys, refs, "selective_attn", &lr);
    if (rc != MPIC_OK) return rc;
    if (c.dtype == MPIC_F32) {
      a.src_inst = plan->dev.src_inst;
      a.src_row = plan->dev.src_row;
      a.rope_cos = plan->dev.rope_cos;
      a.rope_sin = plan->dev.rope_sin;
      MPIC_HIP(ctx, mpic::launch_attn_f32(a, plan->n_q, &lr, stream));
    } else {
      MPIC_HIP(ctx, mpic::launch_attn_bf16(a, nullptr, nullptr, &lr, stream));
    }
    if (next)
      return mpic::assemble_parts(ctx, plan, next->srcs, next->n_srcs, nullptr, nullptr, 0, next->k_ctx, next->v_ctx,
                                  n_ctx_slots, MPIC_PART_CACHED, stream_);
    return MPIC_OK;
  }
  if (fuse_next) {
    mpic::AssembleArgs la{};
    la.src_inst = plan->dev.src_inst;
    la.src_row = plan->dev.src_row;
    la.dst_slot = plan->dev.dst_slot;
    la.rope_cos = plan->dev.rope_cos;
    la.rope_sin = plan->dev.rope_sin;
    la.k_ctx = next->k_ctx;
    la.v_ctx = next->v_ctx;
    la.pos_begin = 0;
    la.pos_end = plan->n_ctx;
    la.inst_base = 0;
    la.n_inst = static_cast<int32_t>(plan->inst_src.size());
    la.n_kv_heads = c.n_kv_heads;
    la.head_dim = c.head_dim;
    la.interleaved = c.rope_interleaved;
    la.skip_fresh = 1;
    mpic::AssembleSrcTable tab{};
    for (size_t i = 0; i < plan->inst_src.size(); ++i) {
      tab.k[i] = next->srcs[plan->inst_src[i]].k;
      tab.v[i] = next->srcs[plan->inst_src[i]].v;
    }
    MPIC_HIP(ctx, mpic::launch_attn_bf16(a, &la, &tab, nullptr, stream));
    return MPIC_OK;
  }
  if (c.dtype == MPIC_F32) {
    MPIC_HIP(ctx, mpic::launch_attn_f32(a, plan->n_q, nullptr, stream));
  } else {
    MPIC_HIP(ctx, mpic::launch_attn_bf16(a, nullptr, nullptr, nullptr, stream));
  }
  if (next)  // same result, one launch more
    return mpic::assemble_parts(ctx, plan, next->srcs, next->n_srcs, nullptr, nullptr, 0, next->k_ctx, next->v_ctx,
                                n_ctx_slots, MPIC_PART_CACHED, stream_);
  return MPIC_OK;
}

// static_scratch: the partial results go to the library's file-scope device array instead of
// the context's workspace, and the call allocates nothing (it then needs a context and a plan
// that an earlier call has already brought to the GPU).
static int decode_attn_impl(mpic_ctx* ctx, mpic_plan* plan, const void* q, const void* new_k,
                            const void* new_v, const void* k_ctx, const void* v_ctx,
                            int64_t n_ctx_slots, double softmax_scale, void* out, float* lse,
                            void* stream_, bool static_scratch, const mpic::SrcRefs* refs = nullptr) {
  if (!ctx) return MPIC_ERR_INVALID;
  const bool lazy = ctx->cfg.lazy_rope != 0;
  if (refs && !lazy) return fail(ctx, MPIC_ERR_INVALID, "decode_attn_in_place: the context was not created with lazy_rope");
  if (!plan || plan->ctx != ctx) return fail(ctx, MPIC_ERR_INVALID, "decode_attn: plan does not belong to this context");
  if (!(softmax_scale > 0.0) || !std::isfinite(softmax_scale)) return fail(ctx, MPIC_ERR_INVALID, "decode_attn: softmax_scale must be finite and positive");
  if (!q || !out) return fail(ctx, MPIC_ERR_INVALID, "decode_attn: null buffer");
  if ((new_k == nullptr) != (new_v == nullptr)) return fail(ctx, MPIC_ERR_INVALID, "decode_attn: new_k and new_v go together");
  if (plan->n_ctx > 0 && (!k_ctx || !v_ctx)) return fail(ctx, MPIC_ERR_INVALID, "decode_attn: k_ctx / v_ctx missing");
  if (plan->n_ctx > 0 && n_ctx_slots <= plan->max_slot) return fail(ctx, MPIC_ERR_INVALID, "decode_attn: context buffers smaller than the plan's largest slot");
  if (!mpic::aligned16(q) || !mpic::aligned16(out) || !mpic::aligned16(k_ctx) || !mpic::aligned16(v_ctx) ||
      !mpic::aligned16(new_k) || !mpic::aligned16(new_v))
    return fail(ctx, MPIC_ERR_INVALID, "decode_attn: buffers must be 16-byte aligned");
  int rc = MPIC_OK;
  if (static_scratch) {
    int dev = -1;
    MPIC_HIP(ctx, hipGetDevice(&dev));
    if (ctx->device < 0 || !plan->dev.block)
      return fail(ctx, MPIC_ERR_INVALID, "decode_attn_static: the plan is not on the GPU yet (an earlier call with this plan, "
                                         "e.g. mpic_assemble_kv, uploads it)");
    if (ctx->device != dev || plan->dev.device != dev)
      return fail(ctx, MPIC_ERR_INVALID, "decode_attn_static: context and plan live on another GPU than the current one");
  } else {
    rc = mpic::bind_device(ctx);
    if (rc != MPIC_OK) return rc;
    rc = mpic::upload_plan(ctx, plan);
    if (rc != MPIC_OK) return rc;
  }
  const mpic_config& c = ctx->cfg;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  // longest context of the batch; lazy_rope (bf16): in slots of the requests' 32-key blocks
  const bool by_blocks = lazy && c.dtype == MPIC_BF16;
  int32_t max_ctx = 0;
  for (int b = 0; b < plan->n_requests; ++b)
    max_ctx = std::max(max_ctx, by_blocks ? (plan->kblk_first[0][b + 1] - plan->kblk_first[0][b]) * 32
                                          : plan->ctx_off[b + 1] - plan->ctx_off[b]);
  // Splits: a workgroup fills a compute unit's LDS, so the keys are cut so that one round of
  // workgroups covers the chip (fewer when the batch alone supplies that many); each split
  // is a multiple of 128 keys.
  int32_t n_splits = 1, keys_per_split = std::max(max_ctx, 1);
  if (c.dtype == MPIC_BF16 && max_ctx > 0) {
    constexpr int64_t kTargetWorkgroups = 256;  // one round over the compute units
    const int64_t lanes = static_cast<int64_t>(plan->n_requests) * c.n_kv_heads * ((ctx->group + 31) / 32);
    const int64_t want = std::max<int64_t>(1, kTargetWorkgroups / lanes);
    int64_t kps = (max_ctx + want - 1) / want;
    kps = (kps + mpic::kDecodeBlockKeys - 1) / mpic::kDecodeBlockKeys * mpic::kDecodeBlockKeys;
    keys_per_split = static_cast<int32_t>(kps);
    n_splits = static_cast<int32_t>((max_ctx + kps - 1) / kps);  // <= 256, the merge kernel holds up to 1024 weights
  }
  const size_t rows = static_cast<size_t>(plan->n_requests) * c.n_q_heads;
  const size_t need = rows * n_splits * (c.head_dim + 1) * sizeof(float);
  float* ws = nullptr;
  if (static_scratch) {
    size_t have = 0;
    MPIC_HIP(ctx, mpic::decode_static_scratch(&ws, &have));
    if (need > have)
      return fail(ctx, MPIC_ERR_UNSUPPORTED, "decode_attn_static: the partial results of this batch (" + std::to_string(need) +
                                             " bytes) exceed the static scratch array (" + std::to_string(have) + " bytes)");
  } else if (need > ctx->decode_ws_bytes) {
    // growing the workspace is rare (first call / larger batch): drain what may still read it
    MPIC_HIP(ctx, hipDeviceSynchronize());
    if (ctx->decode_ws) MPIC_HIP(ctx, hipFree(ctx->decode_ws));
    ctx->decode_ws = nullptr;
    ctx->decode_ws_bytes = 0;
    if (hipMalloc(&ctx->decode_ws, need) != hipSuccess) {
      (void)hipGetLastError();
      return fail(ctx, MPIC_ERR_OOM, "decode_attn: workspace allocation failed");
    }
    ctx->decode_ws_bytes = need;
  }
  mpic::DecodeArgs a{};
  a.ctx_off = plan->dev.ctx_off;
  a.dst_slot = plan->dev.dst_slot;
  a.kv_off16 = plan->dev.kv_off16;
  a.q = q;
  a.new_k = new_k;
  a.new_v = new_v;
  a.k_ctx = k_ctx;
  a.v_ctx = v_ctx;
  a.out = out;
  a.lse = lse;
  if (!static_scratch) ws = static_cast<float*>(ctx->decode_ws);
  a.ws_o = ws;
  a.ws_lse = a.ws_o + rows * n_splits * c.head_dim;
  a.scale = static_cast<float>(softmax_scale);
  a.n_q_heads = c.n_q_heads;
  a.n_kv_heads = c.n_kv_heads;
  a.head_dim = c.head_dim;
  a.n_requests = plan->n_requests;
  a.n_splits = n_splits;
  a.keys_per_split = keys_per_split;
  a.max_ctx = max_ctx;
  if (lazy) {
    mpic::LazyRefs lr;
    rc = mpic::fill_lazy_refs(ctx, plan, 32, refs, "decode_attn", &lr);
    if (rc != MPIC_OK) return rc;
    a.interleaved = c.rope_interleaved;
    a.blk_first = by_blocks ? plan->dev.kblk_first[0] : nullptr;
    a.src_inst = plan->dev.src_inst;
    a.src_row = plan->dev.src_row;
    a.rope_cos = plan->dev.rope_cos;
    a.rope_sin = plan->dev.rope_sin;
    MPIC_HIP(ctx, mpic::launch_decode(c.dtype, a, &lr, stream));
    return MPIC_OK;
  }
  MPIC_HIP(ctx, mpic::launch_decode(c.dtype, a, nullptr, stream));
  return MPIC_OK;
}

// The entry points proper: nothing may be thrown across the C boundary, so a failed host
// allocation inside the implementations above becomes MPIC_ERR_OOM here.
#define MPIC_GUARDED(ctx, call)                                         \
  try {                                                                 \
    return call;                                                        \
  } catch (const std::bad_alloc&) {                                     \
    return fail(ctx, MPIC_ERR_OOM, "out of host memory");               \
  }

extern "C" int mpic_assemble_kv_parts(mpic_ctx* ctx, mpic_plan* plan, const mpic_chunk_src* srcs,
                                      int32_t n_srcs, const void* fresh_k, const void* fresh_v,
                                      int64_t n_fresh_rows, void* k_ctx, void* v_ctx,
                                      int64_t n_ctx_slots, uint32_t parts, void* stream) {
  MPIC_GUARDED(ctx, mpic::assemble_parts(ctx, plan, srcs, n_srcs, fresh_k, fresh_v, n_fresh_rows, k_ctx, v_ctx,
                                           n_ctx_slots, parts, stream))
}

extern "C" int mpic_selective_attn(mpic_ctx* ctx, mpic_plan* plan, const void* fresh_q,
                                   int64_t n_fresh_rows, const void* k_ctx, const void* v_ctx,
                                   int64_t n_ctx_slots, double softmax_scale, void* out, float* lse,
                                   void* stream) {
  MPIC_GUARDED(ctx, mpic::attend(ctx, plan, fresh_q, n_fresh_rows, k_ctx, v_ctx, n_ctx_slots, softmax_scale,
                                        out, lse, stream, nullptr))
}

extern "C" int mpic_selective_attn_in_place(mpic_ctx* ctx, mpic_plan* plan, const void* fresh_q,
                                            int64_t n_fresh_rows, const mpic_chunk_src* srcs, int32_t n_srcs,
                                            const void* k_ctx, const void* v_ctx, int64_t n_ctx_slots,
                                            double softmax_scale, void* out, float* lse, void* stream) {
  const mpic::SrcRefs refs{srcs, n_srcs};
  MPIC_GUARDED(ctx, mpic::attend(ctx, plan, fresh_q, n_fresh_rows, k_ctx, v_ctx, n_ctx_slots, softmax_scale,
                                 out, lse, stream, nullptr, 0, &refs))
}

extern "C" int mpic_set_option(mpic_ctx* ctx, int32_t option, int64_t value) {
  if (!ctx) return MPIC_ERR_INVALID;
  switch (option) {
    case MPIC_OPT_ATTN_BLOCK_KEYS:
      if (value != 0 && value != 64 && value != 96) return fail(ctx, MPIC_ERR_INVALID, "set_option: attention block must be 0, 64 or 96 keys");
      ctx->attn_block_keys = static_cast<int32_t>(value);
      return MPIC_OK;
#ifdef MPIC_PROBE_BUILD
    case mpic::kProbeOptionAblate:  // probe library only: timing runs of the bf16 kernel with parts left out
      if (value < 0 || value > 127) return fail(ctx, MPIC_ERR_INVALID, "set_option: ablation mask must be 0..127 (a mask the kernel is not built for fails at the launch)");
      ctx->attn_ablate = static_cast<int32_t>(value);
      return MPIC_OK;
#endif
    default:
      return fail(ctx, MPIC_ERR_INVALID, "set_option: unknown option");
  }
}

extern "C" int mpic_selective_attn_link_next(mpic_ctx* ctx, mpic_plan* plan, const void* fresh_q,
                                             int64_t n_fresh_rows, const void* k_ctx, const void* v_ctx,
                                             int64_t n_ctx_slots, double softmax_scale, void* out, float* lse,
                                             const mpic_chunk_src* next_srcs, int32_t n_srcs, void* next_k_ctx,
                                             void* next_v_ctx, void* stream) {
  const mpic::NextLink next{next_srcs, n_srcs, next_k_ctx, next_v_ctx};
  MPIC_GUARDED(ctx, mpic::attend(ctx, plan, fresh_q, n_fresh_rows, k_ctx, v_ctx, n_ctx_slots, softmax_scale,
                                 out, lse, stream, &next))
}

extern "C" int mpic_decode_attn(mpic_ctx* ctx, mpic_plan* plan, const void* q, const void* new_k,
                                const void* new_v, const void* k_ctx, const void* v_ctx,
                                int64_t n_ctx_slots, double softmax_scale, void* out, float* lse,
                                void* stream) {
  MPIC_GUARDED(ctx, decode_attn_impl(ctx, plan, q, new_k, new_v, k_ctx, v_ctx, n_ctx_slots, softmax_scale, out, lse,
                                     stream, false))
}

extern "C" int mpic_decode_attn_in_place(mpic_ctx* ctx, mpic_plan* plan, const void* q, const void* new_k,
                                         const void* new_v, const mpic_chunk_src* srcs, int32_t n_srcs,
                                         const void* k_ctx, const void* v_ctx, int64_t n_ctx_slots,
                                         double softmax_scale, void* out, float* lse, void* stream) {
  const mpic::SrcRefs refs{srcs, n_srcs};
  MPIC_GUARDED(ctx, decode_attn_impl(ctx, plan, q, new_k, new_v, k_ctx, v_ctx, n_ctx_slots, softmax_scale, out, lse,
                                     stream, false, &refs))
}

extern "C" int mpic_decode_attn_static(mpic_ctx* ctx, mpic_plan* plan, const void* q, const void* new_k,
                                       const void* new_v, const void* k_ctx, const void* v_ctx,
                                       int64_t n_ctx_slots, double softmax_scale, void* out, float* lse,
                                       void* stream) {
  MPIC_GUARDED(ctx, decode_attn_impl(ctx, plan, q, new_k, new_v, k_ctx, v_ctx, n_ctx_slots, softmax_scale, out, lse,
                                     stream, true))
}

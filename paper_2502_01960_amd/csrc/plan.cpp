// Host-side integer planner of libmpic (no GPU calls in this file).
//
// Selection rule, Sec. 4.2: the recompute set is every text token plus the first k
// tokens of every image chunk.  Linking, Fig. 7 step 2 / Sec. 4.1: rows of the
// recompute set are replaced by freshly generated K/V (text slots are only
// placeholders before that), every other row comes from the stored chunk cache.
// The planner turns a batch of segment lists into range-wise filled index maps,
// the rotary tables of the chunk shifts and the launch order of attention tiles.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <new>
#include <numeric>

#include "common.h"

namespace mpic {

int fail(mpic_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->last_error = msg;
  return code;
}

int fail_hip(mpic_ctx* ctx, hipError_t e, const char* what) {
  if (ctx) ctx->last_error = std::string(what) + ": " + hipGetErrorString(e);
  return MPIC_ERR_HIP;
}

namespace {

constexpr int kXcds = 8;  // L2 domains of the chip; workgroup i is dispatched to domain i % 8
constexpr int kComputeUnits = 256;

// Cut the recompute set of every request into attention tiles and order them for launch.
//
// A tile is a range of "flattened rows" of one (request, kv head): all G query heads
// of a fresh row are adjacent, fresh rows follow each other in position order.  Tiles
// are cut every kAttnTileRows rows regardless of run boundaries: the kernel masks per
// row and every wavefront stops at the last key its own rows can see, so a tile that
// straddles two runs costs no more than its parts while full tiles keep the K/V
// stream per flop low.
//
// Small and medium problems do not have a tile per compute unit, or only a few, very
// unequal ones (a tile's work grows with the position of its rows).  Such tiles are also
// cut along the keys: every piece visits a range of 64-key blocks and leaves a partial
// result (normalised output + log-sum-exp) that a merge kernel combines.  The piece size
// is chosen so that the pieces make kSplitRounds rounds over the chip at most -- one round
// when the whole problem is only a few blocks per compute unit -- and never less than
// kMinPieceBlocks blocks (the fixed cost of a workgroup is about one and a half blocks).
// Large problems (more blocks per compute unit than the longest tile has) are not cut.
//
// Launch order: tiles that read the same K/V (same request and kv head) are dealt to the
// same L2 domain, and inside a domain the longest tiles come first so the tail of the
// launch is made of short work.
void build_tiles(mpic_plan& p, int group, int n_kv_heads) {
  struct Item {
    AttnTile t;
    int64_t cost;
  };
  constexpr int64_t kBlock = 64;          // keys per block of the attention kernel
  constexpr int64_t kMinPieceBlocks = 4;
  constexpr int64_t kSplitRounds = 2;
  const int B = p.n_requests;
  const int n_combo = B * n_kv_heads;
  auto last_pos = [&](int b, int64_t row_end) {  // position of the last fresh row below flattened row `row_end`
    return static_cast<int64_t>(p.q_pos[p.q_off[b] + (row_end - 1) / group]);
  };
  // Tile height: full tiles unless even pieces of the smallest size would leave compute
  // units without work; then the height is halved (down to two wavefronts' worth of rows).
  int64_t tile_rows = kAttnTileRows;
  auto count_pieces = [&](int64_t h, int64_t* total_blocks) {
    int64_t n = 0, tot = 0;
    for (int b = 0; b < B; ++b) {
      const int64_t rows = static_cast<int64_t>(p.q_off[b + 1] - p.q_off[b]) * group;
      for (int64_t row = 0; row < rows; row += h) {
        const int64_t blocks = (last_pos(b, std::min(rows, row + h)) + 1 + kBlock - 1) / kBlock;
        n += (blocks + kMinPieceBlocks - 1) / kMinPieceBlocks * n_kv_heads;
        tot += blocks * n_kv_heads;
      }
    }
    if (total_blocks) *total_blocks = tot;
    return n;
  };
  while (tile_rows > 64 && count_pieces(tile_rows, nullptr) < kComputeUnits) tile_rows /= 2;
  int64_t total_blocks = 0;
  count_pieces(tile_rows, &total_blocks);
  const int64_t per_cu = (total_blocks + kComputeUnits - 1) / kComputeUnits;
  const int64_t rounds = std::max<int64_t>(1, std::min<int64_t>(kSplitRounds, per_cu / 16));
  int64_t cap = std::max<int64_t>(kMinPieceBlocks, (total_blocks + kComputeUnits * rounds - 1) / (kComputeUnits * rounds));
  // rounding up per tile makes more pieces than total / cap: grow the cap until they fit the rounds
  auto count_at_cap = [&](int64_t c) {
    int64_t n = 0;
    for (int b = 0; b < B; ++b) {
      const int64_t rows = static_cast<int64_t>(p.q_off[b + 1] - p.q_off[b]) * group;
      for (int64_t row = 0; row < rows; row += tile_rows) {
        const int64_t blocks = (last_pos(b, std::min(rows, row + tile_rows)) + 1 + kBlock - 1) / kBlock;
        n += (blocks + c - 1) / c * n_kv_heads;
      }
    }
    return n;
  };
  while (count_at_cap(cap) > kComputeUnits * rounds && cap < total_blocks) cap += std::max<int64_t>(1, cap / 16);
  // One candidate launch: the tiles cut with pieces of at most `cap` blocks, dealt to the L2
  // domains and ordered inside each.
  struct Layout {
    std::vector<std::vector<Item>> queue;  // per L2 domain, in launch order
    std::vector<AttnMerge> merges;
    int32_t n_parts = 0;
  };
  auto by_cost = [](const Item& a, const Item& b) { return a.cost > b.cost; };
  auto lay_out = [&](int64_t cap_blocks) {
    Layout out;
    std::vector<std::vector<Item>> per_combo(n_combo);
    for (int b = 0; b < B; ++b) {
      const int64_t rows = static_cast<int64_t>(p.q_off[b + 1] - p.q_off[b]) * group;
      for (int64_t row = 0; row < rows; row += tile_rows) {
        const int64_t n = std::min<int64_t>(tile_rows, rows - row);
        const int64_t n_keys = last_pos(b, row + n) + 1;
        const int64_t blocks = (n_keys + kBlock - 1) / kBlock;
        int64_t parts = (blocks > cap_blocks) ? (blocks + cap_blocks - 1) / cap_blocks : 1;
        const int64_t per = (blocks + parts - 1) / parts;  // blocks per piece
        parts = (blocks + per - 1) / per;
        for (int64_t i = 0; i < parts; ++i) {
          const int64_t key0 = i * per * kBlock;
          const int64_t key1 = std::min<int64_t>(n_keys, (i + 1) * per * kBlock);
          // cost = keys visited, summed over the wavefronts of 32 rows (each stops at its own last row)
          int64_t cost = 64;
          for (int64_t w = row; w < row + n; w += 32)
            cost += std::max<int64_t>(0, std::min<int64_t>(last_pos(b, std::min(w + 32, row + n)) + 1, key1) - key0);
          for (int g = 0; g < n_kv_heads; ++g) {
            Item it{};
            it.t.req = b;
            it.t.kv_head = g;
            it.t.row0 = static_cast<int32_t>(row);
            it.t.n_rows = static_cast<int32_t>(n);
            it.t.n_keys = static_cast<int32_t>(key1);
            it.t.key0 = static_cast<int32_t>(key0);
            it.t.part = -1;  // set below for the pieces of a cut tile
            it.cost = cost;
            per_combo[b * n_kv_heads + g].push_back(it);
          }
        }
        if (parts > 1) {
          for (int g = 0; g < n_kv_heads; ++g) {
            AttnMerge m{};
            m.req = b;
            m.kv_head = g;
            m.row0 = static_cast<int32_t>(row);
            m.n_rows = static_cast<int32_t>(n);
            m.first_part = out.n_parts;
            m.n_parts = static_cast<int32_t>(parts);
            out.n_parts += static_cast<int32_t>(parts);
            out.merges.push_back(m);
            // the pieces of this (tile, g) were pushed last into their group, in key order
            auto& v = per_combo[b * n_kv_heads + g];
            for (int64_t i = 0; i < parts; ++i) v[v.size() - parts + i].t.part = m.first_part + static_cast<int32_t>(i);
          }
        }
      }
    }
    out.queue.assign(kXcds, {});
    if (n_combo >= kXcds) {
      // whole (request, kv head) groups go to the currently lightest domain, heaviest first
      std::vector<int> order(n_combo);
      std::iota(order.begin(), order.end(), 0);
      std::vector<int64_t> total(n_combo, 0);
      for (int c = 0; c < n_combo; ++c)
        for (const Item& it : per_combo[c]) total[c] += it.cost;
      std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return total[a] > total[b]; });
      std::vector<int64_t> load(kXcds, 0);
      for (int c : order) {
        const int x = static_cast<int>(std::min_element(load.begin(), load.end()) - load.begin());
        load[x] += total[c];
        out.queue[x].insert(out.queue[x].end(), per_combo[c].begin(), per_combo[c].end());
      }
    } else {
      // fewer groups than domains: spread each group over `share` domains, tile by tile
      const int share = std::max(1, kXcds / std::max(1, n_combo));
      for (int c = 0; c < n_combo; ++c) {
        std::stable_sort(per_combo[c].begin(), per_combo[c].end(), by_cost);
        for (size_t i = 0; i < per_combo[c].size(); ++i)
          out.queue[(c * share + static_cast<int>(i % share)) % kXcds].push_back(per_combo[c][i]);
      }
    }
    for (auto& q : out.queue) std::stable_sort(q.begin(), q.end(), by_cost);
    return out;
  };
  // Predicted duration of a launch, in blocks: every L2 domain hands its tiles in order to
  // whichever of its compute units is free first; a piece of a cut tile costs three blocks
  // more than its keys (prologue, partial result, share of the merge).
  int64_t busy_blocks = 0;  // compute-unit time the tiles of the last simulated layout take, in blocks
  auto predicted_makespan = [&](const Layout& l) {
    int64_t worst = 0;
    busy_blocks = 0;
    auto heavier = std::greater<int64_t>();
    for (const auto& q : l.queue) {
      std::vector<int64_t> load(kComputeUnits / kXcds, 0);  // min-heap of compute unit loads
      for (const Item& it : q) {
        std::pop_heap(load.begin(), load.end(), heavier);
        const int64_t cost = (it.t.n_keys - it.t.key0 + kBlock - 1) / kBlock + 2 + (it.t.part >= 0 ? 3 : 0);
        load.back() += cost;
        busy_blocks += cost;
        std::push_heap(load.begin(), load.end(), heavier);
      }
      worst = std::max(worst, *std::max_element(load.begin(), load.end()));
    }
    return worst;
  };
  Layout chosen = lay_out(cap);
  // Large problems are not cut by the rule above, but a few tiles may be so long that the
  // launch ends with most compute units idle (one request of 75K tokens: the longest tile is
  // two thirds of a compute unit's whole share).  Whether cutting those pays is decided by
  // simulating the launch for a few piece sizes; the uncut launch is kept unless a cut one
  // is predicted to finish at least 3 % earlier.
  if (chosen.n_parts == 0) {
    int64_t longest = 0;
    for (int b = 0; b < B; ++b) {
      const int64_t rows = static_cast<int64_t>(p.q_off[b + 1] - p.q_off[b]) * group;
      if (rows > 0) longest = std::max(longest, (last_pos(b, rows) + 1 + kBlock - 1) / kBlock);
    }
    if (2 * longest > per_cu) {
      const int64_t uncut = predicted_makespan(chosen);
      int64_t best = uncut - uncut * 3 / 100;
      for (const int64_t c : {per_cu * 7 / 10, per_cu * 6 / 10, per_cu / 2, per_cu * 4 / 10}) {
        if (c < kMinPieceBlocks || c >= longest) continue;
        Layout cand = lay_out(c);
        const int64_t m = predicted_makespan(cand);
        if (m < best) {
          best = m;
          chosen = std::move(cand);
        }
      }
    }
  }
  // what the launch is predicted to leave idle: room for work that rides along in its tail
  p.est_makespan_blocks = predicted_makespan(chosen);
  p.est_idle_blocks = p.est_makespan_blocks * kComputeUnits - busy_blocks;
  p.merges = std::move(chosen.merges);
  p.n_parts = chosen.n_parts;
  size_t depth = 0;
  for (const auto& q : chosen.queue) depth = std::max(depth, q.size());
  p.tiles.clear();
  p.tiles.reserve(depth * kXcds);
  for (size_t i = 0; i < depth; ++i)
    for (int x = 0; x < kXcds; ++x) {
      if (i < chosen.queue[x].size()) {
        p.tiles.push_back(chosen.queue[x][i].t);
      } else {
        p.tiles.push_back(AttnTile{});  // padding keeps the i % 8 dealing intact
      }
    }
  while (!p.tiles.empty() && p.tiles.back().n_rows == 0) p.tiles.pop_back();
}

// Key blocks of a lazy_rope plan (see KeyBlock).  A block ends where the source of the keys
// changes (next chunk instance, or stored rows <-> fresh rows), where a tile that was cut
// along the keys starts a new piece (so that a piece owns whole blocks), and after BN keys.
// The list of a request holds its fresh blocks first and its stored blocks after them, each
// part in position order: a kernel that walks a tile in list order changes the shift its
// queries are turned back by once per chunk instance instead of twice (softmax does not care
// about the order of the keys; the mask goes by the positions the blocks carry).  The tiles are
// restated as two ranges of block indices, once per kernel shape.
void build_key_blocks(mpic_plan& p) {
  const int B = p.n_requests;
  std::vector<std::vector<int32_t>> cuts(B);
  for (const AttnTile& t : p.tiles)
    if (t.n_rows > 0 && t.key0 > 0) cuts[t.req].push_back(t.key0);
  for (auto& c : cuts) {
    std::sort(c.begin(), c.end());
    c.erase(std::unique(c.begin(), c.end()), c.end());
  }
  for (int s = 0; s < kNumBlockSizes; ++s) {
    const int32_t bn = kBlockSizes[s];
    auto& blocks = p.kblk[s];
    auto& first = p.kblk_first[s];
    auto& mid = p.kblk_mid[s];
    blocks.clear();
    first.assign(1, 0);
    mid.clear();
    std::vector<KeyBlock> fresh, stored;
    for (int b = 0; b < B; ++b) {
      const int32_t ctx0 = p.ctx_off[b], n = p.ctx_off[b + 1] - ctx0;
      fresh.clear();
      stored.clear();
      size_t next_cut = 0;
      for (int32_t pos = 0; pos < n;) {
        while (next_cut < cuts[b].size() && cuts[b][next_cut] <= pos) ++next_cut;
        const int32_t limit = next_cut < cuts[b].size() ? std::min(n, cuts[b][next_cut]) : n;
        const int32_t inst = p.src_inst[ctx0 + pos];
        int32_t end = pos + 1;
        while (end < limit && p.src_inst[ctx0 + end] == inst) ++end;
        for (int32_t q = pos; q < end; q += bn) (inst < 0 ? fresh : stored).push_back(KeyBlock{q, std::min(bn, end - q), inst, b});
        pos = end;
      }
      blocks.insert(blocks.end(), fresh.begin(), fresh.end());
      mid.push_back(static_cast<int32_t>(blocks.size()));
      blocks.insert(blocks.end(), stored.begin(), stored.end());
      first.push_back(static_cast<int32_t>(blocks.size()));
    }
    p.kblk_flat[s].resize(blocks.size() * 4);
    if (!blocks.empty()) std::memcpy(p.kblk_flat[s].data(), blocks.data(), blocks.size() * sizeof(KeyBlock));
    p.lazy_range[s].clear();
    if (bn == 32) continue;  // the decode kernel splits its blocks at launch
    // blocks of [lo, hi) whose first position is below `pos` (the parts are in position order)
    auto below = [&](int32_t lo, int32_t hi, int32_t pos) {
      const KeyBlock* it = std::lower_bound(blocks.data() + lo, blocks.data() + hi, pos,
                                            [](const KeyBlock& k, int32_t v) { return k.pos0 < v; });
      return static_cast<int32_t>(it - (blocks.data() + lo));
    };
    // per tile: fresh blocks [f0, f1) and stored blocks [s0, s1), counted inside their parts.  A
    // piece starts at a forced block boundary, so every block with a first position in
    // [first key, end key) belongs to it, and only those
    p.lazy_range[s].reserve(p.tiles.size() * 4);
    for (const AttnTile& t : p.tiles) {
      if (t.n_rows <= 0) {
        p.lazy_range[s].insert(p.lazy_range[s].end(), {0, 0, 0, 0});
        continue;
      }
      const int32_t f_lo = first[t.req], f_hi = mid[t.req], s_hi = first[t.req + 1];
      p.lazy_range[s].insert(p.lazy_range[s].end(), {below(f_lo, f_hi, t.key0), below(f_lo, f_hi, t.n_keys),
                                                      below(f_hi, s_hi, t.key0), below(f_hi, s_hi, t.n_keys)});
    }
  }
}

// Rotary tables of the fresh rows, for contexts whose fresh Q/K arrive without positions:
// one table row per distinct position id of the batch (requests with the same layout share
// all of them) and an index per fresh row.  cos/sin of p * w_i are evaluated in double
// from p = 256 * hi + lo by the angle-addition formulas, which needs (max_p / 256 + 256)
// evaluations per frequency instead of one per position, and are rounded once to float.
void build_fresh_rope(mpic_plan& p, const mpic_config& c) {
  const int half = c.head_dim / 2;
  const size_t nq = p.q_pos.size();
  p.fresh_rot.resize(nq);
  if (nq == 0) return;
  const int32_t max_pos = *std::max_element(p.q_pos.begin(), p.q_pos.end());
  std::vector<int32_t> row_of(static_cast<size_t>(max_pos) + 1, -1);
  std::vector<int32_t> uniq;
  for (size_t r = 0; r < nq; ++r) {
    int32_t& u = row_of[p.q_pos[r]];
    if (u < 0) {
      u = static_cast<int32_t>(uniq.size());
      uniq.push_back(p.q_pos[r]);
    }
    p.fresh_rot[r] = u;
  }
  constexpr int kLo = 256;
  const int n_hi = max_pos / kLo + 1;
  std::vector<double> hi_c(static_cast<size_t>(n_hi) * half), hi_s(hi_c.size());
  std::vector<double> lo_c(static_cast<size_t>(kLo) * half), lo_s(lo_c.size());
  for (int j = 0; j < half; ++j) {
    const double w = std::pow(c.rope_theta, -2.0 * j / c.head_dim);
    for (int h = 0; h < n_hi; ++h) {
      const double phi = static_cast<double>(h) * kLo * w;
      hi_c[static_cast<size_t>(h) * half + j] = std::cos(phi);
      hi_s[static_cast<size_t>(h) * half + j] = std::sin(phi);
    }
    for (int l = 0; l < kLo; ++l) {
      const double phi = static_cast<double>(l) * w;
      lo_c[static_cast<size_t>(l) * half + j] = std::cos(phi);
      lo_s[static_cast<size_t>(l) * half + j] = std::sin(phi);
    }
  }
  p.fresh_cos.resize(uniq.size() * half);
  p.fresh_sin.resize(uniq.size() * half);
  for (size_t u = 0; u < uniq.size(); ++u) {
    const double* hc = &hi_c[static_cast<size_t>(uniq[u] / kLo) * half];
    const double* hs = &hi_s[static_cast<size_t>(uniq[u] / kLo) * half];
    const double* lc = &lo_c[static_cast<size_t>(uniq[u] % kLo) * half];
    const double* ls = &lo_s[static_cast<size_t>(uniq[u] % kLo) * half];
    for (int j = 0; j < half; ++j) {
      p.fresh_cos[u * half + j] = static_cast<float>(hc[j] * lc[j] - hs[j] * ls[j]);
      p.fresh_sin[u * half + j] = static_cast<float>(hs[j] * lc[j] + hc[j] * ls[j]);
    }
  }
}

}  // namespace
}  // namespace mpic

using mpic::fail;

extern "C" int mpic_create(mpic_ctx** out, const mpic_config* config) {
  if (!out || !config) return MPIC_ERR_INVALID;
  *out = nullptr;
  const mpic_config& c = *config;
  if (c.n_q_heads <= 0 || c.n_kv_heads <= 0 || c.head_dim <= 0 || c.n_q_heads % c.n_kv_heads != 0 ||
      (c.head_dim & 1) || !(c.rope_theta > 0.0) || !std::isfinite(c.rope_theta) || c.page_size < 0 ||
      (c.rope_interleaved != 0 && c.rope_interleaved != 1) || (c.fresh_pre_rope != 0 && c.fresh_pre_rope != 1) ||
      (c.lazy_rope != 0 && c.lazy_rope != 1))
    return MPIC_ERR_INVALID;
  if (c.dtype == MPIC_F32) {
    if (c.head_dim != 64 && c.head_dim != 128) return MPIC_ERR_UNSUPPORTED;
  } else if (c.dtype == MPIC_BF16) {
    if (c.head_dim != 128) return MPIC_ERR_UNSUPPORTED;
  } else {
    return MPIC_ERR_INVALID;
  }
  mpic_ctx* ctx = new (std::nothrow) mpic_ctx();
  if (!ctx) return MPIC_ERR_OOM;
  ctx->cfg = c;
  ctx->group = c.n_q_heads / c.n_kv_heads;
  *out = ctx;
  return MPIC_OK;
}

extern "C" int mpic_plan_create(mpic_ctx* ctx, int32_t n_requests, const int32_t* seg_off,
                                const mpic_segment* segs, int32_t default_k,
                                const int32_t* page_table, const int32_t* page_table_off,
                                int64_t n_pool_pages, mpic_plan** out) {
  return mpic_plan_create_selected(ctx, n_requests, seg_off, segs, default_k, nullptr, nullptr, page_table,
                                   page_table_off, n_pool_pages, out);
}

extern "C" int mpic_plan_create_selected(mpic_ctx* ctx, int32_t n_requests, const int32_t* seg_off,
                                         const mpic_segment* segs, int32_t default_k,
                                         const int32_t* sel_off, const int32_t* sel_idx,
                                         const int32_t* page_table, const int32_t* page_table_off,
                                         int64_t n_pool_pages, mpic_plan** out) {
  if (!ctx) return MPIC_ERR_INVALID;
  if (!out) return fail(ctx, MPIC_ERR_INVALID, "plan_create: out is NULL");
  *out = nullptr;
  if (n_requests < 1 || !seg_off || default_k < 0)
    return fail(ctx, MPIC_ERR_INVALID, "plan_create: need n_requests >= 1, seg_off, default_k >= 0");
  const int ps = ctx->cfg.page_size;
  if (ps > 0 && (!page_table_off || n_pool_pages <= 0))
    return fail(ctx, MPIC_ERR_INVALID, "plan_create: paged layout needs page table offsets and a pool size");
  if (seg_off[0] != 0) return fail(ctx, MPIC_ERR_INVALID, "plan_create: seg_off[0] must be 0");
  for (int b = 0; b < n_requests; ++b)
    if (seg_off[b + 1] < seg_off[b]) return fail(ctx, MPIC_ERR_INVALID, "plan_create: seg_off must not decrease");
  if (seg_off[n_requests] > 0 && !segs) return fail(ctx, MPIC_ERR_INVALID, "plan_create: segs is NULL");

  // pass 1: validate and size
  int64_t n_ctx = 0, n_q = 0;
  for (int32_t s = 0; s < seg_off[n_requests]; ++s) {
    const mpic_segment& g = segs[s];
    if (g.len < 0 || (g.kind != 0 && g.kind != 1)) return fail(ctx, MPIC_ERR_INVALID, "plan_create: bad segment kind or negative len");
    if (g.kind == 1 && g.chunk < 0) return fail(ctx, MPIC_ERR_INVALID, "plan_create: negative chunk index");
    n_ctx += g.len;
    if (g.kind == 0) {
      n_q += g.len;
    } else if (g.k == MPIC_K_LISTED) {
      if (!sel_off || sel_off[s + 1] < sel_off[s] || (sel_off[s + 1] > sel_off[s] && !sel_idx))
        return fail(ctx, MPIC_ERR_INVALID, "plan_create: a listed recompute set needs sel_off / sel_idx");
      for (int32_t i = sel_off[s]; i < sel_off[s + 1]; ++i)
        if (sel_idx[i] < 0 || sel_idx[i] >= g.len) return fail(ctx, MPIC_ERR_INVALID, "plan_create: listed token outside its chunk");
      n_q += std::min<int64_t>(sel_off[s + 1] - sel_off[s], g.len);  // upper bound (duplicates allowed)
    } else {
      const int64_t k = g.k < 0 ? default_k : g.k;
      n_q += std::min<int64_t>(k, g.len);
    }
  }
  const int64_t slot_limit = ps > 0 ? n_pool_pages * ps : n_ctx;
  if (n_ctx >= INT32_MAX || slot_limit >= INT32_MAX || n_q * ctx->group >= INT32_MAX)
    return fail(ctx, MPIC_ERR_INVALID, "plan_create: batch too large for 32-bit indices");

  mpic_plan* p = new (std::nothrow) mpic_plan();
  if (!p) return fail(ctx, MPIC_ERR_OOM, "plan_create: out of host memory");
  try {
    p->ctx = ctx;
    p->n_requests = n_requests;
    p->n_ctx = n_ctx;
    p->ctx_off.assign(1, 0);
    p->q_off.assign(1, 0);
    p->q_pos.reserve(n_q);
    p->q_req.reserve(n_q);
    p->slot_map.reserve(n_q);
    p->src_inst.resize(n_ctx);
    p->src_row.resize(n_ctx);
    p->dst_slot.resize(n_ctx);
    std::vector<char> page_used, mark;
    if (ps > 0) page_used.assign(n_pool_pages, 0);

    for (int b = 0; b < n_requests; ++b) {
      const int32_t ctx0 = p->ctx_off.back();
      const int32_t q0 = p->q_off.back();
      int32_t pos = 0;  // position inside the request
      int32_t row = q0; // next fresh row
      auto take_fresh = [&](int32_t first, int32_t count) {
        if (count <= 0) return;
        const bool extends = !p->runs.empty() && p->runs[p->runs.size() - 4] == b &&
                             p->runs[p->runs.size() - 1] + p->runs[p->runs.size() - 2] == first;
        if (extends) {
          p->runs[p->runs.size() - 2] += count;
        } else {
          p->runs.insert(p->runs.end(), {b, row, count, first});
        }
        for (int32_t t = 0; t < count; ++t) {
          p->src_inst[ctx0 + first + t] = -1;
          p->src_row[ctx0 + first + t] = row;
          p->q_pos.push_back(first + t);
          p->q_req.push_back(b);
          ++row;
        }
      };
      for (int32_t s = seg_off[b]; s < seg_off[b + 1]; ++s) {
        const mpic_segment& g = segs[s];
        if (g.kind == 0) {
          take_fresh(pos, g.len);
        } else {
          // which tokens of the chunk are recomputed: the first k, or the listed ones
          mark.assign(g.len, 0);
          if (g.k == MPIC_K_LISTED) {
            for (int32_t i = sel_off[s]; i < sel_off[s + 1]; ++i) mark[sel_idx[i]] = 1;
          } else {
            const int64_t k = g.k < 0 ? default_k : g.k;
            std::fill(mark.begin(), mark.begin() + std::min<int64_t>(k, g.len), 1);
          }
          int32_t k_eff = 0;  // length of the leading recomputed run
          while (k_eff < g.len && mark[k_eff]) ++k_eff;
          const int32_t inst = static_cast<int32_t>(p->inst_src.size());
          p->inst_src.push_back(g.chunk);
          p->inst_delta.push_back(pos);
          p->inst_len.push_back(g.len);
          p->inst_k.push_back(k_eff);
          p->inst_req.push_back(b);
          p->max_src = std::max(p->max_src, g.chunk);
          int32_t cached = 0;
          for (int32_t t = 0; t < g.len;) {
            int32_t e = t;
            if (mark[t]) {
              while (e < g.len && mark[e]) ++e;
              take_fresh(pos + t, e - t);
            } else {
              while (e < g.len && !mark[e]) {
                p->src_inst[ctx0 + pos + e] = inst;
                p->src_row[ctx0 + pos + e] = e;
                ++e;
              }
              cached += e - t;
            }
            t = e;
          }
          p->inst_cached.push_back(cached);
        }
        pos += g.len;
      }
      // physical slots
      if (ps > 0) {
        const int64_t have = static_cast<int64_t>(page_table_off[b + 1]) - page_table_off[b];
        const int64_t need = (static_cast<int64_t>(pos) + ps - 1) / ps;
        if (have < need || (need > 0 && !page_table)) {
          delete p;
          return fail(ctx, MPIC_ERR_INVALID, "plan_create: page table missing or shorter than the request");
        }
        const int32_t* tab = page_table + page_table_off[b];
        for (int64_t pg = 0; pg < need; ++pg) {
          const int32_t id = tab[pg];
          if (id < 0 || id >= n_pool_pages || page_used[id]) {
            delete p;
            return fail(ctx, MPIC_ERR_INVALID, "plan_create: page id out of range or used twice");
          }
          page_used[id] = 1;
        }
        for (int32_t t = 0; t < pos; ++t) p->dst_slot[ctx0 + t] = tab[t / ps] * ps + t % ps;
      } else {
        for (int32_t t = 0; t < pos; ++t) p->dst_slot[ctx0 + t] = ctx0 + t;
      }
      for (int32_t r = q0; r < row; ++r) p->slot_map.push_back(p->dst_slot[ctx0 + p->q_pos[r]]);
      p->ctx_off.push_back(ctx0 + pos);
      p->q_off.push_back(row);
    }
    for (int32_t s : p->dst_slot) p->max_slot = std::max<int64_t>(p->max_slot, s);
    p->n_q = static_cast<int64_t>(p->q_pos.size());

    // rotary tables: one angle vector per chunk instance, evaluated in double
    const int half = ctx->cfg.head_dim / 2;
    p->rope_cos.resize(p->inst_src.size() * half);
    p->rope_sin.resize(p->inst_src.size() * half);
    for (size_t i = 0; i < p->inst_src.size(); ++i)
      for (int j = 0; j < half; ++j) {
        const double inv_freq = std::pow(ctx->cfg.rope_theta, -2.0 * j / ctx->cfg.head_dim);
        const double phi = static_cast<double>(p->inst_delta[i]) * inv_freq;
        p->rope_cos[i * half + j] = static_cast<float>(std::cos(phi));
        p->rope_sin[i * half + j] = static_cast<float>(std::sin(phi));
      }
    if (ctx->cfg.fresh_pre_rope) mpic::build_fresh_rope(*p, ctx->cfg);
    mpic::build_tiles(*p, ctx->group, ctx->cfg.n_kv_heads);
    if (ctx->cfg.lazy_rope) {
      mpic::build_key_blocks(*p);
      for (int s = 0; s < mpic::kNumBlockSizes; ++s) {
        p->kblk_parts[s].clear();
        for (int b = 0; b < n_requests; ++b)
          p->kblk_parts[s].insert(p->kblk_parts[s].end(), {p->kblk_first[s][b], p->kblk_mid[s][b], p->kblk_first[s][b + 1]});
      }
    }
    {
      auto clamp = [](int64_t x) { return static_cast<int32_t>(std::min<int64_t>(x, INT32_MAX)); };
      p->launch_est = {clamp(p->est_makespan_blocks), clamp(p->est_idle_blocks),
                       mpic::can_link_in_attention(ctx, p) ? 1 : 0,
                       mpic::can_link_in_attention(ctx, p) && mpic::link_fits_attention_tail(ctx, p) ? 1 : 0};
    }
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(ctx, MPIC_ERR_OOM, "plan_create: out of host memory");
  }
  *out = p;
  return MPIC_OK;
}

extern "C" int mpic_plan_get(const mpic_plan* plan, int32_t what, const int32_t** host_ptr, size_t* n) {
  if (!plan || !host_ptr || !n) return MPIC_ERR_INVALID;
  const std::vector<int32_t>* v = nullptr;
  switch (what) {
    case MPIC_PLAN_CTX_OFF: v = &plan->ctx_off; break;
    case MPIC_PLAN_Q_OFF: v = &plan->q_off; break;
    case MPIC_PLAN_Q_POS: v = &plan->q_pos; break;
    case MPIC_PLAN_Q_REQ: v = &plan->q_req; break;
    case MPIC_PLAN_SLOT_MAP: v = &plan->slot_map; break;
    case MPIC_PLAN_SRC_INST: v = &plan->src_inst; break;
    case MPIC_PLAN_SRC_ROW: v = &plan->src_row; break;
    case MPIC_PLAN_DST_SLOT: v = &plan->dst_slot; break;
    case MPIC_PLAN_INST_SRC: v = &plan->inst_src; break;
    case MPIC_PLAN_INST_DELTA: v = &plan->inst_delta; break;
    case MPIC_PLAN_INST_LEN: v = &plan->inst_len; break;
    case MPIC_PLAN_INST_K: v = &plan->inst_k; break;
    case MPIC_PLAN_INST_REQ: v = &plan->inst_req; break;
    case MPIC_PLAN_RUNS: v = &plan->runs; break;
    case MPIC_PLAN_LAUNCH_ESTIMATE: v = &plan->launch_est; break;
    case MPIC_PLAN_KEY_BLOCKS_32: v = &plan->kblk_flat[0]; break;
    case MPIC_PLAN_KEY_BLOCKS_64: v = &plan->kblk_flat[1]; break;
    case MPIC_PLAN_KEY_BLOCKS_96: v = &plan->kblk_flat[2]; break;
    case MPIC_PLAN_LAZY_TILES_64: v = &plan->lazy_range[1]; break;
    case MPIC_PLAN_LAZY_TILES_96: v = &plan->lazy_range[2]; break;
    case MPIC_PLAN_KEY_BLOCK_PARTS_32: v = &plan->kblk_parts[0]; break;
    case MPIC_PLAN_KEY_BLOCK_PARTS_64: v = &plan->kblk_parts[1]; break;
    case MPIC_PLAN_KEY_BLOCK_PARTS_96: v = &plan->kblk_parts[2]; break;
    case MPIC_PLAN_ATTN_TILES:
      *host_ptr = reinterpret_cast<const int32_t*>(plan->tiles.data());
      *n = plan->tiles.size() * 8;
      return MPIC_OK;
    default:
      return fail(plan->ctx, MPIC_ERR_INVALID, "plan_get: unknown selector");
  }
  *host_ptr = v->data();
  *n = v->size();
  return MPIC_OK;
}

extern "C" int mpic_plan_get_rope(const mpic_plan* plan, const float** cos_tab, const float** sin_tab,
                                  size_t* n) {
  if (!plan || !cos_tab || !sin_tab || !n) return MPIC_ERR_INVALID;
  *cos_tab = plan->rope_cos.data();
  *sin_tab = plan->rope_sin.data();
  *n = plan->rope_cos.size();
  return MPIC_OK;
}

extern "C" int mpic_plan_get_fresh_rope(const mpic_plan* plan, const int32_t** table_row,
                                        const float** cos_tab, const float** sin_tab, size_t* n_rows) {
  if (!plan || !table_row || !cos_tab || !sin_tab || !n_rows) return MPIC_ERR_INVALID;
  *table_row = plan->fresh_rot.data();
  *cos_tab = plan->fresh_cos.data();
  *sin_tab = plan->fresh_sin.data();
  *n_rows = plan->fresh_cos.size() / (plan->ctx->cfg.head_dim / 2);
  return MPIC_OK;
}

extern "C" const char* mpic_strerror(int status) {
  switch (status) {
    case MPIC_OK: return "ok";
    case MPIC_ERR_INVALID: return "invalid argument";
    case MPIC_ERR_UNSUPPORTED: return "unsupported configuration";
    case MPIC_ERR_OOM: return "out of memory";
    case MPIC_ERR_HIP: return "HIP runtime error";
    case MPIC_ERR_IO: return "file of the disk tier could not be written";
    case MPIC_ERR_CACHE_MISS: return "stored cache missing or failed to load";
    default: return "unknown status";
  }
}

extern "C" const char* mpic_last_error(const mpic_ctx* ctx) { return ctx ? ctx->last_error.c_str() : ""; }

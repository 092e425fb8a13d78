// bf16 selective attention of libmpic on the gfx950 matrix cores.
//
// Fig. 7 step 3 / App. A: every row of the recompute set is multiplied with the
// whole linked K cache, softmax-normalised over the positions it may see
// (j <= its own position) and multiplied with the linked V cache.
//
// Work decomposition.  A workgroup (8 wavefronts) owns one tile of the plan: up to
// 256 "flattened rows" (fresh row x query head of one kv group) of one request and
// kv head, all of which read the same K/V.  Each wavefront owns 32 of those rows and
// walks the keys 0..n_keys-1 in blocks of 96 (or 64, see Geo below) that the workgroup
// stages through LDS rings with direct global->LDS loads (no register round trip): the
// next blocks are in flight while one is consumed, and two barriers per block keep the
// rings safe and the two wavefronts of a SIMD in anti-phase.
// The kernel is bound by the L2->LDS stream of K/V blocks as much as by the matrix
// cores, which is why a tile is as tall as the register file allows.
//
// Matrix-core formulation (v_mfma_f32_32x32x16_bf16, verified lane layout:
// A[i][k]: lane i + 32*(k/8), element k%8;  B[k][j]: lane j + 32*(k/8), element k%8;
// C[i][j]: lane j + 32*((i/4)%2), register (i/8)*4 + i%4).
// Both products are computed transposed so that a query is a *column*:
//   S^T[key][query] = K . Q^T        A = K rows from LDS,  B = Q rows kept in registers
//   O^T[d][query]   = V^T . P^T      A = V^T via the LDS transpose read, B = P^T
// With a query per lane column, the softmax statistics (running max, running sum,
// rescale factor) are per-lane scalars, the row reductions are in-register plus one
// exchange with lane^32, and the S^T accumulator registers already hold P^T in the
// B-operand layout of the second product (no data movement between the two MFMAs:
// the contraction index may be permuted freely as long as A and B agree).
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "link_rows.h"
#include "wave_ops.h"

namespace mpic {
namespace {

constexpr int D = 128;   // head dim
constexpr int WAVES = 8;
constexpr int ROWS_PER_WAVE = 32;
constexpr int THREADS = WAVES * 64;
constexpr int ROW_BYTES = D * 2;  // one staged key or value row

// Keys per LDS block and what follows from it.  Two shapes are built:
//   64 keys: K and V rings of four slots (128 KB), loads two blocks ahead, 202 registers -- leaves
//            room on every SIMD for a wave of another kernel (linking on a second stream);
//   96 keys: K ring of two slots, V ring of three (120 KB), loads one block ahead, 238 registers --
//            a third fewer barriers and phase changes per key, 1 to 2.6 % faster alone, but nothing
//            fits beside it (two-stream step of 8 requests x 16 chunks: 2.19 -> 2.32 ms).
template <int kBlockKeys>
struct Geo {
  static_assert(kBlockKeys == 64 || kBlockKeys == 96, "block shapes with a ring layout");
  static constexpr int BN = kBlockKeys;
  static constexpr int KB = BN / 32;                 // 32-key matrix tiles per block
  static constexpr int TILE_BYTES = BN * ROW_BYTES;  // one staged K (or V) block
  static constexpr int K_SLOTS = BN == 64 ? 4 : 2;
  static constexpr int V_SLOTS = BN == 64 ? 4 : 3;
  static constexpr int AHEAD = BN == 64 ? 2 : 1;     // blocks the loads run ahead of their first use
  static constexpr int LDS_BYTES = (K_SLOTS + V_SLOTS) * TILE_BYTES;
  static constexpr int ROWS_LOADED_PER_WAVE = BN / WAVES;               // rows of K (and of V) a wave stages per block
  static constexpr int LOADS_PER_STAGE = 2 * ROWS_LOADED_PER_WAVE / 4;  // direct loads each wave issues per block
  // the V ring comes first: its fragment reads step through a block with immediate offsets (16 keys =
  // 4 KB apart) that must stay below 64 KB, which a ring base of its own would use up
  __device__ static int v_slot_off(int t) { return (t % V_SLOTS) * TILE_BYTES; }
  __device__ static int k_slot_off(int t) { return V_SLOTS * TILE_BYTES + (t % K_SLOTS) * TILE_BYTES; }
};
constexpr int kLinkRounds = 2;  // trips of the linking loop per trailing workgroup
constexpr int kLinkDepth = 2;   // items a thread of a trailing workgroup keeps in flight
constexpr float kSumLimit = 4096.0f;  // lazy rescale: a lane's share of a block's row sum may reach this
static_assert(WAVES * ROWS_PER_WAVE == kAttnTileRows, "tile size and kernel shape must agree");

// Staged rows are 256 bytes = 16 columns of 16 bytes, unpadded (a direct global->LDS
// load writes 64 lanes x 16 bytes contiguously).  Bank conflicts are avoided by
// storing logical column c of row r at column c ^ swizzle(r); the loader permutes its
// *global* addresses accordingly.
//   K, read 16 bytes per lane by 16+ consecutive rows:      swizzle = row & 15
//   V, transpose-read as 4 rows x 64 bytes per 32 lanes:    swizzle = (row & 3) << 2

// Second job a launch may carry: the stored rows of the *next* layer's context, linked by
// workgroups that come after the attention tiles in the grid.  The dispatcher hands out
// workgroups in order, so these start as the attention drains and use the compute units its
// last, longest tiles leave idle (the linking is bandwidth bound and needs no LDS).
struct NoLink {};
struct LinkNext {
  AssembleArgs args;
  AssembleSrcTable tab;
  int32_t n_wgs;  // workgroups after the attention tiles
};

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

__device__ inline void link_share(const LinkNext& ln, int j) {
  const link::Shape sh = link::shape_of<__bf16>(ln.args);
  // workgroup j links rows [lo, hi) of the range; a thread keeps its unit pair and walks down
  // the rows (the launcher only fuses shapes whose pairs per row divide the workgroup)
  const int64_t n_rows = ln.args.pos_end - ln.args.pos_begin;
  const int64_t per = (n_rows + ln.n_wgs - 1) / ln.n_wgs;
  const int64_t lo = ln.args.pos_begin + j * per;
  const int64_t hi = lo + per < ln.args.pos_end ? lo + per : ln.args.pos_end;
  const int u = static_cast<int>(threadIdx.x) % sh.pairs_per_row;
  const int step = THREADS / sh.pairs_per_row;  // rows the workgroup covers per pass
  // One workgroup per compute unit fits beside nothing else (the launch reserves the LDS ring),
  // so each thread keeps kLinkDepth items in flight, all of their loads before the first store.
  // (Depth 1 to 4 and one to four trips per workgroup measured within 5 us of each other on the
  // 18K-token batch of 4: the launch lasts 13-18 us longer than the attention alone, against the
  // 51 us of a linking launch of its own; depth 8 spills and costs 45 us.)
  auto run = [&](auto interleaved) {
    constexpr bool kI = decltype(interleaved)::value;
    for (int64_t r0 = lo + static_cast<int>(threadIdx.x) / sh.pairs_per_row; r0 < hi; r0 += kLinkDepth * step) {
      link::Loaded<__bf16> it[kLinkDepth];
#pragma unroll
      for (int d = 0; d < kLinkDepth; ++d) {
        const int64_t r = r0 + d * step;
        it[d].kdst = nullptr;
        if (r < hi) it[d] = link::load_item_at<__bf16, kI>(ln.args, ln.tab, sh, r, u);
      }
#pragma unroll
      for (int d = 0; d < kLinkDepth; ++d) link::finish_item<__bf16, kI>(it[d], sh);
    }
  };
  if (ln.args.interleaved) {
    run(std::true_type{});
  } else {
    run(std::false_type{});
  }
}

template <int kBlockKeys, typename Extra, int kAblate = 0>
__global__ __launch_bounds__(THREADS, 2) void attn_bf16_kernel(AttnArgs a, Extra extra) {
  using G = Geo<kBlockKeys>;
  constexpr int BN = G::BN, KB = G::KB, TILE_BYTES = G::TILE_BYTES, AHEAD = G::AHEAD;
  constexpr int ROWS_LOADED_PER_WAVE = G::ROWS_LOADED_PER_WAVE, LOADS_PER_STAGE = G::LOADS_PER_STAGE;
  auto k_slot_off = [](int t) { return G::k_slot_off(t); };
  auto v_slot_off = [](int t) { return G::v_slot_off(t); };
  extern __shared__ __attribute__((aligned(1024))) char lds[];  // G::LDS_BYTES: rings of K and V blocks

  if constexpr (std::is_same<Extra, LinkNext>::value) {
    if (static_cast<int>(blockIdx.x) >= a.n_tiles) {
      link_share(extra, static_cast<int>(blockIdx.x) - a.n_tiles);
      return;
    }
  }
  const AttnTile tile = a.tiles[blockIdx.x];
  if (tile.n_rows <= 0) return;  // padding entry of the launch order
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int col = lane & 31;  // query column owned by this lane
  const int hi = lane >> 5;   // which half of the contraction index this lane feeds
  const int group = a.n_q_heads / a.n_kv_heads;
  constexpr bool kLazy = std::is_same<Extra, LazyRefs>::value;
  const int b = tile.req, g = tile.kv_head;
  const int key0 = kLazy ? 0 : tile.key0;  // pieces of a tile cut along the keys start here;
  const int n_keys = tile.n_keys - key0;   // from here on keys and positions are relative to it
  // context row offsets in 16-byte units; read with scalar loads (the table is padded so
  // that reading up to 64 entries past the last key of the tile stays in bounds)
  const __attribute__((address_space(4))) uint32_t* off_of;
  // lazy: the tile visits fresh blocks [fb, fb + nf) and then stored blocks [sb, sb + ns) of the
  // batch's block list (its request's fresh part and stored part); step t of the walk is block bid(t)
  int fb = 0, nf = 0, sb = 0, ns = 0;
  if constexpr (kLazy) {
    const i32x4 rg = *(const __attribute__((address_space(4))) i32x4*)(extra.range + 4 * static_cast<int64_t>(blockIdx.x));
    fb = extra.first[b] + rg[0];
    nf = rg[1] - rg[0];
    sb = extra.mid[b] + rg[2];
    ns = rg[3] - rg[2];
    off_of = (const __attribute__((address_space(4))) uint32_t*)extra.voff;
  } else {
    off_of = (const __attribute__((address_space(4))) uint32_t*)(a.kv_off16 + a.ctx_off[b] + key0);
  }
  auto bid = [&](int t) __attribute__((always_inline)) { return t < nf ? fb + t : sb + (t - nf); };
  const char* kbase = static_cast<const char*>(a.k_ctx) + g * ROW_BYTES;
  const char* vbase = static_cast<const char*>(a.v_ctx) + g * ROW_BYTES;
  const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(MPIC_LDS_PTR(char, lds)));

  // ---- this lane's query ----
  const int local = wave * ROWS_PER_WAVE + col;
  const bool valid = local < tile.n_rows;
  const int flat = tile.row0 + (valid ? local : 0);
  const int64_t fresh_row = a.q_off[b] + flat / group;
  const int head = g * group + flat % group;
  // Last key of this tile (or piece) the row may see.  Padding columns see every key; a row
  // below key0 (negative here) sees none of this piece; a row beyond the end of a piece sees the
  // piece up to its last key (blocks need not end where pieces do).
  // (lazy: positions stay absolute, the blocks carry theirs; a piece owns whole blocks)
  const int my_pos = kLazy ? (valid ? a.q_pos[fresh_row] : 0x3fffffff)
                           : min(valid ? a.q_pos[fresh_row] - key0 : 0x7fffffff, n_keys - 1);
  const int n_iter = kLazy ? nf + ns : (n_keys + BN - 1) / BN;
  // descriptor of key block blk of this tile (lazy only; a scalar load)
  auto desc_of = [&](int blk) __attribute__((always_inline)) {
    blk = blk < n_iter ? blk : n_iter - 1;
    KeyBlock d{};
    if constexpr (kLazy) {
      const i32x4 raw = *(const __attribute__((address_space(4))) i32x4*)(extra.blocks + bid(blk));
      d.pos0 = raw[0];
      d.n_valid = raw[1];
      d.inst = raw[2];
    }
    return d;
  };
  // does the row see any key of this tile (or piece)?
  // first position of the tile (or piece): the smaller of its first fresh and first stored block's
  const int piece_pos0 = kLazy ? min(desc_of(0).pos0, desc_of(nf < n_iter ? nf : 0).pos0) : 0;
  auto sees = [&]() { return my_pos >= piece_pos0; };
  const __bf16* qp = static_cast<const __bf16*>(a.q) + (fresh_row * a.n_q_heads + head) * D;
  bf16x8 qf[8];
  // (Re)load this lane's query fragments.  Queries that arrive without positions are turned by
  // their position id, in fp32; with lazy_rope the query is also turned *back* by the shift of
  // the chunk instance whose keys come next (inst >= 0); one rounding after both.  This lane
  // holds coordinates d = 16*ks + 8*hi + e: a rotate-half pair (d, d + 64) is (qf[ks],
  // qf[ks + 4]) element by element, an interleaved pair (2i, 2i + 1) is two neighbouring
  // elements of one fragment.
  auto fetch_q = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16 + hi * 8);
  };
  auto turn_q = [&](int inst) __attribute__((always_inline)) {
    const bool fwd = a.q_rot != nullptr;
    const bool back = kLazy && inst >= 0;
    if (!fwd && !back) return;
    const float* ct = nullptr;
    const float* st = nullptr;
    const float* cb = nullptr;
    const float* sb = nullptr;
    if (fwd) {
      const int64_t u = a.q_rot[fresh_row];
      ct = a.q_cos + u * (D / 2);
      st = a.q_sin + u * (D / 2);
    }
    if constexpr (kLazy) {
      if (back) {
        cb = extra.rope_cos + static_cast<int64_t>(inst) * (D / 2);
        sb = extra.rope_sin + static_cast<int64_t>(inst) * (D / 2);
      }
    }
    if (a.interleaved) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        f32x8 x = __builtin_convertvector(qf[ks], f32x8);
        if (fwd) {
          const f32x4 c = *reinterpret_cast<const f32x4*>(ct + ks * 8 + hi * 4);
          const f32x4 s = *reinterpret_cast<const f32x4*>(st + ks * 8 + hi * 4);
          f32x8 y;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            y[2 * i] = x[2 * i] * c[i] - x[2 * i + 1] * s[i];
            y[2 * i + 1] = x[2 * i] * s[i] + x[2 * i + 1] * c[i];
          }
          x = y;
        }
        if (back) {
          const f32x4 c = *reinterpret_cast<const f32x4*>(cb + ks * 8 + hi * 4);
          const f32x4 s = *reinterpret_cast<const f32x4*>(sb + ks * 8 + hi * 4);
          f32x8 y;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            y[2 * i] = x[2 * i] * c[i] + x[2 * i + 1] * s[i];
            y[2 * i + 1] = x[2 * i + 1] * c[i] - x[2 * i] * s[i];
          }
          x = y;
        }
        qf[ks] = __builtin_convertvector(x, bf16x8);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        f32x8 x0 = __builtin_convertvector(qf[ks], f32x8);
        f32x8 x1 = __builtin_convertvector(qf[ks + 4], f32x8);
        if (fwd) {
          const f32x8 c = *reinterpret_cast<const f32x8*>(ct + ks * 16 + hi * 8);
          const f32x8 s = *reinterpret_cast<const f32x8*>(st + ks * 16 + hi * 8);
          const f32x8 y0 = x0 * c - x1 * s, y1 = x0 * s + x1 * c;
          x0 = y0;
          x1 = y1;
        }
        if (back) {
          const f32x8 c = *reinterpret_cast<const f32x8*>(cb + ks * 16 + hi * 8);
          const f32x8 s = *reinterpret_cast<const f32x8*>(sb + ks * 16 + hi * 8);
          const f32x8 y0 = x0 * c + x1 * s, y1 = x1 * c - x0 * s;
          x0 = y0;
          x1 = y1;
        }
        qf[ks] = __builtin_convertvector(x0, bf16x8);
        qf[ks + 4] = __builtin_convertvector(x1, bf16x8);
        __builtin_amdgcn_sched_barrier(0);  // one pair of fragments at a time: few registers in flight
      }
    }
  };
  int q_inst = kLazy ? desc_of(0).inst : -1;  // the instance whose shift qf is turned back by
  if constexpr (kLazy) {
    fetch_q();
    turn_q(q_inst);
  } else {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16 + hi * 8);
    if (a.q_rot) {
      const int64_t u = a.q_rot[fresh_row];
      const float* ct = a.q_cos + u * (D / 2);
      const float* st = a.q_sin + u * (D / 2);
      if (a.interleaved) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const f32x4 c = *reinterpret_cast<const f32x4*>(ct + ks * 8 + hi * 4);
          const f32x4 s = *reinterpret_cast<const f32x4*>(st + ks * 8 + hi * 4);
          const f32x8 x = __builtin_convertvector(qf[ks], f32x8);
          f32x8 y;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            y[2 * i] = x[2 * i] * c[i] - x[2 * i + 1] * s[i];
            y[2 * i + 1] = x[2 * i] * s[i] + x[2 * i + 1] * c[i];
          }
          qf[ks] = __builtin_convertvector(y, bf16x8);
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const f32x8 c = *reinterpret_cast<const f32x8*>(ct + ks * 16 + hi * 8);
          const f32x8 s = *reinterpret_cast<const f32x8*>(st + ks * 16 + hi * 8);
          const f32x8 x0 = __builtin_convertvector(qf[ks], f32x8);
          const f32x8 x1 = __builtin_convertvector(qf[ks + 4], f32x8);
          qf[ks] = __builtin_convertvector(x0 * c - x1 * s, bf16x8);
          qf[ks + 4] = __builtin_convertvector(x0 * s + x1 * c, bf16x8);
        }
      }
    }
  }

  const int wave_hi_pos = wave_max_i32(valid ? my_pos : -1);  // negative: idle wave
  const int wave_lo_pos = wave_min_i32(valid ? my_pos : 0x7fffffff);

  const float scale_log2 = a.scale * 1.4426950408889634f;
  float m_run = -INFINITY;  // running reference maximum of the raw logits (scale > 0 keeps the order)
  float l_run = 0.f;        // this lane's share of the running sum (other share: lane^32)
  f32x16 acc_o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc_o[i] = f32x16{0};

  // ---- loader: wave w stages rows (BN/8)w .. (BN/8)(w+1)-1 of K and of V, four rows per 1 KB
  // direct load; lane i of load p owns LDS column i&15 of row (BN/8)w + 4p + (i>>4) ----
  const int ld_sub = lane >> 4;
  const uint32_t ld_col = lane & 15;
  const uint32_t ld_v16 = ld_col ^ (ld_sub << 2);               //          V swizzle = (row & 3) << 2
  const uint32_t sel0 = ld_sub == 0 ? ~0u : 0u, sel1 = ld_sub == 1 ? ~0u : 0u;
  const uint32_t sel2 = ld_sub == 2 ? ~0u : 0u, sel3 = ld_sub == 3 ? ~0u : 0u;
  // BN / 8 rows per wave and block: kLoadPairs loads of four rows for K and as many for V
  constexpr int kLoadPairs = ROWS_LOADED_PER_WAVE / 4;
  struct RowOffs {
    u32x4_a4 q[kLoadPairs];
    int inst;  // lazy: the chunk instance that stores the block's rows, -1 = the context
  };
  auto fetch_rows = [&](int blk) {
    blk = blk < n_iter ? blk : n_iter - 1;
    if constexpr ((kAblate & kAblateSameRows) != 0) blk = 0;  // timing-only variant
    const __attribute__((address_space(4))) u32x4_a4* src = reinterpret_cast<const __attribute__((address_space(4))) u32x4_a4*>(
        off_of + (kLazy ? static_cast<int64_t>(bid(blk)) : static_cast<int64_t>(blk)) * BN + wave * ROWS_LOADED_PER_WAVE);
    RowOffs r;
#pragma unroll
    for (int p = 0; p < kLoadPairs; ++p) r.q[p] = src[p];
    if constexpr (kLazy) r.inst = extra.by_ref ? desc_of(blk).inst : -1;
    return r;
  };
  // `ro` holds the offsets of the block whose loads go out next.  It is refilled at the start
  // of the wave's softmax phase, which touches neither LDS nor scalar memory: the scalar load
  // shares its counter with the LDS reads and returns out of order, so whatever waits on
  // that counter next (the first fragment reads of a matrix part, a barrier) waits for it.
  RowOffs ro = fetch_rows(0);
  int ld_inst = -1;  // lazy: the source the loader's base addresses point to
  const char* ld_kb = kbase;
  const char* ld_vb = vbase;
  auto issue_loads = [&](int blk) {
    const RowOffs cur = ro;
    // the loads go out back to back, each from its own address registers; this lane's row of
    // each group of four is picked with per-lane masks (branch-free)
    const uint32_t row0 = wave * ROWS_LOADED_PER_WAVE;
    const uint32_t dk = lds_base + k_slot_off(blk) + row0 * ROW_BYTES;
    const uint32_t dv = lds_base + v_slot_off(blk) + row0 * ROW_BYTES;
    const void* gk[kLoadPairs];
    const void* gv[kLoadPairs];
    if constexpr (kLazy) {
      // the base of the rows changes only where the source does: the two table entries are
      // read then, not per block (a scalar load that the next instructions wait for)
      if (cur.inst != ld_inst) {
        ld_inst = cur.inst;
        ld_kb = (ld_inst < 0 ? static_cast<const char*>(a.k_ctx) : static_cast<const char*>(extra.k[ld_inst])) + g * ROW_BYTES;
        ld_vb = (ld_inst < 0 ? static_cast<const char*>(a.v_ctx) : static_cast<const char*>(extra.v[ld_inst])) + g * ROW_BYTES;
      }
    }
    const char* kb = kLazy ? ld_kb : kbase;
    const char* vb = kLazy ? ld_vb : vbase;
#pragma unroll
    for (int p = 0; p < kLoadPairs; ++p) {
      const uint32_t r = (cur.q[p][0] & sel0) | (cur.q[p][1] & sel1) | (cur.q[p][2] & sel2) | (cur.q[p][3] & sel3);
      const uint32_t kx = ld_col ^ ((row0 + 4 * p + ld_sub) & 15);  // K swizzle = row & 15
      gk[p] = kb + (static_cast<uint64_t>(r + kx) << 4);
      gv[p] = vb + (static_cast<uint64_t>(r + ld_v16) << 4);
    }
    if constexpr ((kAblate & kAblateAddressesOnly) != 0) {  // timing-only variant: the addresses are formed, nothing is loaded
#pragma unroll
      for (int p = 0; p < kLoadPairs; ++p) asm volatile("" : : "v"(gk[p]), "v"(gv[p]), "s"(dk), "s"(dv));
    } else if constexpr (kLoadPairs == 3) {
      load3x2_to_lds_16B(static_cast<const char*>(gk[0]), static_cast<const char*>(gk[1]), static_cast<const char*>(gk[2]),
                         static_cast<const char*>(gv[0]), static_cast<const char*>(gv[1]), static_cast<const char*>(gv[2]), dk, dv);
    } else {
      static_assert(kLoadPairs == 2 || kLoadPairs == 3, "rows staged per wavefront and block");
      static_assert(4 * ROW_BYTES == 1024, "the loaders step 1024 bytes from one load to the next");
      load2x2_to_lds_16B(static_cast<const char*>(gk[0]), static_cast<const char*>(gk[1]), static_cast<const char*>(gv[0]),
                         static_cast<const char*>(gv[1]), dk, dv);
    }
  };

  // ---- LDS byte offsets of this lane's operand fragments ----
  // K (A operand of S^T): row kb*32 + col, logical column 2*ks + hi
  const int k_row_off = col * ROW_BYTES;
  const int k_col_x = hi ^ (col & 15);  // ^ (ks << 1) per step
  // V^T (A operand of O^T) through the transpose read: 16 lanes fetch a 4-key x 16-d
  // patch, lane i of the patch supplies the address of key i/4, d-offset 4*(i%4) and
  // receives d = patch_d0 + i for the four keys.
  const int i16 = lane & 15;
  const int v_row = hi * 4 + (i16 >> 2);                                                   // + kh*16 (+8)
  const int v_col_x = ((((lane >> 4) & 1) << 1) | ((i16 & 3) >> 1)) ^ ((v_row & 3) << 2);  // ^ (db << 2)
  const int v_off = v_row * ROW_BYTES + (i16 & 1) * 8;

  // every ordinary load (query fragments, positions) is complete before the first direct
  // load is issued: from here on the outstanding-load counter only counts ring traffic
  MPIC_WAIT_VMCNT(0);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < AHEAD; ++i) {
    if (i < n_iter) issue_loads(i);
    ro = fetch_rows(i + 1);
  }

  // Ping-pong schedule.  The two wavefronts that share a SIMD (w and w+4) belong to
  // different groups and run half a block apart: while one group keeps the matrix
  // core busy with O^T += V^T P^T of block t-1 and S^T = K Q^T of block t, the other
  // does the softmax of its block on the vector ALU; a workgroup barrier at every
  // half step keeps them in anti-phase.  Group gp runs its matrix part of block t in
  // half step 2t + gp and its softmax of block t in half step 2t + gp + 1.
  //   K of block t is read in half steps 2t and 2t + 1, V of block t in 2t + 2 and 2t + 3.
  //   The loads of block t + AHEAD are issued at half step 2t (behind its barrier) into the
  //   slots of the blocks whose last reads were in half step 2t - 1: with 64 keys per block K
  //   and V of block t - 2 (rings of four, AHEAD = 2), with 96 keys K of block t - 1 (ring of
  //   two) and V of block t - 2 (ring of three), AHEAD = 1.
  const int gp = wave >> 2;
  f32x16 acc_s[KB];
#pragma unroll
  for (int i = 0; i < KB; ++i) acc_s[i] = f32x16{0};
  bf16x8 pf[2 * KB] = {};

  auto k_frag = [&](const char* stage, int kb, int ks) {
    if constexpr ((kAblate & kAblateLdsReads) != 0) return qf[(ks + kb) & 7];  // timing-only variant
    return *reinterpret_cast<const bf16x8*>(stage + k_row_off + kb * 32 * ROW_BYTES + ((k_col_x ^ (ks << 1)) << 4));
  };
  auto v_frag = [&](const char* stage, int kh, int db) {
    if constexpr ((kAblate & kAblateLdsReads) != 0) return qf[(kh + db) & 7];  // timing-only variant
    const char* vp = stage + v_off + kh * 16 * ROW_BYTES + ((v_col_x ^ (db << 2)) << 4);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MPIC_LDS_PTR(s16x4, vp));
    const s16x4 up = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MPIC_LDS_PTR(s16x4, vp + 8 * ROW_BYTES));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, up, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  // O^T += V^T . P^T of block t: 16 keys per step, each fragment register refilled for the
  // next step right behind the MFMA that read it; the scheduling barriers pin that order
  auto pv_block = [&](int t) {
    const char* stage = lds + v_slot_off(t);
    bf16x8 vf[4];
#pragma unroll
    for (int db = 0; db < 4; ++db) vf[db] = v_frag(stage, 0, db);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kh = 0; kh < 2 * KB; ++kh) {  // kb = kh/2, half = kh%2
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db], pf[kh], acc_o[db], 0, 0, 0);
        if (kh + 1 < 2 * KB) vf[db] = v_frag(stage, kh + 1, db);  // refill behind the MFMA that consumed it
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  // S^T = K . Q^T of block t for 64 keys x 32 queries; LDS reads run kPre steps ahead of
  // the MFMAs and the two key sub-blocks alternate
  auto qk_block = [&](int t) {
    const char* stage = lds + k_slot_off(t);
    constexpr int kPre = 2;
    bf16x8 kf[KB][8];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) acc_s[kb] = f32x16{0};
#pragma unroll
    for (int ks = 0; ks < kPre; ++ks)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) kf[kb][ks] = k_frag(stage, kb, ks);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if (ks + kPre < 8) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb][ks + kPre] = k_frag(stage, kb, ks + kPre);
      }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf[ks], acc_s[kb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // softmax of block t: S^T (acc_s) -> P^T (pf), running sum and reference maximum
  KeyBlock kd{};  // lazy: descriptor of the block softmax_block works on
  auto softmax_block = [&](int t) {
    if constexpr ((kAblate & kAblateSoftmax) != 0) {  // timing-only variant: the products stay connected, nothing else
#pragma unroll
      for (int i = 0; i < 2 * KB; ++i) {
        const f32x4 raw = {acc_s[i / 2][(i & 1) * 8], acc_s[i / 2][(i & 1) * 8 + 1], acc_s[i / 2][(i & 1) * 8 + 2],
                           acc_s[i / 2][(i & 1) * 8 + 3]};
        pf[i] = __builtin_bit_cast(bf16x8, raw);
      }
      m_run = 0.f;
      l_run += 1.f;
      return;
    }
    if constexpr (kLazy) {
      // keys of the block sit at positions pos0 .. pos0 + n_valid - 1; slots behind them are
      // padding; masked on blocks with padding and on the diagonal blocks
      if (kd.n_valid < BN || kd.pos0 + BN - 1 > wave_lo_pos) {
        const int bound = min(my_pos - kd.pos0, kd.n_valid - 1) - hi * 4;  // last visible slot (may be negative)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int slot = kb * 32 + (v >> 2) * 8 + (v & 3);
            acc_s[kb][v] = slot <= bound ? acc_s[kb][v] : -INFINITY;
          }
      }
    } else {
    const int j0 = t * BN;
    // causal mask by position, on the diagonal blocks only
    if (j0 + BN - 1 > wave_lo_pos) {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = j0 + kb * 32 + (v >> 2) * 8 + hi * 4 + (v & 3);
          acc_s[kb][v] = key <= my_pos ? acc_s[kb][v] : -INFINITY;
        }
    }
    }
    // Lazy rescale without a block maximum.  The probabilities are first computed against the
    // current reference point m_run.  All of them are positive, so if this lane's share of the
    // row sum stays below kSumLimit no single one exceeded it, and the reference point may stay:
    // exact in the end because numerator and denominator share it.  (All earlier blocks are
    // already in acc_o: the matrix part of block t-1 ran in the previous half step.)  Only when
    // the sum says otherwise, and as long as a row has no reference point yet, the block is
    // redone the careful way: block maximum, new reference point, accumulators rescaled.  After
    // the first blocks of a row that is rare, and the fast path saves the maximum over the block
    // (a seventh of the vector instructions of the phase the barriers wait for: +2.1 %).
    bool careful = m_run == -INFINITY && sees();  // (rows below a piece never see a key: left alone)
    float l_blk = 0.f;
    if (__builtin_amdgcn_ballot_w64(careful) == 0) {
      const float m_scaled0 = m_run * scale_log2;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          f32x8 p;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            p[e] = __builtin_amdgcn_exp2f(fmaf(acc_s[kb][half * 8 + e], scale_log2, -m_scaled0));
            l_blk += p[e];
          }
          pf[kb * 2 + half] = __builtin_convertvector(p, bf16x8);
        }
      careful = sees() && !(l_blk <= kSumLimit);  // (also true for NaN)
    }
    if (__builtin_amdgcn_ballot_w64(careful) != 0) {
      float m_blk = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) m_blk = fmaxf(m_blk, acc_s[kb][v]);
      m_blk = max_across_halves(m_blk);
      const float m_new = fmaxf(m_run, m_blk);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);  // first block: 0
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db) acc_o[db] *= alpha;
      const float m_scaled = m_run * scale_log2;
      l_blk = 0.f;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          f32x8 p;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            p[e] = __builtin_amdgcn_exp2f(fmaf(acc_s[kb][half * 8 + e], scale_log2, -m_scaled));
            l_blk += p[e];
          }
          pf[kb * 2 + half] = __builtin_convertvector(p, bf16x8);
        }
    }
    l_run += l_blk;
  };

  // even half step 2t: block t must be complete in LDS, then the loads of block t+2 go out
  auto even_sync = [&](int t) {
    if constexpr ((kAblate & kAblateNoLoadWaits) != 0) {  // timing-only variant (with kAblateLdsReads: nothing reads the rings)
      if (t == n_iter) MPIC_WAIT_VMCNT(0);  // no load is in flight when the workgroup gives its LDS back
    } else if (t < n_iter) {
      // this wave's share of block t has landed when at most the loads of the blocks issued
      // after it are still outstanding
      if (AHEAD == 2 && t + 1 < n_iter) {
        MPIC_WAIT_VMCNT(LOADS_PER_STAGE);
      } else {
        MPIC_WAIT_VMCNT(0);
      }
    }
    __syncthreads();
    if constexpr ((kAblate & kAblateLoads) != 0) {  // timing-only variant: the rings are filled once
      if (t + AHEAD < n_iter && t + AHEAD < G::K_SLOTS + G::V_SLOTS) issue_loads(t + AHEAD);
    } else {
      if (t + AHEAD < n_iter) issue_loads(t + AHEAD);
    }
  };
  // matrix half step of block t: finish block t-1 (if this wave needed it), start block t (if it
  // needs it: blocks past the last key the wave can see are skipped; the barriers stay aligned)
  auto matrix_part = [&](int t, bool do_qk, bool do_pv, int inst) __attribute__((always_inline)) {
    __builtin_amdgcn_s_setprio(1);  // the wave that feeds the matrix core is issued first
    if (do_qk) {
      if (do_pv) pv_block(t - 1);
      if constexpr (kLazy) {
        if (inst != q_inst) {  // the keys of this block lack another shift than the last one's:
          // the fragments were fetched again during the softmax phase before, now they are turned
          __builtin_amdgcn_sched_barrier(0);  // (keeps the rotation out of the matrix parts around it)
          turn_q(inst);
          q_inst = inst;
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      qk_block(t);
    } else if (do_pv) {
      pv_block(t - 1);
    }
    __builtin_amdgcn_s_setprio(0);
  };
  if constexpr (kLazy) {
    // the same two loops over the tile's key blocks: a block is needed while its first position
    // is within the wave's reach.  Descriptors are fetched two steps ahead at the start of the
    // softmax phase, like the row offsets, so that nothing waits for a scalar load.  When the
    // keys of the next block lack another shift than the query fragments are turned back by,
    // the fragments are fetched again during the softmax phase (their registers are idle until
    // the next matrix part, which then turns them before its first product).
    bool prev_needed = false;
    if (gp == 0) {
      KeyBlock cur = desc_of(0), nxt = desc_of(1);
      for (int t = 0; t <= n_iter; ++t) {
        const bool needed = t < n_iter && cur.pos0 <= wave_hi_pos;
        even_sync(t);
        matrix_part(t, needed, prev_needed, cur.inst);
        __syncthreads();  // odd half step 2t+1
        ro = fetch_rows(t + AHEAD + 1);
        const KeyBlock nxt2 = desc_of(t + 2);
        if (t + 1 < n_iter && nxt.pos0 <= wave_hi_pos && nxt.inst != q_inst) fetch_q();
        if (needed) {
          kd = cur;
          softmax_block(t);
        }
        prev_needed = needed;
        cur = nxt;
        nxt = nxt2;
      }
    } else {
      KeyBlock sm = desc_of(0), nxt = desc_of(0);  // block of the softmax phase, of the matrix part after it
      for (int t = 0; t <= n_iter; ++t) {
        even_sync(t);
        ro = fetch_rows(t + AHEAD + 1);
        const KeyBlock nxt2 = desc_of(t + 1);
        const bool needed = t < n_iter && nxt.pos0 <= wave_hi_pos;
        if (needed && nxt.inst != q_inst) fetch_q();
        if (prev_needed) {
          kd = sm;
          softmax_block(t - 1);
        }
        __syncthreads();  // odd half step 2t+1
        matrix_part(t, needed, prev_needed, nxt.inst);
        prev_needed = needed;
        sm = nxt;
        nxt = nxt2;
      }
    }
  } else {
    auto matrix_old = [&](int t) {
      const bool do_pv = t >= 1 && (t - 1) * BN <= wave_hi_pos;
      __builtin_amdgcn_s_setprio(1);
      if (t < n_iter && t * BN <= wave_hi_pos) {
        if (do_pv) pv_block(t - 1);
        qk_block(t);
      } else if (do_pv) {
        pv_block(t - 1);
      }
      __builtin_amdgcn_s_setprio(0);
    };
    if (gp == 0) {
      for (int t = 0; t <= n_iter; ++t) {
        even_sync(t);
        matrix_old(t);
        __syncthreads();  // odd half step 2t+1
        ro = fetch_rows(t + AHEAD + 1);
        if (t < n_iter && t * BN <= wave_hi_pos) softmax_block(t);
      }
    } else {
      for (int t = 0; t <= n_iter; ++t) {
        even_sync(t);
        ro = fetch_rows(t + AHEAD + 1);
        if (t >= 1 && (t - 1) * BN <= wave_hi_pos) softmax_block(t - 1);
        __syncthreads();  // odd half step 2t+1
        matrix_old(t);
      }
    }
  }

  // ---- epilogue: normalise and store this lane's query column ----
  if (!valid) return;
  const float l_tot = sum_across_halves(l_run);
  if (tile.part >= 0) {
    // piece of a tile cut along the keys: normalised fp32 partial + log-sum-exp for the merge
    // kernel.  A row that lies below key0 saw no key (its registers may hold NaN: selected
    // away, never multiplied).
    const bool seen = sees();
    const float inv_p = seen ? 1.f / l_tot : 0.f;
    const int64_t slot = static_cast<int64_t>(tile.part) * kAttnTileRows + local;
    float* po = a.ws_o + slot * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = seen ? acc_o[db][q4 * 4 + e] * inv_p : 0.f;
        *reinterpret_cast<f32x4*>(po + db * 32 + q4 * 8 + hi * 4) = o;
      }
    if (hi == 0) a.ws_lse[slot] = seen ? m_run * a.scale + logf(l_tot) : -INFINITY;
    return;
  }
  const float inv = 1.f / l_tot;
  __bf16* op = static_cast<__bf16*>(a.out) + (fresh_row * a.n_q_heads + head) * D;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      f32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = acc_o[db][q4 * 4 + e] * inv;
      *reinterpret_cast<bf16x4*>(op + db * 32 + q4 * 8 + hi * 4) = __builtin_convertvector(o, bf16x4);
    }
  if (a.lse && hi == 0) a.lse[fresh_row * a.n_q_heads + head] = m_run * a.scale + logf(l_tot);
}


// Merge the pieces of tiles that were cut along the keys: one workgroup per 8 rows of a
// cut tile, a thread per four output coordinates of one row.  Every read misses (other
// compute units wrote the partials), so the pieces are fetched four at a time before they
// are combined, with a running reference maximum (one pass).
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a) {
  const AttnMerge m = a.merges[blockIdx.x];
  const int local = blockIdx.y * 8 + (threadIdx.x >> 5);
  if (local >= m.n_rows) return;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int d = (threadIdx.x & 31) * 4;
  const int flat = m.row0 + local;
  const int64_t fresh_row = a.q_off[m.req] + flat / group;
  const int head = m.kv_head * group + flat % group;
  const int64_t slot0 = static_cast<int64_t>(m.first_part) * kAttnTileRows + local;
  // the first piece starts at key 0, which every row sees: the maximum is finite from the
  // first piece on; later pieces a row did not reach carry -inf and weigh nothing
  float mx = -INFINITY, z = 0.f;
  f32x4 o = f32x4{0};
  for (int p0 = 0; p0 < m.n_parts; p0 += 4) {
    float lse[4];
    f32x4 x[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t slot = slot0 + static_cast<int64_t>(min(p0 + i, m.n_parts - 1)) * kAttnTileRows;
      lse[i] = p0 + i < m.n_parts ? a.ws_lse[slot] : -INFINITY;
      x[i] = *reinterpret_cast<const f32x4*>(a.ws_o + slot * D + d);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (lse[i] == -INFINITY) continue;
      const float m_new = fmaxf(mx, lse[i]);
      const float keep = expf(mx - m_new);  // first piece: exp(-inf) = 0
      const float w = expf(lse[i] - m_new);
      z = z * keep + w;
      o = o * keep + w * x[i];
      mx = m_new;
    }
  }
  o *= 1.f / z;
  *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(a.out) + (fresh_row * a.n_q_heads + head) * D + d) =
      __builtin_convertvector(o, bf16x4);
  if (a.lse && d == 0) a.lse[fresh_row * a.n_q_heads + head] = mx + logf(z);
}

}  // namespace

namespace {

inline int64_t n_pos_of(const AssembleArgs* next) { return next ? next->pos_end - next->pos_begin : 0; }

template <int kBlockKeys>
hipError_t launch_shape(const AttnArgs& a, const AssembleArgs* next, const AssembleSrcTable* next_tab,
                        const LazyRefs* lazy, int dev, hipStream_t stream) {
  using G = Geo<kBlockKeys>;
  static LdsOptIn opt_in;  // one per kernel shape
  const hipError_t eo = opt_in.ensure(dev, [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel<kBlockKeys, NoLink>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel<kBlockKeys, LinkNext>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel<kBlockKeys, LazyRefs>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
  });
  if (eo != hipSuccess) return eo;
#ifdef MPIC_PROBE_BUILD
  if (a.ablate != 0 && !lazy && n_pos_of(next) == 0) {
    auto go = [&](auto mask) {
      constexpr int kM = decltype(mask)::value;
      static LdsOptIn probe_opt_in;
      const hipError_t e = probe_opt_in.ensure(dev, [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel<kBlockKeys, NoLink, kM>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
      });
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL((attn_bf16_kernel<kBlockKeys, NoLink, kM>), dim3(a.n_tiles), dim3(THREADS), G::LDS_BYTES, stream, a,
                         NoLink{});
      return hipSuccess;
    };
    switch (a.ablate) {
      case 1: return go(std::integral_constant<int, 1>{});
      case 2: return go(std::integral_constant<int, 2>{});
      case 3: return go(std::integral_constant<int, 3>{});
      case 4: return go(std::integral_constant<int, 4>{});
      case 5: return go(std::integral_constant<int, 5>{});
      case 6: return go(std::integral_constant<int, 6>{});
      case 7: return go(std::integral_constant<int, 7>{});
      case 8: return go(std::integral_constant<int, 8>{});
      case 6 | 8: return go(std::integral_constant<int, 6 | 8>{});
      case 6 | 32: return go(std::integral_constant<int, 6 | 32>{});
      case 6 | 64: return go(std::integral_constant<int, 6 | 64>{});
      default: return hipErrorInvalidValue;
    }
  }
#endif
  if (lazy) {
    hipLaunchKernelGGL((attn_bf16_kernel<kBlockKeys, LazyRefs>), dim3(a.n_tiles), dim3(THREADS), G::LDS_BYTES, stream, a,
                       *lazy);
    return hipSuccess;
  }
  const int64_t n_pos = next ? next->pos_end - next->pos_begin : 0;
  if (n_pos > 0) {
    LinkNext ln;
    ln.args = *next;
    ln.tab = *next_tab;
    // kLinkRounds trips of the loop per workgroup: short enough to fill the gaps the last
    // attention tiles leave
    const int64_t rows_per_pass = THREADS / (next->n_kv_heads * (next->head_dim / 2 / 8));
    const int64_t rows_per_wg = kLinkRounds * kLinkDepth * rows_per_pass;
    ln.n_wgs = static_cast<int32_t>(std::max<int64_t>(1, (n_pos + rows_per_wg - 1) / rows_per_wg));
    hipLaunchKernelGGL((attn_bf16_kernel<kBlockKeys, LinkNext>), dim3(a.n_tiles + ln.n_wgs), dim3(THREADS), G::LDS_BYTES,
                       stream, a, ln);
  } else {
    hipLaunchKernelGGL((attn_bf16_kernel<kBlockKeys, NoLink>), dim3(a.n_tiles), dim3(THREADS), G::LDS_BYTES, stream, a,
                       NoLink{});
  }
  return hipSuccess;
}

}  // namespace

hipError_t launch_attn_bf16(const AttnArgs& a, const AssembleArgs* next, const AssembleSrcTable* next_tab,
                            const LazyRefs* lazy, hipStream_t stream) {
  if (a.n_tiles <= 0) return hipSuccess;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = a.block_keys == 96 ? launch_shape<96>(a, next, next_tab, lazy, dev, stream)
                         : launch_shape<64>(a, next, next_tab, lazy, dev, stream);
  if (e != hipSuccess) return e;
  if (a.n_merges > 0)
    hipLaunchKernelGGL(attn_merge_kernel, dim3(a.n_merges, kAttnTileRows / 8), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace mpic

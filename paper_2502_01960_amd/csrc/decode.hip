// Decode-step attention of libmpic over a linked context (gfx950).
//
// App. A (autoregressive generation): after the prefill the model emits one token at a
// time; the query of the new token attends to every cached position and, its key and
// value being appended to the cache, to itself.  Here the cache is the context that the
// linker wrote (Fig. 7 step 2), contiguous or paged, and the new token of request b sits
// at position N_b.
//
// The step reads every context row once and does 4*D flops per (query head, key), so it
// is bound by HBM bandwidth.  Work decomposition of the bf16 kernel: the keys of one
// (request, kv head) are cut into splits; a workgroup of four wavefronts owns one split
// and its wavefronts take the 32-key blocks of the split in turn, each through its own
// double-buffered LDS staging area filled by direct global->LDS loads (no barrier inside
// the loop: a wavefront only reads what it loaded itself).  The query heads of the kv
// group are the columns of a 32-column matrix-core tile (S^T = K.Q^T, O^T = V^T.P^T, the
// transposed formulation of the prefill kernel: softmax statistics are per-lane
// scalars).  The four wavefronts merge their partial results through LDS and write one
// (O, log-sum-exp) partial per split; a second small kernel merges the splits and adds
// the new token itself.
#include <type_traits>

#include "common.h"
#include "wave_ops.h"

namespace mpic {
namespace {

constexpr int D = 128;
constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;
constexpr int BN = 32;                           // keys per wavefront block
constexpr int ROW_BYTES = D * 2;
constexpr int TILE_BYTES = BN * ROW_BYTES;       // one staged K (or V) block: 8 KB
constexpr int STAGE_BYTES = 2 * TILE_BYTES;      // K block followed by V block
constexpr int STAGES = 2;                        // blocks in flight per wavefront: STAGES - 1
constexpr int WAVE_LDS = STAGES * STAGE_BYTES;
constexpr int LDS_BYTES = WAVES * WAVE_LDS;
constexpr int LOADS_PER_BLOCK = 16;              // direct loads per wavefront and block
constexpr float kSlack = 8.0f;                   // lazy-rescale threshold, log2 units
static_assert(kDecodeBlockKeys % BN == 0, "a split is a whole number of key blocks");
static_assert(LDS_BYTES <= 160 * 1024 && LOADS_PER_BLOCK * (STAGES - 1) <= 63, "LDS size / load counter range");
static_assert(WAVES * 32 * D * 4 + 2 * WAVES * 32 * 4 <= LDS_BYTES, "merge area must fit the staging area");

// wait until at most `blocks` blocks of loads are outstanding; the empty asm keeps the
// compiler from moving an LDS read above the wait
__device__ inline void wait_loads(int blocks) {
  if (blocks >= 3) {
    MPIC_WAIT_VMCNT(48);
  } else if (blocks == 2) {
    MPIC_WAIT_VMCNT(32);
  } else if (blocks == 1) {
    MPIC_WAIT_VMCNT(16);
  } else {
    MPIC_WAIT_VMCNT(0);
  }
  asm volatile("" ::: "memory");
}
static_assert(LOADS_PER_BLOCK == 16, "wait_loads spells the count out");

// Extra = LazyRefs (lazy_rope contexts): the wavefronts walk the request's 32-key blocks of the
// plan (KeyBlock: one source and one missing shift per block, slots past n_valid are padding),
// stage each block from its source's base address, and turn the query back by the block's shift
// whenever it changes, <Rot(-s) q, k> = <q, Rot(s) k>; a.keys_per_split then counts slots of
// those blocks.
struct NoLazy {};
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

template <typename Extra>
__global__ __launch_bounds__(THREADS) void decode_bf16_kernel(DecodeArgs a, Extra extra) {
  constexpr bool kLazy = std::is_same<Extra, LazyRefs>::value;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int col = lane & 31;
  const int hi = lane >> 5;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int col_blocks = (group + 31) / 32;
  const int split = blockIdx.x;
  const int g = blockIdx.y / col_blocks;
  const int cb = blockIdx.y % col_blocks;
  const int b = blockIdx.z;
  // keys of this request, or (lazy) slots of its key blocks
  int n_ctx = a.ctx_off[b + 1] - a.ctx_off[b];
  int vb0 = 0;
  if constexpr (kLazy) {
    n_ctx = (extra.first[b + 1] - extra.first[b]) * BN;
    vb0 = extra.first[b] + split * (a.keys_per_split / BN);
  }
  const int key0 = split * a.keys_per_split;
  if (key0 >= n_ctx) return;  // this request has fewer splits (the whole workgroup leaves)
  const int n_keys = min(n_ctx, key0 + a.keys_per_split) - key0;
  const int n_blk = (n_keys + BN - 1) / BN;

  const __attribute__((address_space(4))) uint32_t* off_of;
  if constexpr (kLazy) {
    off_of = (const __attribute__((address_space(4))) uint32_t*)(extra.voff + static_cast<int64_t>(vb0) * BN);
  } else {
    off_of = (const __attribute__((address_space(4))) uint32_t*)(a.kv_off16 + a.ctx_off[b] + key0);
  }
  auto desc_of = [&](int blk) __attribute__((always_inline)) {
    blk = blk < n_blk ? blk : n_blk - 1;
    KeyBlock d{};
    if constexpr (kLazy) {
      const i32x4 raw = *(const __attribute__((address_space(4))) i32x4*)(extra.blocks + vb0 + blk);
      d.pos0 = raw[0];
      d.n_valid = raw[1];
      d.inst = raw[2];
    }
    return d;
  };
  const char* kbase_ctx = static_cast<const char*>(a.k_ctx) + g * ROW_BYTES;
  const char* vbase_ctx = static_cast<const char*>(a.v_ctx) + g * ROW_BYTES;
  char* my_lds = lds + wave * WAVE_LDS;
  const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(MPIC_LDS_PTR(char, my_lds)));

  // ---- this lane's query column: head cb*32 + col of the kv group (columns past the group
  // repeat its first head and are never written) ----
  const int in_group = cb * 32 + col;
  const bool valid = in_group < group;
  const int head = g * group + (valid ? in_group : cb * 32);
  const __bf16* qp = static_cast<const __bf16*>(a.q) + (static_cast<int64_t>(b) * a.n_q_heads + head) * D;
  bf16x8 qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16 + hi * 8);
  // lazy: the query as handed over, and the query turned back by the shift of instance `inst`
  // (fp32 arithmetic, one rounding).  This lane holds coordinates d = 16*ks + 8*hi + e: a
  // rotate-half pair (d, d + 64) is (q[ks], q[ks + 4]), an interleaved pair two neighbours.
  bf16x8 q0[8];
  int q_inst = -1;
  if constexpr (kLazy) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) q0[ks] = qf[ks];
  }
  auto turn_back = [&](int inst) __attribute__((always_inline)) {
    if (inst < 0) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) qf[ks] = q0[ks];
      return;
    }
    const float* cb = nullptr;
    const float* sb = nullptr;
    if constexpr (kLazy) {
      cb = extra.rope_cos + static_cast<int64_t>(inst) * (D / 2);
      sb = extra.rope_sin + static_cast<int64_t>(inst) * (D / 2);
    }
    if (a.interleaved) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const f32x4 c = *reinterpret_cast<const f32x4*>(cb + ks * 8 + hi * 4);
        const f32x4 s = *reinterpret_cast<const f32x4*>(sb + ks * 8 + hi * 4);
        const f32x8 x = __builtin_convertvector(q0[ks], f32x8);
        f32x8 y;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          y[2 * i] = x[2 * i] * c[i] + x[2 * i + 1] * s[i];
          y[2 * i + 1] = x[2 * i + 1] * c[i] - x[2 * i] * s[i];
        }
        qf[ks] = __builtin_convertvector(y, bf16x8);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const f32x8 c = *reinterpret_cast<const f32x8*>(cb + ks * 16 + hi * 8);
        const f32x8 s = *reinterpret_cast<const f32x8*>(sb + ks * 16 + hi * 8);
        const f32x8 x0 = __builtin_convertvector(q0[ks], f32x8);
        const f32x8 x1 = __builtin_convertvector(q0[ks + 4], f32x8);
        qf[ks] = __builtin_convertvector(x0 * c + x1 * s, bf16x8);
        qf[ks + 4] = __builtin_convertvector(x1 * c - x0 * s, bf16x8);
      }
    }
  };

  const float scale_log2 = a.scale * 1.4426950408889634f;
  float m_run = -INFINITY;
  float l_run = 0.f;
  f32x16 acc_o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc_o[i] = f32x16{0};

  // ---- loader: load p (0..7) stages rows 4p..4p+3 of K and of V; lane i owns LDS column
  // i&15 of row 4p + (i>>4).  Logical column c of row r is stored at column c ^ swizzle(r):
  // K swizzle = r & 15, V swizzle = (r & 3) << 2 (conflict-free fragment reads below) ----
  const int ld_sub = lane >> 4;
  const uint32_t ld_col = lane & 15;
  const uint32_t ld_k16 = ld_col ^ ld_sub;        // ^ ((p & 3) << 2)
  const uint32_t ld_v16 = ld_col ^ (ld_sub << 2);
  struct Rows {
    u32x8_a4 r[4];
    const char* kb;  // lazy: base of the block's rows (context, or the chunk's cache)
    const char* vb;
  };
  auto fetch_rows = [&](int blk) {
    blk = blk < n_blk ? blk : n_blk - 1;
    Rows x;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      x.r[i] = *reinterpret_cast<const __attribute__((address_space(4))) u32x8_a4*>(off_of + blk * BN + i * 8);
    if constexpr (kLazy) {
      const int inst = desc_of(blk).inst;
      const bool in_ctx = inst < 0 || !extra.by_ref;
      x.kb = (in_ctx ? static_cast<const char*>(a.k_ctx) : static_cast<const char*>(extra.k[inst])) + g * ROW_BYTES;
      x.vb = (in_ctx ? static_cast<const char*>(a.v_ctx) : static_cast<const char*>(extra.v[inst])) + g * ROW_BYTES;
    }
    return x;
  };
  auto issue_loads = [&](const Rows& cur, int stage) {
    const char* kbase = kbase_ctx;
    const char* vbase = vbase_ctx;
    if constexpr (kLazy) {
      kbase = cur.kb;
      vbase = cur.vb;
    }
    const uint32_t dst = lds_base + stage * STAGE_BYTES;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const u32x8_a4 q8 = cur.r[p >> 1];
      const int o = (p & 1) * 4;
      const uint32_t r16 = ld_sub == 0 ? q8[o] : ld_sub == 1 ? q8[o + 1] : ld_sub == 2 ? q8[o + 2] : q8[o + 3];
      load_to_lds_16B_nt(kbase + (static_cast<uint64_t>(r16 + (ld_k16 ^ ((p & 3) << 2))) << 4), dst + p * 4 * ROW_BYTES);
      load_to_lds_16B_nt(vbase + (static_cast<uint64_t>(r16 + ld_v16) << 4), dst + TILE_BYTES + p * 4 * ROW_BYTES);
    }
  };

  // ---- LDS byte offsets of this lane's operand fragments (layout of
  // v_mfma_f32_32x32x16_bf16: A[i][k] lane i + 32*(k/8), element k%8; B likewise with the
  // column in place of i; C[i][j] lane j + 32*((i/4)%2), register (i/8)*4 + i%4) ----
  const int k_row_off = col * ROW_BYTES;
  const int k_col_x = hi ^ (col & 15);
  const int i16 = lane & 15;
  const int v_row = hi * 4 + (i16 >> 2);
  const int v_col_x = ((((lane >> 4) & 1) << 1) | ((i16 & 3) >> 1)) ^ ((v_row & 3) << 2);
  const int v_off = TILE_BYTES + v_row * ROW_BYTES + (i16 & 1) * 8;

  // every ordinary load is complete before the first direct load: from here on the
  // outstanding-load counter only counts staging traffic
  MPIC_WAIT_VMCNT(0);
  __builtin_amdgcn_sched_barrier(0);

  // Software pipeline: the loads of the next STAGES-1 blocks of this wavefront are in
  // flight while one block is consumed; row offsets (scalar loads) are fetched one block
  // ahead of the loads that use them.
  const int first = wave;
  const int my_blocks = first < n_blk ? (n_blk - first + WAVES - 1) / WAVES : 0;
  Rows rows = fetch_rows(first);
  int issued = 0;
#pragma unroll
  for (int i = 0; i < STAGES - 1; ++i)
    if (issued < my_blocks) {
      issue_loads(rows, issued % STAGES);
      ++issued;
      rows = fetch_rows(first + issued * WAVES);
    }
  for (int it = 0; it < my_blocks; ++it) {
    const int blk = first + it * WAVES;
    const int stage = it % STAGES;
    if (issued < my_blocks) {
      issue_loads(rows, issued % STAGES);
      ++issued;
      rows = fetch_rows(first + issued * WAVES);
    }
    wait_loads(issued - it - 1);
    const char* st = my_lds + stage * STAGE_BYTES;
    KeyBlock kd{};
    if constexpr (kLazy) {
      kd = desc_of(blk);
      if (kd.inst != q_inst) {  // the keys of this block lack another shift than the last block's
        turn_back(kd.inst);
        q_inst = kd.inst;
      }
    }

    // S^T = K . Q^T for 32 keys x 32 query columns
    f32x16 acc_s = f32x16{0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(st + k_row_off + ((k_col_x ^ (ks << 1)) << 4));
      acc_s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s, 0, 0, 0);
    }
    // keys past the end of the context (ragged last block) take no weight
    if constexpr (kLazy) {
      if (kd.n_valid < BN) {  // slots past the block's keys are padding
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int slot = (v >> 2) * 8 + hi * 4 + (v & 3);
          acc_s[v] = slot < kd.n_valid ? acc_s[v] : -INFINITY;
        }
      }
    } else {
    const int j0 = blk * BN;
    if (j0 + BN > n_keys) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = j0 + (v >> 2) * 8 + hi * 4 + (v & 3);
        acc_s[v] = key < n_keys ? acc_s[v] : -INFINITY;
      }
    }
    }
    float m_blk = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) m_blk = fmaxf(m_blk, acc_s[v]);
    m_blk = max_across_halves(m_blk);
    // lazy rescale: the reference maximum only moves when a block maximum exceeds it by
    // more than kSlack (log2 units); exact because numerator and denominator share it
    if (__builtin_amdgcn_ballot_w64((m_blk - m_run) * scale_log2 > kSlack) != 0) {
      const float m_new = fmaxf(m_run, m_blk);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db) acc_o[db] *= alpha;
    }
    const float m_scaled = m_run * scale_log2;
    bf16x8 pf[2];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      f32x8 p;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = __builtin_amdgcn_exp2f(fmaf(acc_s[half * 8 + e], scale_log2, -m_scaled));
        l_run += p[e];
      }
      pf[half] = __builtin_convertvector(p, bf16x8);
    }
    // O^T += V^T . P^T, 16 keys per step; V^T fragments through the LDS transpose read
#pragma unroll
    for (int kh = 0; kh < 2; ++kh)
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const char* vp = st + v_off + kh * 16 * ROW_BYTES + ((v_col_x ^ (db << 2)) << 4);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MPIC_LDS_PTR(s16x4, vp));
        const s16x4 up = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MPIC_LDS_PTR(s16x4, vp + 8 * ROW_BYTES));
        const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, up, 0, 1, 2, 3, 4, 5, 6, 7));
        acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kh], acc_o[db], 0, 0, 0);
      }
  }

  // ---- merge the four wavefronts through LDS (the staging areas are free now) ----
  const float l_wave = sum_across_halves(l_run);
  __syncthreads();
  float* m_o = reinterpret_cast<float*>(lds);               // [WAVES][32 columns][D]
  float* m_m = m_o + WAVES * 32 * D;                        // [WAVES][32]
  float* m_l = m_m + WAVES * 32;                            // [WAVES][32]
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      f32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = acc_o[db][q4 * 4 + e];
      *reinterpret_cast<f32x4*>(m_o + (wave * 32 + col) * D + db * 32 + q4 * 8 + hi * 4) = o;
    }
  if (hi == 0) {
    m_m[wave * 32 + col] = m_run;
    m_l[wave * 32 + col] = l_wave;
  }
  __syncthreads();
  {
    const int d0 = (tid & 7) * 16;  // this thread's 16 output coordinates
    for (int c = tid >> 3; c < 32; c += THREADS / 8) {  // of these columns
      const int hg = cb * 32 + c;
      if (hg >= group) break;
      float m_tot = -INFINITY;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) m_tot = fmaxf(m_tot, m_m[w * 32 + c]);
      float wgt[WAVES];
      float l_tot = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) {
        const float mw = m_m[w * 32 + c];
        wgt[w] = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mw - m_tot) * scale_log2);
        l_tot += wgt[w] * m_l[w * 32 + c];
      }
      const float inv = 1.f / l_tot;  // a split holds at least one key, so l_tot > 0
      const int64_t part = (static_cast<int64_t>(b) * a.n_q_heads + g * group + hg) * a.n_splits + split;
      float* po = a.ws_o + part * D + d0;
#pragma unroll
      for (int i = 0; i < 16; i += 4) {
        f32x4 acc = f32x4{0};
#pragma unroll
        for (int w = 0; w < WAVES; ++w) acc += wgt[w] * *reinterpret_cast<const f32x4*>(m_o + (w * 32 + c) * D + d0 + i);
        *reinterpret_cast<f32x4*>(po + i) = acc * inv;
      }
      if ((tid & 7) == 0) a.ws_lse[part] = m_tot * a.scale + logf(l_tot);
    }
  }
}

// Merge the splits of one (request, query head) and the new token itself; one thread per
// output coordinate.  The partials were written by other compute units, so every read
// here goes to memory: the split weights are computed once by the first wavefront (one
// split per lane) and the partial outputs are fetched eight at a time before they are
// used, so that the latencies overlap instead of adding up.
template <typename T, int kD>
__global__ __launch_bounds__(kD) void decode_merge_kernel(DecodeArgs a) {
  constexpr int kMaxSplits = 1024;
  __shared__ float red[kD / 64];
  __shared__ float wgt[kMaxSplits];
  __shared__ float stat[2];  // reference maximum, denominator
  const int d = threadIdx.x;
  const int64_t row = blockIdx.x;  // b * Hq + h
  const int b = static_cast<int>(row / a.n_q_heads);
  const int h = static_cast<int>(row % a.n_q_heads);
  const int g = h / (a.n_q_heads / a.n_kv_heads);
  // keys of the request, or (lazy_rope, bf16) slots of its 32-key blocks
  const int n_ctx = a.blk_first ? (a.blk_first[b + 1] - a.blk_first[b]) * 32 : a.ctx_off[b + 1] - a.ctx_off[b];
  const int n_s = (n_ctx + a.keys_per_split - 1) / a.keys_per_split;
  float self = -INFINITY;
  float v_new = 0.f;
  if (a.new_k) {
    const int64_t kv = (static_cast<int64_t>(b) * a.n_kv_heads + g) * kD + d;
    float part = static_cast<float>(static_cast<const T*>(a.q)[row * kD + d]) *
                 static_cast<float>(static_cast<const T*>(a.new_k)[kv]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
    if ((d & 63) == 0) red[d >> 6] = part;
    v_new = static_cast<float>(static_cast<const T*>(a.new_v)[kv]);
  }
  __syncthreads();
  if (a.new_k) {
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < kD / 64; ++i) dot += red[i];
    self = dot * a.scale;
  }
  if (d < 64) {
    // lane l owns splits l, l + 64, ...
    float m = self;
    for (int s = d; s < n_s; s += 64) m = fmaxf(m, a.ws_lse[row * a.n_splits + s]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    float z = 0.f;
    if (m != -INFINITY) {
      for (int s = d; s < n_s; s += 64) {
        const float w = expf(a.ws_lse[row * a.n_splits + s] - m);
        wgt[s] = w;
        z += w;
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) z += __shfl_xor(z, off);
    if (d == 0) {
      stat[0] = m;
      stat[1] = z;
    }
  }
  __syncthreads();
  const float m = stat[0];
  float z = stat[1];
  float o = 0.f;
  if (m != -INFINITY) {
    const float* po = a.ws_o + row * a.n_splits * kD + d;
    int s = 0;
    for (; s + 8 <= n_s; s += 8) {
      float x[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) x[i] = po[static_cast<int64_t>(s + i) * kD];
#pragma unroll
      for (int i = 0; i < 8; ++i) o = fmaf(wgt[s + i], x[i], o);
    }
    for (; s < n_s; ++s) o = fmaf(wgt[s], po[static_cast<int64_t>(s) * kD], o);
    if (a.new_k) {
      const float w = expf(self - m);
      z += w;
      o = fmaf(w, v_new, o);
    }
    o /= z;
  }
  static_cast<T*>(a.out)[row * kD + d] = static_cast<T>(o);
  if (a.lse && d == 0) a.lse[row] = m == -INFINITY ? -INFINITY : m + logf(z);
}

// fp32 path: one wavefront per (request, query head), lanes stride over the keys, two
// passes (maximum, then weighted sum); writes its result as the only split of the row.
// kLazy (lazy_rope contexts): stored keys are turned to their position as they are read, in
// fp32, inside the dot product (see the fp32 prefill kernel); refs.by_ref: stored rows are read
// in their caches.
template <int kD, bool kLazy>
__global__ __launch_bounds__(256) void decode_f32_kernel(DecodeArgs a, LazyRefs refs) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= static_cast<int64_t>(a.n_requests) * a.n_q_heads) return;
  const int b = static_cast<int>(row / a.n_q_heads);
  const int h = static_cast<int>(row % a.n_q_heads);
  const int g = h / (a.n_q_heads / a.n_kv_heads);
  const int n_ctx = a.ctx_off[b + 1] - a.ctx_off[b];
  if (n_ctx == 0) return;  // the merge kernel sees no split for this row
  const int32_t* slot_of = a.dst_slot + a.ctx_off[b];
  const int64_t row_elems = static_cast<int64_t>(a.n_kv_heads) * kD;
  const float* K = static_cast<const float*>(a.k_ctx) + g * kD;
  const float* V = static_cast<const float*>(a.v_ctx) + g * kD;
  float q[kD];
  const float* qp = static_cast<const float*>(a.q) + row * kD;
#pragma unroll
  for (int d = 0; d < kD; d += 4) {
    const float4 t = *reinterpret_cast<const float4*>(qp + d);
    q[d] = t.x; q[d + 1] = t.y; q[d + 2] = t.z; q[d + 3] = t.w;
  }
  const int32_t* inst_of = kLazy ? a.src_inst + a.ctx_off[b] : nullptr;
  const int32_t* row_of = kLazy ? a.src_row + a.ctx_off[b] : nullptr;
  auto row_ptr = [&](int j, const float* ctx_base, const void* const* tab) {
    if constexpr (kLazy) {
      const int inst = inst_of[j];
      if (inst >= 0 && refs.by_ref)
        return static_cast<const float*>(tab[inst]) + g * kD + static_cast<int64_t>(row_of[j]) * row_elems;
    }
    return ctx_base + static_cast<int64_t>(slot_of[j]) * row_elems;
  };
  auto logit = [&](int j) {
    const float* kp = row_ptr(j, K, refs.k);
    if constexpr (kLazy) {
      const int inst = inst_of[j];
      if (inst >= 0) {
        const float* ct = a.rope_cos + static_cast<int64_t>(inst) * (kD / 2);
        const float* st = a.rope_sin + static_cast<int64_t>(inst) * (kD / 2);
        float acc = 0.f;
        for (int i = 0; i < kD / 2; ++i) {
          const int ix = a.interleaved ? 2 * i : i, iy = a.interleaved ? 2 * i + 1 : i + kD / 2;
          const float x = kp[ix], y = kp[iy], c = ct[i], s = st[i];
          acc = fmaf(q[ix], x * c - y * s, acc);
          acc = fmaf(q[iy], x * s + y * c, acc);
        }
        return acc * a.scale;
      }
    }
    float acc = 0.f;
#pragma unroll
    for (int d = 0; d < kD; d += 4) {
      const float4 t = *reinterpret_cast<const float4*>(kp + d);
      acc = fmaf(q[d], t.x, acc);
      acc = fmaf(q[d + 1], t.y, acc);
      acc = fmaf(q[d + 2], t.z, acc);
      acc = fmaf(q[d + 3], t.w, acc);
    }
    return acc * a.scale;
  };
  float m = -INFINITY;
  for (int j = lane; j < n_ctx; j += 64) m = fmaxf(m, logit(j));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  float o[kD];
#pragma unroll
  for (int d = 0; d < kD; ++d) o[d] = 0.f;
  float z = 0.f;
  for (int j = lane; j < n_ctx; j += 64) {
    const float w = expf(logit(j) - m);
    z += w;
    const float* vp = row_ptr(j, V, refs.v);
#pragma unroll
    for (int d = 0; d < kD; d += 4) {
      const float4 t = *reinterpret_cast<const float4*>(vp + d);
      o[d] = fmaf(w, t.x, o[d]);
      o[d + 1] = fmaf(w, t.y, o[d + 1]);
      o[d + 2] = fmaf(w, t.z, o[d + 2]);
      o[d + 3] = fmaf(w, t.w, o[d + 3]);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    z += __shfl_xor(z, off);
#pragma unroll
    for (int d = 0; d < kD; ++d) o[d] += __shfl_xor(o[d], off);
  }
  const float inv = 1.f / z;
  float* po = a.ws_o + row * a.n_splits * kD;  // split 0 of this row
#pragma unroll
  for (int d = 0; d < kD; ++d)
    if (lane == (d & 63)) po[d] = o[d] * inv;
  if (lane == 0) a.ws_lse[row * a.n_splits] = m + logf(z);
}

}  // namespace

// Scratch of mpic_decode_attn_static: partial results of the key splits for callers that must
// not allocate.  The array exists once per GPU for the life of the process.  In host code its
// name is only a handle: the device address comes from hipGetSymbolAddress, looked up once per
// device with that device current, and only that address is handed to kernels.
constexpr size_t kStaticScratchBytes = size_t{8} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t decode_static_scratch(float** ptr, size_t* bytes) {
  static std::mutex mu;
  static void* addr[64] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = static_cast<float*>(addr[dev]);
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

hipError_t launch_decode(int dtype, const DecodeArgs& a, const LazyRefs* lazy, hipStream_t stream) {
  const int64_t rows = static_cast<int64_t>(a.n_requests) * a.n_q_heads;
  if (rows <= 0) return hipSuccess;
  if (dtype == MPIC_F32) {
    const dim3 grid(static_cast<unsigned>((rows + 3) / 4)), block(256);
    const LazyRefs refs = lazy ? *lazy : LazyRefs{};
    if (a.head_dim == 64) {
      if (lazy)
        hipLaunchKernelGGL((decode_f32_kernel<64, true>), grid, block, 0, stream, a, refs);
      else
        hipLaunchKernelGGL((decode_f32_kernel<64, false>), grid, block, 0, stream, a, refs);
      hipLaunchKernelGGL((decode_merge_kernel<float, 64>), dim3(static_cast<unsigned>(rows)), dim3(64), 0, stream, a);
    } else {
      if (lazy)
        hipLaunchKernelGGL((decode_f32_kernel<128, true>), grid, block, 0, stream, a, refs);
      else
        hipLaunchKernelGGL((decode_f32_kernel<128, false>), grid, block, 0, stream, a, refs);
      hipLaunchKernelGGL((decode_merge_kernel<float, 128>), dim3(static_cast<unsigned>(rows)), dim3(128), 0, stream, a);
    }
    return hipGetLastError();
  }
  static LdsOptIn opt_in;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = opt_in.ensure(dev, [] {
    const hipError_t e0 = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_bf16_kernel<NoLazy>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e0 != hipSuccess) return e0;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(decode_bf16_kernel<LazyRefs>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  });
  if (e != hipSuccess) return e;
  const int group = a.n_q_heads / a.n_kv_heads;
  const dim3 grid(a.n_splits, a.n_kv_heads * ((group + 31) / 32), a.n_requests);
  if (a.max_ctx > 0) {
    if (lazy)
      hipLaunchKernelGGL(decode_bf16_kernel<LazyRefs>, grid, dim3(THREADS), LDS_BYTES, stream, a, *lazy);
    else
      hipLaunchKernelGGL(decode_bf16_kernel<NoLazy>, grid, dim3(THREADS), LDS_BYTES, stream, a, NoLazy{});
  }
  hipLaunchKernelGGL((decode_merge_kernel<__bf16, 128>), dim3(static_cast<unsigned>(rows)), dim3(128), 0, stream, a);
  return hipGetLastError();
}

}  // namespace mpic

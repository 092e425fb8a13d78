// bf16 selective attention of libmpic on the gfx950 matrix cores.
//
// Fig. 7 step 3 / App. A: every row of the recompute set is multiplied with the
// whole linked K cache, softmax-normalised over the positions it may see
// (j <= its own position) and multiplied with the linked V cache.
//
// Work decomposition.  A workgroup (4 wavefronts) owns one tile of the plan: up to
// 128 "flattened rows" (fresh row x query head of one kv group) of one request and
// kv head, all of which read the same K/V.  Each wavefront owns 32 of those rows and
// walks the keys 0..n_keys-1 in blocks of 64 that the workgroup stages through LDS.
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
#include "common.h"

namespace mpic {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;            // head dim
constexpr int BN = 64;            // keys per LDS stage
constexpr int LDS_STRIDE = D + 8; // bf16 elements per staged row (272 B: 16-byte reads of
                                  // consecutive rows fall into different bank groups)
constexpr int WAVES = 4;
constexpr int ROWS_PER_WAVE = 32;
static_assert(WAVES * ROWS_PER_WAVE == kAttnTileRows, "tile size and kernel shape must agree");

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

__device__ inline float wave_min(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fminf(x, __shfl_xor(x, off));
  return x;
}
__device__ inline float wave_max(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}

__global__ __launch_bounds__(256) void attn_bf16_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) __bf16 k_lds[BN * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) __bf16 v_lds[BN * LDS_STRIDE];

  const AttnTile tile = a.tiles[blockIdx.x];
  if (tile.n_rows <= 0) return;  // padding entry of the launch order
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int col = lane & 31;  // query column owned by this lane
  const int hi = lane >> 5;   // which half of the contraction index this lane feeds
  const int group = a.n_q_heads / a.n_kv_heads;
  const int b = tile.req, g = tile.kv_head;
  const int n_keys = tile.n_keys;
  const int32_t* slot_of = a.dst_slot + a.ctx_off[b];
  const int64_t row_elems = static_cast<int64_t>(a.n_kv_heads) * D;
  const __bf16* kbase = static_cast<const __bf16*>(a.k_ctx) + g * D;
  const __bf16* vbase = static_cast<const __bf16*>(a.v_ctx) + g * D;

  // ---- this lane's query ----
  const int local = wave * ROWS_PER_WAVE + col;
  const bool valid = local < tile.n_rows;
  const int flat = tile.row0 + (valid ? local : 0);
  const int64_t fresh_row = a.q_off[b] + flat / group;
  const int head = g * group + flat % group;
  const int my_pos = valid ? a.q_pos[fresh_row] : 0x7fffffff;  // padding columns see every key
  const __bf16* qp = static_cast<const __bf16*>(a.q) + (fresh_row * a.n_q_heads + head) * D;
  bf16x8 qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16 + hi * 8);

  const float posf = static_cast<float>(valid ? my_pos : -1);
  const int wave_hi_pos = static_cast<int>(wave_max(posf));                       // -1: idle wave
  const int wave_lo_pos = static_cast<int>(wave_min(valid ? posf : 3.0e9f));

  const float scale_log2 = a.scale * 1.4426950408889634f;
  float m_run = -INFINITY;  // running maximum, in log2 units of the scaled logits
  float l_run = 0.f;        // this lane's share of the running sum (other share: lane^32)
  f32x16 acc_o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc_o[i] = f32x16{0};

  // ---- staging: each thread moves 4 + 4 units of 16 bytes per key block ----
  u32x4 kreg[4], vreg[4];
  auto prefetch = [&](int j0) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int idx = p * 256 + tid;
      int key = j0 + (idx >> 4);
      key = key < n_keys ? key : n_keys - 1;  // clamped rows are never visible to a valid query
      const int64_t off = static_cast<int64_t>(slot_of[key]) * row_elems + (idx & 15) * 8;
      kreg[p] = *reinterpret_cast<const u32x4*>(kbase + off);
      vreg[p] = *reinterpret_cast<const u32x4*>(vbase + off);
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int idx = p * 256 + tid;
      const int o = (idx >> 4) * LDS_STRIDE + (idx & 15) * 8;
      *reinterpret_cast<u32x4*>(k_lds + o) = kreg[p];
      *reinterpret_cast<u32x4*>(v_lds + o) = vreg[p];
    }
  };

  // LDS offsets (elements) of this lane's operand fragments
  const int k_frag = col * LDS_STRIDE + hi * 8;  // + kb*32*LDS_STRIDE + ks*16
  // transpose read: 16 lanes fetch a 4-key x 16-d patch; lane i of the patch ends up with
  // d = patch_d0 + i and the four keys
  const int i16 = lane & 15;
  const int v_frag = (hi * 4 + (i16 >> 2)) * LDS_STRIDE + ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;

  prefetch(0);
  for (int j0 = 0; j0 < n_keys; j0 += BN) {
    __syncthreads();  // previous block fully consumed
    stage();
    __syncthreads();
    if (j0 + BN < n_keys) prefetch(j0 + BN);
    if (j0 > wave_hi_pos) continue;  // nothing visible to this wave any more (barriers stay aligned)

    // S^T = K . Q^T for 64 keys x 32 queries
    f32x16 acc_s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      acc_s[kb] = f32x16{0};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(k_lds + k_frag + kb * 32 * LDS_STRIDE + ks * 16);
        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s[kb], 0, 0, 0);
      }
    }

    // scaled logits in log2 units, causal mask by position on the diagonal blocks only
    const bool need_mask = j0 + BN - 1 > wave_lo_pos;
    float m_blk = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float x = acc_s[kb][v] * scale_log2;
        if (need_mask) {
          const int key = j0 + kb * 32 + (v >> 2) * 8 + hi * 4 + (v & 3);
          x = key <= my_pos ? x : -INFINITY;
        }
        acc_s[kb][v] = x;
        m_blk = fmaxf(m_blk, x);
      }
    m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32));
    const float m_new = fmaxf(m_run, m_blk);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // first block: exp2(-inf) = 0
    m_run = m_new;
    float l_blk = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        f32x8 p;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          p[e] = __builtin_amdgcn_exp2f(acc_s[kb][half * 8 + e] - m_new);
          l_blk += p[e];
        }
        pf[kb * 2 + half] = __builtin_convertvector(p, bf16x8);
      }
    l_run = l_run * alpha + l_blk;
#pragma unroll
    for (int db = 0; db < 4; ++db) acc_o[db] *= alpha;

    // O^T += V^T . P^T
#pragma unroll
    for (int kh = 0; kh < 4; ++kh) {  // 16 keys each: kb = kh/2, half = kh%2
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const __bf16* vp = v_lds + v_frag + kh * 16 * LDS_STRIDE + db * 32;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, vp));
        const s16x4 up = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, vp + 8 * LDS_STRIDE));
        const s16x8 both = __builtin_shufflevector(lo, up, 0, 1, 2, 3, 4, 5, 6, 7);
        acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[kh],
                                                            acc_o[db], 0, 0, 0);
      }
    }
  }

  // ---- epilogue: normalise and store this lane's query column ----
  if (!valid) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32);
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
  if (a.lse && hi == 0)
    a.lse[fresh_row * a.n_q_heads + head] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
}

}  // namespace

hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t stream) {
  if (a.n_tiles <= 0) return hipSuccess;
  hipLaunchKernelGGL(attn_bf16_kernel, dim3(a.n_tiles), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace mpic

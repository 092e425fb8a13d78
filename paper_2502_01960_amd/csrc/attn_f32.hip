// fp32 selective attention of libmpic (gfx950): the validation-precision path.
//
// App. A: a_ij = exp(q_i.k_j * scale) / sum_{t<=i} exp(q_i.k_t * scale) and
// o_i = sum_{j<=i} a_ij v_j, evaluated for the rows of the recompute set only
// (Fig. 7 step 3), with "j <= i" taken by position inside the linked context.
// One wavefront owns one (fresh row, query head): lanes stride over the keys, the row
// maximum is found first and the weighted sum second, so every exponent is <= 0 and
// the arithmetic is plain fp32 with no rescaling.  This kernel exists for accuracy
// (it serves the fp32 configuration); the bf16 path is the fast one.
#include "common.h"

namespace mpic {
namespace {

// kLazy (lazy_rope contexts): a stored key still lacks its position shift; it is turned to its
// global position as it is read (the pair (x, y) of the key becomes (x cos - y sin, x sin + y cos)
// inside the dot product), in fp32, and never written back.  With refs.by_ref the stored rows
// are read in their caches instead of the context.
template <int D, bool kLazy>
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnArgs a, int64_t n_q, LazyRefs refs) {
  const int lane = threadIdx.x & 63;
  const int64_t item = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (item >= n_q * a.n_q_heads) return;  // whole wave leaves together
  const int64_t r = item / a.n_q_heads;
  const int h = static_cast<int>(item % a.n_q_heads);
  const int g = h / (a.n_q_heads / a.n_kv_heads);
  int b = 0;
  while (b + 1 < a.n_requests && a.q_off[b + 1] <= r) ++b;
  const int32_t* slot_of = a.dst_slot + a.ctx_off[b];
  const int n_keys = a.q_pos[r] + 1;
  const int64_t row_elems = static_cast<int64_t>(a.n_kv_heads) * D;
  const float* K = static_cast<const float*>(a.k_ctx) + g * D;
  const float* V = static_cast<const float*>(a.v_ctx) + g * D;

  float q[D];
  const float* qp = static_cast<const float*>(a.q) + (r * a.n_q_heads + h) * D;
#pragma unroll
  for (int d = 0; d < D; d += 4) {
    const float4 t = *reinterpret_cast<const float4*>(qp + d);
    q[d] = t.x; q[d + 1] = t.y; q[d + 2] = t.z; q[d + 3] = t.w;
  }

  if (a.q_rot) {
    // a query that arrives without its position is turned by its position id first
    const float* ct = a.q_cos + static_cast<int64_t>(a.q_rot[r]) * (D / 2);
    const float* st = a.q_sin + static_cast<int64_t>(a.q_rot[r]) * (D / 2);
    if (a.interleaved) {
#pragma unroll
      for (int i = 0; i < D / 2; ++i) {
        const float x = q[2 * i], y = q[2 * i + 1], c = ct[i], s = st[i];
        q[2 * i] = x * c - y * s;
        q[2 * i + 1] = x * s + y * c;
      }
    } else {
#pragma unroll
      for (int i = 0; i < D / 2; ++i) {
        const float x = q[i], y = q[i + D / 2], c = ct[i], s = st[i];
        q[i] = x * c - y * s;
        q[i + D / 2] = x * s + y * c;
      }
    }
  }

  const int32_t* inst_of = kLazy ? a.src_inst + a.ctx_off[b] : nullptr;
  const int32_t* row_of = kLazy ? a.src_row + a.ctx_off[b] : nullptr;
  // where the key / value row of position j is stored
  auto row_ptr = [&](int j, const float* ctx_base, const void* const* tab) {
    if constexpr (kLazy) {
      const int inst = inst_of[j];
      if (inst >= 0 && refs.by_ref)
        return static_cast<const float*>(tab[inst]) + g * D + static_cast<int64_t>(row_of[j]) * row_elems;
    }
    return ctx_base + static_cast<int64_t>(slot_of[j]) * row_elems;
  };
  auto logit = [&](int j) {
    const float* kp = row_ptr(j, K, refs.k);
    if constexpr (kLazy) {
      const int inst = inst_of[j];
      if (inst >= 0) {
        const float* ct = a.rope_cos + static_cast<int64_t>(inst) * (D / 2);
        const float* st = a.rope_sin + static_cast<int64_t>(inst) * (D / 2);
        float acc = 0.f;
        for (int i = 0; i < D / 2; ++i) {
          const int ix = a.interleaved ? 2 * i : i, iy = a.interleaved ? 2 * i + 1 : i + D / 2;
          const float x = kp[ix], y = kp[iy], c = ct[i], s = st[i];
          acc = fmaf(q[ix], x * c - y * s, acc);
          acc = fmaf(q[iy], x * s + y * c, acc);
        }
        return acc * a.scale;
      }
    }
    float acc = 0.f;
#pragma unroll
    for (int d = 0; d < D; d += 4) {
      const float4 t = *reinterpret_cast<const float4*>(kp + d);
      acc = fmaf(q[d], t.x, acc);
      acc = fmaf(q[d + 1], t.y, acc);
      acc = fmaf(q[d + 2], t.z, acc);
      acc = fmaf(q[d + 3], t.w, acc);
    }
    return acc * a.scale;
  };

  float m = -INFINITY;
  for (int j = lane; j < n_keys; j += 64) m = fmaxf(m, logit(j));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));

  float o[D];
#pragma unroll
  for (int d = 0; d < D; ++d) o[d] = 0.f;
  float z = 0.f;
  for (int j = lane; j < n_keys; j += 64) {
    const float w = expf(logit(j) - m);
    z += w;
    const float* vp = row_ptr(j, V, refs.v);
#pragma unroll
    for (int d = 0; d < D; d += 4) {
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
    for (int d = 0; d < D; ++d) o[d] += __shfl_xor(o[d], off);
  }
  const float inv = 1.f / z;
  float* op = static_cast<float*>(a.out) + (r * a.n_q_heads + h) * D;
#pragma unroll
  for (int d = 0; d < D; ++d)
    if (lane == (d & 63)) op[d] = o[d] * inv;
  if (a.lse && lane == 0) a.lse[r * a.n_q_heads + h] = m + logf(z);
}

}  // namespace

hipError_t launch_attn_f32(const AttnArgs& a, int64_t n_q, const LazyRefs* lazy, hipStream_t stream) {
  const int64_t items = n_q * a.n_q_heads;
  if (items <= 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>((items + 3) / 4)), block(256);
  if (lazy) {
    if (a.head_dim == 64)
      hipLaunchKernelGGL((attn_f32_kernel<64, true>), grid, block, 0, stream, a, n_q, *lazy);
    else
      hipLaunchKernelGGL((attn_f32_kernel<128, true>), grid, block, 0, stream, a, n_q, *lazy);
  } else {
    if (a.head_dim == 64)
      hipLaunchKernelGGL((attn_f32_kernel<64, false>), grid, block, 0, stream, a, n_q, LazyRefs{});
    else
      hipLaunchKernelGGL((attn_f32_kernel<128, false>), grid, block, 0, stream, a, n_q, LazyRefs{});
  }
  return hipGetLastError();
}

}  // namespace mpic

// Token ranking by K distance (gfx950 kernel + host ranking).
//
// Sec. 4.2: the rule "recompute the first k tokens of an image" comes from an experiment
// that compares two KV caches of the same image computed at different positions: the K
// distance of a token is the L1 distance between its two K tensors, and per layer the tokens
// are ranked by it.  The kernel computes that distance for every token of a chunk (one
// wavefront per token, 16-byte loads, fp32 accumulation; it reads both caches once, so
// it is bound by HBM bandwidth); the ranking itself is a partial sort on the host.
#include <algorithm>
#include <new>
#include <numeric>

#include "common.h"

namespace mpic {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename Raw, typename Wide, int kElems>
__global__ __launch_bounds__(256) void k_distance_kernel(const void* ka, const void* kb, int64_t n_tokens,
                                                         int units_per_row, float* dist) {
  const int lane = threadIdx.x & 63;
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (t >= n_tokens) return;  // whole wave leaves together
  const Raw* a = static_cast<const Raw*>(ka) + t * units_per_row;
  const Raw* b = static_cast<const Raw*>(kb) + t * units_per_row;
  float acc = 0.f;
  for (int u = lane; u < units_per_row; u += 64) {
    const Wide x = __builtin_convertvector(__builtin_nontemporal_load(a + u), Wide);
    const Wide y = __builtin_convertvector(__builtin_nontemporal_load(b + u), Wide);
#pragma unroll
    for (int e = 0; e < kElems; ++e) acc += fabsf(x[e] - y[e]);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (lane == 0) dist[t] = acc;
}

}  // namespace
}  // namespace mpic

extern "C" int mpic_k_distance(mpic_ctx* ctx, const void* k_a, const void* k_b, int64_t n_tokens,
                               float* dist, void* stream_) {
  if (!ctx) return MPIC_ERR_INVALID;
  if (n_tokens < 0 || n_tokens >= INT32_MAX) return mpic::fail(ctx, MPIC_ERR_INVALID, "k_distance: bad token count");
  if (n_tokens == 0) return MPIC_OK;
  if (!k_a || !k_b || !dist) return mpic::fail(ctx, MPIC_ERR_INVALID, "k_distance: null buffer");
  if ((reinterpret_cast<uintptr_t>(k_a) | reinterpret_cast<uintptr_t>(k_b)) & 15)
    return mpic::fail(ctx, MPIC_ERR_INVALID, "k_distance: caches must be 16-byte aligned");
  const mpic_config& c = ctx->cfg;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const int row_bytes = c.n_kv_heads * c.head_dim * (c.dtype == MPIC_F32 ? 4 : 2);
  const dim3 grid(static_cast<unsigned>((n_tokens + 3) / 4)), block(256);
  if (c.dtype == MPIC_F32) {
    hipLaunchKernelGGL((mpic::k_distance_kernel<mpic::f32x4, mpic::f32x4, 4>), grid, block, 0, stream, k_a, k_b, n_tokens,
                       row_bytes / 16, dist);
  } else {
    hipLaunchKernelGGL((mpic::k_distance_kernel<mpic::bf16x8, mpic::f32x8, 8>), grid, block, 0, stream, k_a, k_b, n_tokens,
                       row_bytes / 16, dist);
  }
  MPIC_HIP(ctx, hipGetLastError());
  return MPIC_OK;
}

extern "C" int mpic_rank_tokens(const float* dist, int64_t n_tokens, int64_t n_top, int32_t* idx) {
  if (n_tokens < 0 || n_top < 0 || n_tokens >= INT32_MAX) return MPIC_ERR_INVALID;
  n_top = std::min(n_top, n_tokens);
  if (n_top == 0) return MPIC_OK;
  if (!dist || !idx) return MPIC_ERR_INVALID;
  try {
    std::vector<int32_t> order(static_cast<size_t>(n_tokens));
    std::iota(order.begin(), order.end(), 0);
    // larger distance first; of two equal distances the lower index first (NaN ranks last)
    auto before = [&](int32_t x, int32_t y) {
      const float dx = dist[x], dy = dist[y];
      if (dx != dx || dy != dy) return dx == dx && dy != dy ? true : (dx != dx && dy != dy ? x < y : false);
      return dx > dy || (dx == dy && x < y);
    };
    std::partial_sort(order.begin(), order.begin() + n_top, order.end(), before);
    std::sort(order.begin(), order.begin() + n_top);
    std::copy(order.begin(), order.begin() + n_top, idx);
  } catch (const std::bad_alloc&) {
    return MPIC_ERR_OOM;
  }
  return MPIC_OK;
}

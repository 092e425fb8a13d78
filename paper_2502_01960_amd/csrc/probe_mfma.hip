// Sustained-rate probe for the bf16 matrix cores of gfx950 (measurement aid: it is part of
// libmpic_probe.so only, the product library does not contain it).
//
// What rate do the matrix cores hold when nothing else is in the way?  The probe issues the
// matrix instruction of the attention kernel, v_mfma_f32_32x32x16_bf16, on register operands
// (random bf16 values), 48 per wavefront and "block" -- the count of one 96-key block of the
// kernel: 24 for K.Q^T, 24 for V^T.P^T -- with eight wavefronts per workgroup and one
// workgroup per compute unit, and lets the caller add two parts of the kernel's loop:
//   PROBE_PINGPONG  the two wavefronts of a SIMD run half a block apart, two workgroup
//                   barriers per block, matrix part at raised priority (without it: no
//                   barrier at all, every wavefront issues its matrix instructions back to back)
//   PROBE_SOFTMAX   between the two products the vector ALU does the work of the softmax
//                   phase: 48 exp2 of a scaled difference, 48 additions, 24 packed
//                   conversions to bf16 per lane
// Staging through LDS and the global->LDS loads are not imitated here: their cost is read off
// timing-only variants of the kernel itself (kAblate* in common.h).
// Flops counted: 48 x 32 x 32 x 16 x 2 per wavefront and block.  The output is a checksum that
// keeps the compiler from dropping the work.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "wave_ops.h"

namespace mpic {
namespace {

enum { PROBE_PINGPONG = 1, PROBE_SOFTMAX = 2 };

constexpr int WAVES = 8;
constexpr int THREADS = WAVES * 64;
constexpr int KB = 3;                   // 32-key matrix tiles per block of 96 keys
constexpr int LDS_BYTES = 120 * 1024;   // reserved, not used: one workgroup per compute unit, like the kernel

template <int kFlags>
__global__ __launch_bounds__(THREADS, 2) void probe_kernel(int n_blocks, const __bf16* seed, float* sink) {
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  // operands in registers: "query", "key" and "value" fragments
  bf16x8 qf[8], kreg[4], vreg[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) qf[i] = *reinterpret_cast<const bf16x8*>(seed + (lane * 16 + i) * 8);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    kreg[i] = *reinterpret_cast<const bf16x8*>(seed + (lane * 16 + 8 + i) * 8);
    vreg[i] = *reinterpret_cast<const bf16x8*>(seed + (lane * 16 + 12 + i) * 8);
  }
  f32x16 acc_o[4], acc_s[KB];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc_o[i] = f32x16{0};
#pragma unroll
  for (int i = 0; i < KB; ++i) acc_s[i] = f32x16{0};
  bf16x8 pf[2 * KB];
#pragma unroll
  for (int i = 0; i < 2 * KB; ++i) pf[i] = qf[i & 7];
  float l_run = 0.f;
  const float m_scaled = 3.0f;

  auto pv_block = [&]() {  // 24 matrix instructions, four independent accumulators
#pragma unroll
    for (int kh = 0; kh < 2 * KB; ++kh)
#pragma unroll
      for (int db = 0; db < 4; ++db) acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vreg[db], pf[kh], acc_o[db], 0, 0, 0);
  };
  auto qk_block = [&]() {  // 24 matrix instructions, three independent accumulators
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) acc_s[kb] = f32x16{0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kreg[(ks + kb) & 3], qf[ks], acc_s[kb], 0, 0, 0);
  };
  auto softmax_block = [&]() {
    if constexpr ((kFlags & PROBE_SOFTMAX) != 0) {
      float l_blk = 0.f;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          f32x8 p;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            p[e] = __builtin_amdgcn_exp2f(fmaf(acc_s[kb][half * 8 + e], 1.0e-3f, -m_scaled));
            l_blk += p[e];
          }
          pf[kb * 2 + half] = __builtin_convertvector(p, bf16x8);
        }
      l_run += l_blk;
    } else {
      // keeps every product of the block alive at the cost of three additions
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) l_run += acc_s[kb][kb];
    }
  };
  auto sync = [&]() {
    if constexpr ((kFlags & PROBE_PINGPONG) != 0) __syncthreads();
  };
  auto matrix_part = [&](int t) {
    __builtin_amdgcn_s_setprio(1);
    if (t >= 1) pv_block();
    if (t < n_blocks) qk_block();
    __builtin_amdgcn_s_setprio(0);
  };
  const int gp = (kFlags & PROBE_PINGPONG) ? wave >> 2 : 0;
  if (gp == 0) {
    for (int t = 0; t <= n_blocks; ++t) {
      sync();
      matrix_part(t);
      sync();
      if (t < n_blocks) softmax_block();
    }
  } else {
    for (int t = 0; t <= n_blocks; ++t) {
      sync();
      if (t >= 1) softmax_block();
      sync();
      matrix_part(t);
    }
  }
  float s = l_run;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc_o[i][v];
  sink[static_cast<int64_t>(blockIdx.x) * THREADS + tid] = s;
}

template <int kFlags>
hipError_t launch(int n_wgs, int n_blocks, const void* seed, float* sink, hipStream_t stream) {
  static LdsOptIn opt_in;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = opt_in.ensure(dev, [] {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(probe_kernel<kFlags>), hipFuncAttributeMaxDynamicSharedMemorySize,
                               LDS_BYTES);
  });
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((probe_kernel<kFlags>), dim3(n_wgs), dim3(THREADS), LDS_BYTES, stream, n_blocks,
                     static_cast<const __bf16*>(seed), sink);
  return hipGetLastError();
}

}  // namespace
}  // namespace mpic

// One launch of the probe.  flags: PROBE_PINGPONG (1), optionally | PROBE_SOFTMAX (2), or 0.
// n_wgs workgroups of 512 threads run n_blocks blocks each.  seed: device buffer of
// 64 * 16 * 8 bf16 values; sink: device float [n_wgs * 512], written.  Returns 0, -1 (bad
// arguments) or -4 (HIP error).  flops_per_wg_block receives 8 * 48 * 32768.
extern "C" int mpic_probe_mfma(int flags, int n_wgs, int n_blocks, const void* seed, float* sink, void* stream,
                               double* flops_per_wg_block) {
  using namespace mpic;
  if (n_wgs < 1 || n_blocks < 1 || !seed || !sink) return -1;
  if (flops_per_wg_block) *flops_per_wg_block = 8.0 * 48.0 * 32768.0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = hipErrorInvalidValue;
  switch (flags) {
    case 0: e = launch<0>(n_wgs, n_blocks, seed, sink, st); break;
    case PROBE_PINGPONG: e = launch<PROBE_PINGPONG>(n_wgs, n_blocks, seed, sink, st); break;
    case PROBE_PINGPONG | PROBE_SOFTMAX: e = launch<PROBE_PINGPONG | PROBE_SOFTMAX>(n_wgs, n_blocks, seed, sink, st); break;
    default: return -1;
  }
  return e == hipSuccess ? 0 : -4;
}

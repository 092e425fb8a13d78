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
//   PROBE_LDS       (with both of the above) the "key" and "value" fragments are read from LDS the way the
//                   kernel reads them: 24 ds_read_b128 and 48 transpose reads per wavefront and block
//   PROBE_ONE_WAVE  (alone or with PROBE_LDS) the same work divided the other way, see probe_one_wave_kernel
// The global->LDS loads are not imitated here: their cost is read off timing-only variants of the kernel
// itself (kAblate* in common.h).
// Flops counted: 48 x 32 x 32 x 16 x 2 per wavefront and block.  The output is a checksum that
// keeps the compiler from dropping the work.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "wave_ops.h"

namespace mpic {
namespace {

enum { PROBE_PINGPONG = 1, PROBE_SOFTMAX = 2, PROBE_ONE_WAVE = 4, PROBE_LDS = 8 };

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
  // PROBE_LDS: the "key" and "value" fragments come out of LDS, read the way the kernel reads them (one 96-key
  // block of K and one of V, 24 KB each, filled once from the seed; K fragments with ds_read_b128, V^T fragments
  // with two transpose reads each; the kernel's swizzles, so no bank conflicts)
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int col = lane & 31, hi = lane >> 5, i16 = lane & 15;
  const int k_row_off = col * 256, k_col_x = hi ^ (col & 15);
  const int v_row = hi * 4 + (i16 >> 2);
  const int v_col_x = ((((lane >> 4) & 1) << 1) | ((i16 & 3) >> 1)) ^ ((v_row & 3) << 2);
  const int v_off = 24 * 1024 + v_row * 256 + (i16 & 1) * 8;
  if constexpr ((kFlags & PROBE_LDS) != 0) {
    for (int i = tid; i < 48 * 1024 / 16; i += THREADS)
      *reinterpret_cast<bf16x8*>(lds + i * 16) = *reinterpret_cast<const bf16x8*>(seed + (i & 1023) * 8);
    __syncthreads();
  }
  auto k_frag = [&](int kb, int ks) {
    if constexpr ((kFlags & PROBE_LDS) == 0) return kreg[(ks + kb) & 3];
    return *reinterpret_cast<const bf16x8*>(lds + k_row_off + kb * 32 * 256 + ((k_col_x ^ (ks << 1)) << 4));
  };
  auto v_frag = [&](int kh, int db) {
    if constexpr ((kFlags & PROBE_LDS) == 0) return vreg[db];
    const char* vp = lds + v_off + kh * 16 * 256 + ((v_col_x ^ (db << 2)) << 4);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MPIC_LDS_PTR(s16x4, vp));
    const s16x4 up = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MPIC_LDS_PTR(s16x4, vp + 8 * 256));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, up, 0, 1, 2, 3, 4, 5, 6, 7));
  };
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

  auto pv_block = [&]() {  // 24 matrix instructions, four independent accumulators; fragments one step ahead
    bf16x8 vf[4];
#pragma unroll
    for (int db = 0; db < 4; ++db) vf[db] = v_frag(0, db);
    if constexpr ((kFlags & PROBE_LDS) != 0) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kh = 0; kh < 2 * KB; ++kh)
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db], pf[kh], acc_o[db], 0, 0, 0);
        if (kh + 1 < 2 * KB) vf[db] = v_frag(kh + 1, db);
        if constexpr ((kFlags & PROBE_LDS) != 0) __builtin_amdgcn_sched_barrier(0);
      }
  };
  auto qk_block = [&]() {  // 24 matrix instructions, three independent accumulators; fragments two steps ahead
    constexpr int kPre = 2;
    bf16x8 kf[KB][8];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) acc_s[kb] = f32x16{0};
#pragma unroll
    for (int ks = 0; ks < kPre; ++ks)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) kf[kb][ks] = k_frag(kb, ks);
    if constexpr ((kFlags & PROBE_LDS) != 0) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if (ks + kPre < 8) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb][ks + kPre] = k_frag(kb, ks + kPre);
      }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf[ks], acc_s[kb], 0, 0, 0);
      if constexpr ((kFlags & PROBE_LDS) != 0) __builtin_amdgcn_sched_barrier(0);
    }
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

// PROBE_ONE_WAVE: another division of the same work -- one wavefront per SIMD that owns 64 query columns (two
// column groups, so every "key" / "value" fragment feeds two matrix instructions), 96 matrix instructions per
// wavefront and block, and no second wavefront to hide the softmax behind: the products of the neighbouring
// blocks (O += V^T P^T of block t-1, S = K Q^T of block t+1 into a second S buffer) are interleaved with the
// softmax of block t inside one instruction stream (one matrix instruction, then six vector instructions).
// 412 registers, of which 224 are accumulation registers (the output and the second S buffer).
template <bool kLds>
__global__ __launch_bounds__(256) void probe_one_wave_kernel(int n_blocks, const __bf16* seed, float* sink) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int lane = threadIdx.x & 63;
  const int col = lane & 31, hi = lane >> 5, i16 = lane & 15;
  const int k_row_off = col * 256, k_col_x = hi ^ (col & 15);
  const int v_row = hi * 4 + (i16 >> 2);
  const int v_col_x = ((((lane >> 4) & 1) << 1) | ((i16 & 3) >> 1)) ^ ((v_row & 3) << 2);
  const int v_off = 24 * 1024 + v_row * 256 + (i16 & 1) * 8;
  if constexpr (kLds) {
    for (int i = threadIdx.x; i < 48 * 1024 / 16; i += 256)
      *reinterpret_cast<bf16x8*>(lds + i * 16) = *reinterpret_cast<const bf16x8*>(seed + (i & 1023) * 8);
    __syncthreads();
  }
  bf16x8 qf[2][8], kreg[4], vreg[4];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int i = 0; i < 8; ++i) qf[c][i] = *reinterpret_cast<const bf16x8*>(seed + ((lane * 16 + i + c) & 1023) * 8);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    kreg[i] = *reinterpret_cast<const bf16x8*>(seed + (lane * 16 + 8 + i) * 8);
    vreg[i] = *reinterpret_cast<const bf16x8*>(seed + (lane * 16 + 12 + i) * 8);
  }
  f32x16 acc_o[2][4], s_cur[2][KB], s_nxt[2][KB];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc_o[c][i] = f32x16{0};
#pragma unroll
    for (int i = 0; i < KB; ++i) {
      s_cur[c][i] = f32x16{0};
      s_nxt[c][i] = f32x16{0};
    }
  }
  bf16x8 pf[2][2 * KB];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int i = 0; i < 2 * KB; ++i) pf[c][i] = qf[c][i & 7];
  float l_run[2] = {0.f, 0.f};
  const float m_scaled = 3.0f;
  for (int t = 0; t < n_blocks; ++t) {
#pragma unroll
    for (int kh = 0; kh < 2 * KB; ++kh)
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        bf16x8 vf = vreg[db];
        if constexpr (kLds) {
          const char* vp = lds + v_off + kh * 16 * 256 + ((v_col_x ^ (db << 2)) << 4);
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MPIC_LDS_PTR(s16x4, vp));
          const s16x4 up = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MPIC_LDS_PTR(s16x4, vp + 8 * 256));
          vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, up, 0, 1, 2, 3, 4, 5, 6, 7));
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) acc_o[c][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[c][kh], acc_o[c][db], 0, 0, 0);
      }
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) s_nxt[c][kb] = f32x16{0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        bf16x8 kf = kreg[(ks + kb) & 3];
        if constexpr (kLds) kf = *reinterpret_cast<const bf16x8*>(lds + k_row_off + kb * 32 * 256 + ((k_col_x ^ (ks << 1)) << 4));
#pragma unroll
        for (int c = 0; c < 2; ++c) s_nxt[c][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c][ks], s_nxt[c][kb], 0, 0, 0);
      }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      float l_blk = 0.f;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          f32x8 p;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            p[e] = __builtin_amdgcn_exp2f(fmaf(s_cur[c][kb][half * 8 + e], 1.0e-3f, -m_scaled));
            l_blk += p[e];
          }
          pf[c][kb * 2 + half] = __builtin_convertvector(p, bf16x8);
        }
      l_run[c] += l_blk;
    }
    if constexpr (kLds) {
#pragma unroll
      for (int i = 0; i < 24; ++i) {  // per four matrix instructions: three LDS reads, 22 vector instructions
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 96; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one matrix instruction
        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);  // six vector instructions
      }
    }
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) s_cur[c][kb] = s_nxt[c][kb];
  }
  float s = l_run[0] + l_run[1];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) s += acc_o[c][i][v];
#pragma unroll
    for (int i = 0; i < KB; ++i) s += s_cur[c][i][i];
  }
  sink[static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x] = s;
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

// One launch of the probe.  flags: 0, PROBE_PINGPONG (1), 1 | PROBE_SOFTMAX (2), 1 | 2 | PROBE_LDS (8),
// PROBE_ONE_WAVE (4), 4 | 8.  n_wgs workgroups of 512 threads (PROBE_ONE_WAVE: 256) run n_blocks blocks each.  seed: device buffer of
// 64 * 16 * 8 bf16 values; sink: device float [n_wgs * 512], written.  Returns 0, -1 (bad
// arguments) or -4 (HIP error).  flops_per_wg_block receives 8 * 48 * 32768 (PROBE_ONE_WAVE: 4 * 96 * 32768).
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
    case PROBE_PINGPONG | PROBE_SOFTMAX | PROBE_LDS:
      e = launch<PROBE_PINGPONG | PROBE_SOFTMAX | PROBE_LDS>(n_wgs, n_blocks, seed, sink, st);
      break;
    case PROBE_ONE_WAVE:
    case PROBE_ONE_WAVE | PROBE_LDS: {
      const bool with_lds = (flags & PROBE_LDS) != 0;
      static LdsOptIn opt_in;
      int dev = 0;
      e = hipGetDevice(&dev);
      if (e != hipSuccess) break;
      e = opt_in.ensure(dev, [] {
        const hipError_t e0 = hipFuncSetAttribute(reinterpret_cast<const void*>(probe_one_wave_kernel<false>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e0 != hipSuccess) return e0;
        return hipFuncSetAttribute(reinterpret_cast<const void*>(probe_one_wave_kernel<true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
      });
      if (e != hipSuccess) break;
      if (flops_per_wg_block) *flops_per_wg_block = 4.0 * 96.0 * 32768.0;
      if (with_lds)
        hipLaunchKernelGGL(probe_one_wave_kernel<true>, dim3(n_wgs), dim3(256), LDS_BYTES, st, n_blocks,
                           static_cast<const __bf16*>(seed), sink);
      else
        hipLaunchKernelGGL(probe_one_wave_kernel<false>, dim3(n_wgs), dim3(256), LDS_BYTES, st, n_blocks,
                           static_cast<const __bf16*>(seed), sink);
      e = hipGetLastError();
      break;
    }
    default: return -1;
  }
  return e == hipSuccess ? 0 : -4;
}

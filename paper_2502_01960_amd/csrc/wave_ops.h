// Device helpers shared by the matrix-core kernels of libmpic (prefill and decode
// attention): vector types of the MFMA operands, direct global->LDS loads with a
// hand-managed load counter, and the exchange between the two halves of a wavefront.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

namespace mpic {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));  // table entries, dword aligned
typedef uint32_t u32x8_a4 __attribute__((ext_vector_type(8), aligned(4)));

#define MPIC_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt fields left at "no wait").  The builtin rather
// than inline assembly: the compiler's own wait insertion sees it and adds nothing on top.
#define MPIC_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

// Direct global->LDS load of 16 bytes per lane: LDS[lds_addr + 16*lane] = *gptr.  Written as
// inline assembly so that the outstanding-load counter is managed by hand: the compiler
// would otherwise wait for *all* direct loads before any LDS read, which defeats a ring that
// keeps blocks in flight.  `nt` variant: non-temporal hint for rows that are read once.
__device__ inline void load_to_lds_16B(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_addr) : "memory", "m0");
}
__device__ inline void load_to_lds_16B_nt(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" : : "v"(gptr), "s"(lds_addr) : "memory", "m0");
}
// Combine a value with the one held by lane ^ 32 (the other half of a query column) with
// v_permlane32_swap (verified: swapping two copies of a register leaves the low half's values
// in one result and the high half's in the other, in both halves).  A plain cross-lane shuffle
// would go through the LDS pipeline, whose command queue the fragment reads keep full.
// (The two results are copied into scalars before they are reinterpreted: a bit cast applied
// directly to an element of the returned vector reads element 0 for both.)
struct Halves {
  float lo, hi;
};
__device__ inline Halves split_halves(float x) {
  const unsigned a = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
  const unsigned r0 = r[0], r1 = r[1];
  return Halves{__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1)};
}
__device__ inline float max_across_halves(float x) {
  const Halves h = split_halves(x);
  return fmaxf(h.lo, h.hi);
}
__device__ inline float sum_across_halves(float x) {
  const Halves h = split_halves(x);
  return h.lo + h.hi;
}

// Wave-wide minimum / maximum of an integer (positions are reduced as integers: a float
// holds them exactly only below 2^24).
__device__ inline int wave_min_i32(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = min(x, __shfl_xor(x, off));
  return x;
}
__device__ inline int wave_max_i32(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = max(x, __shfl_xor(x, off));
  return x;
}

// The rows a wavefront stages per block, as two runs of direct loads -- K rows to LDS address lk,
// lk + 1024, (lk + 2048), V rows likewise from lv -- with one M0 per run: the instruction offset of a
// direct load moves the global *and* the LDS address, so the caller passes the global address of
// run element i reduced by i * 1024 (verified: same bytes in LDS as with an M0 per load, and
// 0.3 % faster in the attention kernel: four or two scalar moves and wait states fewer per block).
__device__ inline void load3x2_to_lds_16B(const char* k0, const char* k1, const char* k2, const char* v0, const char* v1,
                                          const char* v2, uint32_t lk, uint32_t lv) {
  asm volatile(
      "s_mov_b32 m0, %6\n\ts_nop 0\n\t"
      "global_load_lds_dwordx4 %0, off\n\t"
      "global_load_lds_dwordx4 %1, off offset:1024\n\t"
      "global_load_lds_dwordx4 %2, off offset:2048\n\t"
      "s_mov_b32 m0, %7\n\ts_nop 0\n\t"
      "global_load_lds_dwordx4 %3, off\n\t"
      "global_load_lds_dwordx4 %4, off offset:1024\n\t"
      "global_load_lds_dwordx4 %5, off offset:2048"
      :
      : "v"(k0), "v"(k1 - 1024), "v"(k2 - 2048), "v"(v0), "v"(v1 - 1024), "v"(v2 - 2048), "s"(lk), "s"(lv)
      : "memory", "m0");
}
__device__ inline void load2x2_to_lds_16B(const char* k0, const char* k1, const char* v0, const char* v1, uint32_t lk,
                                          uint32_t lv) {
  asm volatile(
      "s_mov_b32 m0, %4\n\ts_nop 0\n\t"
      "global_load_lds_dwordx4 %0, off\n\t"
      "global_load_lds_dwordx4 %1, off offset:1024\n\t"
      "s_mov_b32 m0, %5\n\ts_nop 0\n\t"
      "global_load_lds_dwordx4 %2, off\n\t"
      "global_load_lds_dwordx4 %3, off offset:1024"
      :
      : "v"(k0), "v"(k1 - 1024), "v"(v0), "v"(v1 - 1024), "s"(lk), "s"(lv)
      : "memory", "m0");
}

// More than 64 KB of dynamic LDS needs an explicit opt-in per kernel, once per device.
// `flags` is the kernel's own per-device record; the mutex makes the first launches of
// several host threads (each with its own context) safe.
struct LdsOptIn {
  std::mutex mu;
  bool done[64] = {};
  template <typename Fn>
  hipError_t ensure(int dev, Fn&& set_attributes) {
    if (dev < 0 || dev >= 64) return set_attributes();
    std::lock_guard<std::mutex> lock(mu);
    if (done[dev]) return hipSuccess;
    const hipError_t e = set_attributes();
    if (e == hipSuccess) done[dev] = true;
    return e;
  }
};

}  // namespace mpic
